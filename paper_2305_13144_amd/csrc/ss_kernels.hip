// gfx950 kernels of the decode path.  One wavefront = 64 lanes; matrix work uses
// v_mfma_f32_16x16x32_f16 (A: 16 rows x 32 k, B: 32 k x 16 cols, 8 halves per lane;
// D: lane holds rows 4*(lane/16)..+3 of column lane%16).
//
// Convention for every contraction here: the weight strip is the A operand (its 16 output
// columns become D's rows) and the activation strip is the B operand (its 16 token rows become
// D's columns), so a lane ends up with 4 consecutive output columns of one token row.
#include "ss_kernels.h"

#include <hip/hip_runtime.h>

#include <algorithm>

#include "ss_internal.h"

namespace ss {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));  // one 16-byte operand fragment

// ------------------------------------------------------------------------------------------ helpers
__device__ __forceinline__ float bf2f(bf16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

__device__ __forceinline__ bf16_t f2bf(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);  // round to nearest, ties to even (inputs are finite)
    return (bf16_t)(u >> 16);
}

// Both operands of every projection are IEEE half.  A bf16 weight keeps its exact value in that format (8
// significand bits fit in 11; see k_pack_weight for the two ends of the range).  An activation that feeds a
// projection is rounded to half once: 11 significand bits, where a bf16 operand would keep 8 - one such rounding
// per projection input, six per layer over 32+ layers, is the dominant term of the logit error, and at 8 bits it
// is as large as the whole tolerance.  Finite values saturate, like the key/value slots below; a NaN stays a NaN.
__device__ __forceinline__ f16_t f2h(float f)
{
    const float c = fminf(fmaxf(f, -65504.f), 65504.f);   // of a NaN and a number these return the number
    return __builtin_bit_cast(f16_t, (_Float16)(f != f ? f : c));
}

// Key/value slots are stored as IEEE half: the same 2 bytes per element as bf16 with three more
// significand bits; keys and values are projections of RMS-normalised activations, far inside its range.
__device__ __forceinline__ float kv2f(kv_t b) { return (float)__builtin_bit_cast(_Float16, b); }
// Saturating: a value beyond the half range is stored as the largest finite half, never as infinity (an infinite
// key would turn the softmax into NaN and the token choice into an arbitrary id).
__device__ __forceinline__ kv_t f2kv(float f)
{
    return __builtin_bit_cast(kv_t, (_Float16)fminf(fmaxf(f, -65504.f), 65504.f));
}

// Element (r, k) of a packed [rows, Kp] matrix.
__device__ __forceinline__ size_t pk_index(int r, int k, int Kp)
{
    return ((size_t)(r >> 4) * (size_t)(Kp >> 5) + (size_t)(k >> 5)) * 512u +
           (size_t)(((((k & 31) >> 3) << 4) + (r & 15)) * 8 + (k & 7));
}

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
    return v;
}

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v = fmaxf(v, __shfl_xor(v, m, 64));
    return v;
}

// ------------------------------------------------------------------------------------------ weight packing
// src is row-major [n_src, k] (bf16 bits or fp32, rounded to bf16 first); source row r lands in packed row
// (r/16 * blk_stride + blk_off) * 16 + r%16.  One thread moves 8 consecutive k.  The packed element is the bf16
// value written as IEEE half: the same number for 2^-17 <= |w| <= 65504 (half subnormals included); smaller
// magnitudes are rounded to a multiple of 2^-24 (an absolute error below 3e-8 per weight), larger ones saturate.
__global__ void k_pack_weight(const void* __restrict__ src, int src_f32, f16_t* __restrict__ dst, int n_src, int k,
                              int kp, int blk_stride, int blk_off)
{
    const int groups = k >> 3;
    const size_t total = (size_t)n_src * groups;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        const int r = (int)(i / groups), kg = (int)(i % groups);
        bf16_t v[8];
        if (src_f32) {
            const float* sp = (const float*)src + (size_t)r * k + kg * 8;
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = f2bf(sp[e]);
        } else {
            const uint4 raw = *(const uint4*)((const bf16_t*)src + (size_t)r * k + kg * 8);
            *(uint4*)v = raw;
        }
        f16_t o[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = f2h(bf2f(v[e]));
        const int rd = ((r >> 4) * blk_stride + blk_off) * 16 + (r & 15);
        *(uint4*)(dst + pk_index(rd, kg * 8, kp)) = *(const uint4*)o;
    }
}

__global__ void k_cast_rows(const void* __restrict__ src, int src_f32, bf16_t* __restrict__ dst, size_t count)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += (size_t)gridDim.x * blockDim.x)
        dst[i] = src_f32 ? f2bf(((const float*)src)[i]) : ((const bf16_t*)src)[i];
}

__global__ void k_fill_i32(int32_t* p, int32_t v, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = v;
}

// ------------------------------------------------------------------------------------------ embedding
__global__ __launch_bounds__(256) void k_embed(MbState st, const bf16_t* __restrict__ embed, float* __restrict__ x,
                                               int d)
{
    const int j = blockIdx.x;
    if (j >= *st.d_n) return;
    const bf16_t* e = embed + (size_t)st.tr_tok[j] * d;
    float* xr = x + (size_t)j * d;
    for (int c = threadIdx.x * 8; c < d; c += 256 * 8) {
        const uint4 raw = *(const uint4*)(e + c);
        const bf16_t* v = (const bf16_t*)&raw;
        float4 a = make_float4(bf2f(v[0]), bf2f(v[1]), bf2f(v[2]), bf2f(v[3]));
        float4 b = make_float4(bf2f(v[4]), bf2f(v[5]), bf2f(v[6]), bf2f(v[7]));
        *(float4*)(xr + c) = a;
        *(float4*)(xr + c + 4) = b;
    }
}

// ------------------------------------------------------------------------------------------ RMSNorm
// Row j (or sel[j]) of the residual stream: x += sum over k-slices of the previous projection's
// partial sums (written back when sel is null), then h = x * rsqrt(mean x^2 + eps) * w as packed halves.
// T threads per row, at most ITER float4 chunks per thread (T * ITER * 4 >= d, d <= 8192); the loads of all k-slices of a
// chunk are issued together (the slice loop is unrolled with a predicate), so a row costs about one
// memory round trip instead of one per slice.
constexpr int kNormMaxSplit = 8;
constexpr int kNormNarrowFrom = 384;   // token-rows from which a row gets 256 threads instead of 1024

template <int T, int ITER>
__global__ __launch_bounds__(T) void k_rmsnorm(const int32_t* __restrict__ d_count, float* __restrict__ x,
                                                  const float* __restrict__ part, int ksplit, size_t part_stride,
                                                  const bf16_t* __restrict__ w, float eps,
                                                  const int32_t* __restrict__ sel, f16_t* __restrict__ h, int d)
{
    const int j = blockIdx.x;
    // The row count, the row, its partial sums and the norm weights are all requested before anything waits:
    // the kernel is a chain of dependent round trips otherwise (count, then the row, then the weights), and its
    // whole cost is latency.  Rows at or beyond the count are loaded as well (the buffers are sized for the grid)
    // and dropped before the first store; with a selection list the index itself is only valid below the count.
    const int count = *d_count;
    int src = j;
    if (sel) {
        if (j >= count) return;
        src = sel[j];
    }
    float4 v[ITER];
    uint2 wr[ITER];
    float ss = 0.f;
#pragma unroll
    for (int it = 0; it < ITER; ++it) {
        const int c = threadIdx.x * 4 + it * T * 4;
        if (c < d) {
            float4 a = *(const float4*)(x + (size_t)src * d + c);
            float4 p[kNormMaxSplit];
#pragma unroll
            for (int s = 0; s < kNormMaxSplit; ++s)
                p[s] = s < ksplit ? *(const float4*)(part + (size_t)s * part_stride + (size_t)src * d + c)
                                  : make_float4(0.f, 0.f, 0.f, 0.f);
            wr[it] = *(const uint2*)(w + c);
#pragma unroll
            for (int s = 0; s < kNormMaxSplit; ++s) { a.x += p[s].x; a.y += p[s].y; a.z += p[s].z; a.w += p[s].w; }
            v[it] = a;
            ss += a.x * a.x + a.y * a.y + a.z * a.z + a.w * a.w;
        }
    }
    if (j >= count) return;   // block-uniform
    if (ksplit > 0 && !sel) {
#pragma unroll
        for (int it = 0; it < ITER; ++it) {
            const int c = threadIdx.x * 4 + it * T * 4;
            if (c < d) *(float4*)(x + (size_t)src * d + c) = v[it];
        }
    }
    __shared__ float red[T / 64];
    ss = wave_sum(ss);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
    __syncthreads();
    float tot = 0.f;
#pragma unroll
    for (int i = 0; i < T / 64; ++i) tot += red[i];
    const float r = rsqrtf(tot / (float)d + eps);
#pragma unroll
    for (int it = 0; it < ITER; ++it) {
        const int c = threadIdx.x * 4 + it * T * 4;
        if (c < d) {
            const bf16_t* wv = (const bf16_t*)&wr[it];
            const f16_t o[4] = {f2h(v[it].x * r * bf2f(wv[0])), f2h(v[it].y * r * bf2f(wv[1])),
                                f2h(v[it].z * r * bf2f(wv[2])), f2h(v[it].w * r * bf2f(wv[3]))};
            const size_t at = pk_index(j, c, d);   // d is a multiple of 64: Kp == d
            *(uint2*)(h + at) = *(const uint2*)o;
        }
    }
}

// ------------------------------------------------------------------------------------------ skinny GEMM
// Up to 64 token rows (MT strips of 16); the whole cost is streaming the weights once from HBM.
// A workgroup of 4 wavefronts owns NB strips of 16 output columns and one outer k-slice; its waves cut
// that slice into 4 contiguous k-ranges, so every wave streams NB contiguous runs of 1 KiB operand
// blocks (non-temporal: each weight byte is used exactly once per step) and never waits for another
// wave until the end.  Loads are double-buffered in registers: while the MFMAs of KD k-blocks run, the
// next KD*NB KiB are already in flight.  The activation operands (MT per k-block) come from L2.
// At the end waves 1..3 hand their accumulators to wave 0 through LDS; wave 0 runs the epilogue.
__device__ __forceinline__ float silu_f(float z) { return z / (1.f + __expf(-z)); }

template <int MT, int NB, int KD>
struct SkinnyFrags {
    u32x4 w[NB][KD];
    u32x4 x[MT][KD];
};

// Loads for k-blocks kb..kb+KD-1; k-blocks at or beyond kend are clamped re-reads whose activation
// operands are zeroed in skinny_mma, so they add 0.
template <int MT, int NB, int KD>
__device__ __forceinline__ void skinny_load(SkinnyFrags<MT, NB, KD>& f, const u32x4* __restrict__ Wl,
                                            const u32x4* __restrict__ Xl, int KB, int nb0, int nvalid, int kb,
                                            int kend)
{
#pragma unroll
    for (int q = 0; q < KD; ++q) {
        const int kk = min(kb + q, kend - 1);
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const int nb = nb0 + (i < nvalid ? i : 0);
            f.w[i][q] = __builtin_nontemporal_load(Wl + ((size_t)nb * KB + kk) * 64);
        }
#pragma unroll
        for (int m = 0; m < MT; ++m) f.x[m][q] = Xl[((size_t)m * KB + kk) * 64];
    }
}

template <int MT, int NB, int KD>
__device__ __forceinline__ void skinny_mma(const SkinnyFrags<MT, NB, KD>& f, f32x4 (&acc)[NB][MT], int kb, int kend)
{
    const u32x4 zero = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int q = 0; q < KD; ++q) {
        const bool live = kb + q < kend;
#pragma unroll
        for (int m = 0; m < MT; ++m) {
            const u32x4 xv = live ? f.x[m][q] : zero;
#pragma unroll
            for (int i = 0; i < NB; ++i)
                acc[i][m] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, f.w[i][q]),
                                                                   __builtin_bit_cast(f16x8, xv), acc[i][m], 0, 0, 0);
        }
    }
}

template <int MT, int NB, int KD, int EPI>
__global__ __launch_bounds__(256) void k_gemm_skinny(GemmArgs a, int n_groups, int kb_per_slice)
{
    __shared__ f32x4 red[3][NB][MT][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int ng = blockIdx.x % n_groups, ks = blockIdx.x / n_groups;
    const int KB = a.Kp >> 5, NBT = a.N >> 4;
    const int s0 = ks * kb_per_slice, s1 = min(KB, s0 + kb_per_slice);
    const int per_wave = (max(s1 - s0, 0) + 3) >> 2;
    const int kbeg = min(s1, s0 + wave * per_wave), kend = min(s1, kbeg + per_wave);
    const int nb0 = ng * NB;
    const int nvalid = min(NB, NBT - nb0);  // block-uniform

    f32x4 acc[NB][MT];
#pragma unroll
    for (int i = 0; i < NB; ++i)
#pragma unroll
        for (int m = 0; m < MT; ++m) acc[i][m] = (f32x4){0.f, 0.f, 0.f, 0.f};

    const u32x4* Wl = (const u32x4*)a.W + lane;
    const u32x4* Xl = (const u32x4*)a.X + lane;
    if (kbeg < kend) {
        SkinnyFrags<MT, NB, KD> fa, fb;
        skinny_load(fa, Wl, Xl, KB, nb0, nvalid, kbeg, kend);
        // Loads past the wave's k-range are skipped rather than clamped: measured, the wasted re-reads of an
        // unconditional tail cost more (k-ranges are only 4-40 blocks) than the conservative load-counter waits
        // the branches cause; latency is hidden by the 12-20 resident waves per CU, not inside a wave.
        for (int kb = kbeg; kb < kend; kb += 2 * KD) {
            if (kb + KD < kend) skinny_load(fb, Wl, Xl, KB, nb0, nvalid, kb + KD, kend);
            skinny_mma(fa, acc, kb, kend);
            if (kb + 2 * KD < kend) skinny_load(fa, Wl, Xl, KB, nb0, nvalid, kb + 2 * KD, kend);
            if (kb + KD < kend) skinny_mma(fb, acc, kb + KD, kend);
        }
    }
    if (wave > 0) {
#pragma unroll
        for (int i = 0; i < NB; ++i)
#pragma unroll
            for (int m = 0; m < MT; ++m) red[wave - 1][i][m][lane] = acc[i][m];
    }
    __syncthreads();
    if (wave > 0) return;
#pragma unroll
    for (int w = 0; w < 3; ++w)
#pragma unroll
        for (int i = 0; i < NB; ++i)
#pragma unroll
            for (int m = 0; m < MT; ++m) acc[i][m] += red[w][i][m][lane];

    const int col4 = (lane >> 4) * 4;  // first of this lane's 4 consecutive output columns inside a strip
#pragma unroll
    for (int m = 0; m < MT; ++m) {
        const int row = m * 16 + (lane & 15);
        if (row >= a.m_rows) continue;
        if (EPI == EPI_PARTIAL) {
            float* o = a.out + ((size_t)ks * a.m_stride + row) * a.N;
#pragma unroll
            for (int i = 0; i < NB; ++i)
                if (i < nvalid)
                    *(float4*)(o + (nb0 + i) * 16 + col4) =
                        make_float4(acc[i][m][0], acc[i][m][1], acc[i][m][2], acc[i][m][3]);
        } else {
            // strips alternate gate, up for the same 16 MLP columns
#pragma unroll
            for (int i = 0; i + 1 < NB; i += 2)
                if (i + 1 < nvalid) {
                    const int f = ((nb0 + i) >> 1) * 16 + col4;
                    f16_t o[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) o[e] = f2h(silu_f(acc[i][m][e]) * acc[i + 1][m][e]);
                    const size_t at = pk_index(row, f, a.kp_out);
                    *(uint2*)(a.out_packed + at) = *(const uint2*)o;
                }
        }
    }
}

// ------------------------------------------------------------------------------------------ sweep GEMM
// Up to 256 token rows (16 row strips), for projections large enough to give every compute unit one workgroup
// with several waves of work.  What bounds a weight stream on this chip is the number of bytes a compute unit can have in
// flight towards L2/HBM, and every byte requested through the vector memory path counts, also an activation
// operand that hits in L2: in the kernel above, where each wave fetches its own activation operands, those
// take a quarter of that budget (2 strips) or an eighth (4 strips).  Here the waves of a workgroup own
// different output strips and sweep the same k-range together, so an activation chunk (KC k-blocks,
// all row strips) is fetched once per workgroup, staged in LDS (double-buffered, one barrier per chunk) and
// read from there by every wave; one workgroup per compute unit means once per unit.  No wave shares an
// output with another: no reduction at the end, and the SwiGLU epilogue stays inside the wave that owns a
// gate strip and its up strip.  Weight loads run two chunks ahead in two named register slots; nothing in
// the loop is conditional, so the load counter waits are exact.  K-blocks beyond the k-slice and strips
// beyond the matrix read a block of zeros instead of weights (an L2 hit) and add 0.
// With KH = 2 two waves share a unit: wave 2u takes the first half of every chunk's k-blocks, wave 2u + 1 the second
// (each loads only its own weight blocks and reads only its own operands from LDS); the odd wave hands its
// accumulators to the even one through LDS at the end.  Used above 96 rows when a workgroup owns at most 4 units:
// there the matrix-core and LDS work per weight byte grows with the row strips, and 3 or 4 waves (one per SIMD,
// nothing to overlap their waits with) no longer keep up with the weight stream.
template <int NBW, int KQ>
struct SweepSlot {
    u32x4 w[NBW][KQ];   // KQ = k-blocks of a chunk this wave handles
};

template <int NBW, int KQ>
__device__ __forceinline__ void sweep_load_w(SweepSlot<NBW, KQ>& f, const u32x4* __restrict__ Wl,
                                             const u32x4* __restrict__ Zl, int KB, int nb0, int nvalid, int kb, int kend)
{
#pragma unroll
    for (int q = 0; q < KQ; ++q) {
        const bool live = kb + q < kend;
        const int kk = min(kb + q, kend - 1);
#pragma unroll
        for (int i = 0; i < NBW; ++i) {
            // weights or the zero block: selected by address arithmetic (a select between two pointers can be
            // compiled into a branch around the load)
            const uintptr_t wp = (uintptr_t)(Wl + ((size_t)(nb0 + i) * KB + kk) * 64), zp = (uintptr_t)Zl;
            const uintptr_t mask = (live && i < nvalid) ? ~(uintptr_t)0 : (uintptr_t)0;
            f.w[i][q] = __builtin_nontemporal_load((const u32x4*)(zp ^ ((wp ^ zp) & mask)));
        }
    }
}

// An activation chunk is KC*MT operand blocks of 64 x 16 bytes, block m*KC + q = row strip m, k-block q of
// the chunk.  Thread t of the workgroup moves pieces t, t + 64P, ...;
// indices past the end are clamped to the last piece (the same bytes written twice).
template <int P, int MT, int KC>
struct SweepStage {
    static constexpr int PIECES = KC * MT * 64;
    static constexpr int XI = (PIECES + 64 * P - 1) / (64 * P);
    u32x4 v[XI];
};

template <int P, int MT, int KC>
__device__ __forceinline__ void sweep_load_x(SweepStage<P, MT, KC>& xs, const u32x4* __restrict__ X, int KB, int kb,
                                             int kend)
{
#pragma unroll
    for (int i = 0; i < SweepStage<P, MT, KC>::XI; ++i) {
        const int piece = min((int)threadIdx.x + i * 64 * P, SweepStage<P, MT, KC>::PIECES - 1);
        const int b = piece >> 6, l = piece & 63;
        const int m = b / KC, q = b % KC;
        const int kk = min(kb + q, kend - 1);
        xs.v[i] = X[((size_t)m * KB + kk) * 64 + l];
    }
}

template <int P, int MT, int KC>
__device__ __forceinline__ void sweep_store_x(const SweepStage<P, MT, KC>& xs, u32x4* buf)
{
#pragma unroll
    for (int i = 0; i < SweepStage<P, MT, KC>::XI; ++i)
        buf[min((int)threadIdx.x + i * 64 * P, SweepStage<P, MT, KC>::PIECES - 1)] = xs.v[i];
}

// q0: first k-block of the chunk this wave handles (0, or KC/2 for the second wave of a pair).
template <int MT, int NBW, int KC, int KQ>
__device__ __forceinline__ void sweep_mma(const SweepSlot<NBW, KQ>& f, const u32x4* buf, int lane, int q0,
                                          f32x4 (&acc)[NBW][MT])
{
#pragma unroll
    for (int q = 0; q < KQ; ++q) {
        u32x4 xv[MT];
#pragma unroll
        for (int m = 0; m < MT; ++m) xv[m] = buf[(m * KC + q0 + q) * 64 + lane];
#pragma unroll
        for (int m = 0; m < MT; ++m)
#pragma unroll
            for (int i = 0; i < NBW; ++i)
                acc[i][m] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, f.w[i][q]),
                                                                   __builtin_bit_cast(f16x8, xv[m]), acc[i][m], 0, 0, 0);
    }
}

// The k sweep of one wave.  ACTIVE = false is a wave without a unit (the workgroup got fewer than P): it only
// moves its share of the activation chunks and keeps the barriers; weight loads for it, even of the zero
// block, would take their share of the compute unit's memory requests.  The two variants are separate
// straight-line loops, chosen once per wave, because a load under a branch inside the loop would make
// every wait there cover all loads in flight.
template <bool ACTIVE, int P, int MT, int NBW, int KC, int KH>
__device__ __forceinline__ void sweep_run(u32x4* xl0, u32x4* xl1, f32x4 (&acc)[NBW][MT],
                                          const u32x4* __restrict__ Wl, const u32x4* __restrict__ Zl,
                                          const u32x4* __restrict__ X, int KB, int nb0, int nvalid, int s0, int s1,
                                          int C, int lane, int q0)
{
    constexpr int KQ = KC / KH;
    SweepSlot<NBW, KQ> fa, fb;
    SweepStage<P, MT, KC> xs;
    sweep_load_x<P, MT, KC>(xs, X, KB, s0, s1);
    if (ACTIVE) sweep_load_w<NBW, KQ>(fa, Wl, Zl, KB, nb0, nvalid, s0 + q0, s1);
    __builtin_amdgcn_sched_barrier(0);
    sweep_store_x<P, MT, KC>(xs, xl0);
    __builtin_amdgcn_sched_barrier(0);
    sweep_load_x<P, MT, KC>(xs, X, KB, s0 + KC, s1);
    if (ACTIVE) sweep_load_w<NBW, KQ>(fb, Wl, Zl, KB, nb0, nvalid, s0 + KC + q0, s1);
    __builtin_amdgcn_sched_barrier(0);
    __syncthreads();
    // Two chunks per trip (slot fa with LDS buffer 0, slot fb with buffer 1).  Within a chunk: contract it,
    // write the next chunk's activations (loaded one chunk ago) into the other buffer, start the loads of
    // the chunk after that, barrier.  A buffer is rewritten one barrier after its last read.
    for (int c = 0; c < C; c += 2) {
        const int k2 = s0 + (c + 2) * KC, k3 = k2 + KC;
        if (ACTIVE) sweep_mma<MT, NBW, KC, KQ>(fa, xl0, lane, q0, acc);
        __builtin_amdgcn_sched_barrier(0);
        sweep_store_x<P, MT, KC>(xs, xl1);
        __builtin_amdgcn_sched_barrier(0);
        sweep_load_x<P, MT, KC>(xs, X, KB, k2, s1);
        if (ACTIVE) sweep_load_w<NBW, KQ>(fa, Wl, Zl, KB, nb0, nvalid, k2 + q0, s1);
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();
        if (ACTIVE) sweep_mma<MT, NBW, KC, KQ>(fb, xl1, lane, q0, acc);
        __builtin_amdgcn_sched_barrier(0);
        sweep_store_x<P, MT, KC>(xs, xl0);
        __builtin_amdgcn_sched_barrier(0);
        sweep_load_x<P, MT, KC>(xs, X, KB, k3, s1);
        if (ACTIVE) sweep_load_w<NBW, KQ>(fb, Wl, Zl, KB, nb0, nvalid, k3 + q0, s1);
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();
    }
}

// Grid: n_gn workgroups per k-slice x ksplit; workgroup gn of a slice owns units [gn*n_units/n_gn,
// (gn+1)*n_units/n_gn) (a unit = NBW consecutive strips; at most P/KH of them, checked by the launcher), one per
// wave, or with KH = 2 one per pair of waves.
template <int P, int MT, int NBW, int EPI, int KH>
__global__ __launch_bounds__(64 * P) void k_gemm_sweep(GemmArgs a, int n_units, int n_gn, int kb_per_slice)
{
    // k-blocks per chunk: 4 up to 12 row strips (both staging buffers: 8 KiB per row strip, at most 96 KiB), 2 above.
    // Measured: one strip 4 against 2 and 8, 5-8 strips 4 against 2: 4 is the fastest; 9-12 strips 4 against 2: 4 % faster;
    // 13-15 strips: equal; 16 strips: 2 is 10 % faster (128 KiB of LDS and the registers of the widest instantiation).
    constexpr int KC = MT > 12 ? 2 : 4;
    static_assert(KC % KH == 0, "a chunk's k-blocks split evenly between the waves of a unit");
    constexpr int STAGE = SweepStage<P, MT, KC>::PIECES;
    // two staging buffers; after the sweep the same memory carries the odd waves' accumulators (KH = 2)
    constexpr int RED = KH == 2 ? (P / 2) * NBW * MT * 64 : 0;
    __shared__ u32x4 xlds[2 * STAGE > RED ? 2 * STAGE : RED];
    u32x4* const xl0 = xlds;
    u32x4* const xl1 = xlds + STAGE;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int gn = blockIdx.x % n_gn, ks = blockIdx.x / n_gn;
    const int KB = a.Kp >> 5, NBT = a.N >> 4;
    const int s0 = ks * kb_per_slice, s1 = min(KB, s0 + kb_per_slice);
    const int u0 = (int)((long long)gn * n_units / n_gn), u1 = (int)((long long)(gn + 1) * n_units / n_gn);
    const int slot = wave / KH;                   // unit slot of this wave inside the workgroup
    const int q0 = (wave % KH) * (KC / KH);       // first k-block of every chunk this wave handles
    const int unit = u0 + slot;
    const int nb0 = unit * NBW;
    const int nvalid = unit < u1 ? max(min(NBW, NBT - nb0), 0) : 0;
    const bool active = nvalid > 0;   // wave-uniform

    f32x4 acc[NBW][MT];
#pragma unroll
    for (int i = 0; i < NBW; ++i)
#pragma unroll
        for (int m = 0; m < MT; ++m) acc[i][m] = (f32x4){0.f, 0.f, 0.f, 0.f};

    const u32x4* Wl = (const u32x4*)a.W + lane;
    const u32x4* Zl = (const u32x4*)a.zero_blk + lane;
    const u32x4* X = (const u32x4*)a.X;
    const int C = (s1 - s0 + KC - 1) / KC;   // chunks of this slice: the same for every wave of the workgroup
    if (C > 0) {
        if (active)
            sweep_run<true, P, MT, NBW, KC, KH>(xl0, xl1, acc, Wl, Zl, X, KB, nb0, nvalid, s0, s1, C, lane, q0);
        else
            sweep_run<false, P, MT, NBW, KC, KH>(xl0, xl1, acc, Wl, Zl, X, KB, nb0, nvalid, s0, s1, C, lane, q0);
    }
    if (KH == 2) {
        // the odd wave of a pair hands its sums to the even one (the staging buffers are free after the last barrier
        // of the sweep; with no chunk at all nobody has touched them)
        f32x4* red = (f32x4*)xlds;
        if (active && (wave & 1)) {
#pragma unroll
            for (int i = 0; i < NBW; ++i)
#pragma unroll
                for (int m = 0; m < MT; ++m) red[((slot * NBW + i) * MT + m) * 64 + lane] = acc[i][m];
        }
        __syncthreads();
        if (wave & 1) return;
        if (active) {
#pragma unroll
            for (int i = 0; i < NBW; ++i)
#pragma unroll
                for (int m = 0; m < MT; ++m) acc[i][m] += red[((slot * NBW + i) * MT + m) * 64 + lane];
        }
    }
    if (!active) return;

    const int col4 = (lane >> 4) * 4;
#pragma unroll
    for (int m = 0; m < MT; ++m) {
        const int row = m * 16 + (lane & 15);
        if (row >= a.m_rows) continue;
        if (EPI == EPI_PARTIAL) {
            float* o = a.out + ((size_t)ks * a.m_stride + row) * a.N;
#pragma unroll
            for (int i = 0; i < NBW; ++i)
                if (i < nvalid)
                    *(float4*)(o + (nb0 + i) * 16 + col4) =
                        make_float4(acc[i][m][0], acc[i][m][1], acc[i][m][2], acc[i][m][3]);
        } else {
#pragma unroll
            for (int i = 0; i + 1 < NBW; i += 2)
                if (i + 1 < nvalid) {
                    const int f = ((nb0 + i) >> 1) * 16 + col4;
                    f16_t o[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) o[e] = f2h(silu_f(acc[i][m][e]) * acc[i + 1][m][e]);
                    const size_t at = pk_index(row, f, a.kp_out);
                    *(uint2*)(a.out_packed + at) = *(const uint2*)o;
                }
        }
    }
}

// ------------------------------------------------------------------------------------------ tiled GEMM
// More than 64 token rows where the sweep kernel does not apply: prompt forwards (more than 256 token-rows) and
// matrices too small for it.  A workgroup computes
// TMS*16 token rows x 256 output columns; wave w owns 4 strips of 16 columns and every row strip.
// Weights never touch LDS: they are stored in operand order, so each wave loads its own 4 operand
// blocks per k-block straight into registers (1 KiB coalesced each) and is the only wave of the
// workgroup that needs them.  The activation tile is shared by the 4 waves and staged
// through LDS in operand order (conflict-free 1 KiB reads).  One k-block per trip; both streams run
// D k-blocks ahead of the MFMAs in a register ring (6 for a 64-row tile: 150 KiB in flight per CU with two
// workgroups, enough to keep HBM busy when there are few row tiles; 2 for a 128-row
// tile, whose doubled accumulators leave no registers for more).
// Workgroup ids are mapped so that the row tiles of one column tile follow each other at a stride of 8:
// they land on the same XCD (ids are dealt round-robin over the 8 XCDs) at about the same time and share
// that column tile's weights through its L2.
// With KP = 2 the workgroup has 8 waves: two groups of 4 take the two halves of the k-slice (each with its
// own LDS stages) and the second group hands its accumulators to the first through LDS at the end.  Used
// when there are too few tiles to give every CU two workgroups: it doubles the waves per CU and halves
// the serial k loop without sending partial sums through HBM.
template <int TMS, int KP, int EPI>
__global__ __launch_bounds__(256 * KP, 2) void k_gemm_tiled(GemmArgs a, int kb_per_slice, int n_ntiles, int n_mtiles)
{
    constexpr int D = TMS > 4 ? 2 : (KP == 1 ? 6 : 4);   // k-blocks in flight
    constexpr int XV = TMS * 64 / 256;          // 16-byte vectors per thread: one k-block of the activation tile
    __shared__ u32x4 lds_all[KP][2][TMS * 64];                // [k-part][stage][row strip][lane]
    __shared__ f32x4 red[KP > 1 ? 4 * TMS : 1][KP > 1 ? 256 : 1];
    const int part = threadIdx.x >> 8, tid = threadIdx.x & 255, lane = tid & 63, wave = tid >> 6;
    u32x4 (*lds)[TMS * 64] = lds_all[part];
    const int KB = a.Kp >> 5, NBT = a.N >> 4;
    const int MBT = (a.m_rows + 15) >> 4;
    const int per_slice = ((n_ntiles + 7) >> 3) * 8 * n_mtiles;
    const int ks = blockIdx.x / per_slice, r = blockIdx.x % per_slice;
    const int chunk = r / (8 * n_mtiles), within = r % (8 * n_mtiles);
    const int n_tile = chunk * 8 + (within & 7), m_tile = within >> 3;
    if (n_tile >= n_ntiles) return;
    const int nb0 = n_tile * 16 + wave * 4, mb0 = m_tile * TMS;
    const int s0 = ks * kb_per_slice, s1 = min(KB, s0 + kb_per_slice);
    const int part_len = (max(s1 - s0, 0) + KP - 1) / KP;      // trips every wave of the workgroup runs
    const int kb0 = min(s1, s0 + part * part_len), kb1 = min(s1, kb0 + part_len);

    f32x4 acc[4][TMS];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int m = 0; m < TMS; ++m) acc[i][m] = (f32x4){0.f, 0.f, 0.f, 0.f};

    const u32x4* W4 = (const u32x4*)a.W + lane;
    const u32x4* Xh = (const u32x4*)a.X;
    // Ring slots are separately named arrays of native vectors indexed only by unrolled constants, so
    // that they stay in registers (a ring that ends up in scratch memory makes every access wait for all
    // outstanding loads).
    u32x4 w0[4], w1[4], w2[4], w3[4], w4[4], w5[4], x0[XV], x1[XV], x2[XV], x3[XV], x4[XV], x5[XV];
    static_assert(D == 6 || D == 4 || D == 2, "the ring below is written out for 6, 4 and 2 slots");
#define SS_WLOAD(W_, KB_)                                                                       \
    _Pragma("unroll") for (int i_ = 0; i_ < 4; ++i_)                                            \
        W_[i_] = W4[((size_t)min(nb0 + i_, NBT - 1) * KB + (KB_)) * 64];
#define SS_XLOAD(X_, KB_)                                                                       \
    _Pragma("unroll") for (int i_ = 0; i_ < XV; ++i_) {                                         \
        const int c_ = tid + i_ * 256;                                                          \
        const int ln_ = c_ & 63, ms_ = c_ >> 6;                                                 \
        X_[i_] = Xh[((size_t)min(mb0 + ms_, MBT - 1) * KB + (KB_)) * 64 + ln_];                 \
    }
#define SS_XSTORE(STAGE_, X_, LIVE_)                                                            \
    _Pragma("unroll") for (int i_ = 0; i_ < XV; ++i_) lds[STAGE_][tid + i_ * 256] = (LIVE_) ? X_[i_] : zero4;
#define SS_COMPUTE(W_, STAGE_)                                                                  \
    {                                                                                           \
        /* every operand read of the trip is issued before the first MFMA (the reads return in  \
           order, so each MFMA group waits only for its own operand): LDS latency overlaps MFMAs */ \
        u32x4 xh_[TMS];                                                                         \
        _Pragma("unroll") for (int m_ = 0; m_ < TMS; ++m_) xh_[m_] = lds[STAGE_][m_ * 64 + lane]; \
        __builtin_amdgcn_sched_barrier(0x16);   /* only VALU, SALU and global loads may cross */ \
        _Pragma("unroll") for (int m_ = 0; m_ < TMS; ++m_) {                                    \
            _Pragma("unroll") for (int i_ = 0; i_ < 4; ++i_) {                                  \
                acc[i_][m_] = __builtin_amdgcn_mfma_f32_16x16x32_f16(                           \
                    __builtin_bit_cast(f16x8, W_[i_]), __builtin_bit_cast(f16x8, xh_[m_]), acc[i_][m_], 0, 0, 0); \
            }                                                                                   \
        }                                                                                       \
    }
    // One trip: k-block t from ring slot (WC_, XC_); the next k-block's tile (XN_) goes into the other LDS
    // stage first; afterwards the slot is refilled D k-blocks ahead.  Nothing in a trip is conditional: the
    // compiler counts outstanding loads statically, and a load issued under a branch makes it wait for every
    // load in flight at the next use.  K-blocks at or beyond kb1 are clamped re-reads whose activation tile
    // is stored as zeros, so they add 0; every wave of the workgroup runs the same number of trips.
#define SS_TRIP(P_, WC_, XC_, XN_)                                                              \
    {                                                                                           \
        const int t_ = kb0 + it + P_;                                                           \
        SS_XSTORE((P_ + 1) & 1, XN_, t_ + 1 < kb1)                                              \
        SS_COMPUTE(WC_, P_ & 1)                                                                 \
        SS_WLOAD(WC_, min(t_ + D, last)) SS_XLOAD(XC_, min(t_ + D, last))                       \
        __syncthreads();                                                                        \
    }

    const u32x4 zero4 = {0u, 0u, 0u, 0u};
    const int last = max(min(kb1, KB) - 1, 0);   // beyond the range: a harmless in-bounds re-read
    SS_WLOAD(w0, min(kb0, last)) SS_XLOAD(x0, min(kb0, last))
    SS_WLOAD(w1, min(kb0 + 1, last)) SS_XLOAD(x1, min(kb0 + 1, last))
    if (D >= 4) {
        SS_WLOAD(w2, min(kb0 + 2, last)) SS_XLOAD(x2, min(kb0 + 2, last))
        SS_WLOAD(w3, min(kb0 + 3, last)) SS_XLOAD(x3, min(kb0 + 3, last))
    }
    if (D == 6) {
        SS_WLOAD(w4, min(kb0 + 4, last)) SS_XLOAD(x4, min(kb0 + 4, last))
        SS_WLOAD(w5, min(kb0 + 5, last)) SS_XLOAD(x5, min(kb0 + 5, last))
    }
    SS_XSTORE(0, x0, kb0 < kb1)
    __syncthreads();
    if (D == 6) {
        for (int it = 0; it < part_len; it += 6) {
            SS_TRIP(0, w0, x0, x1)
            SS_TRIP(1, w1, x1, x2)
            SS_TRIP(2, w2, x2, x3)
            SS_TRIP(3, w3, x3, x4)
            SS_TRIP(4, w4, x4, x5)
            SS_TRIP(5, w5, x5, x0)
        }
    } else if (D == 4) {
        for (int it = 0; it < part_len; it += 4) {
            SS_TRIP(0, w0, x0, x1)
            SS_TRIP(1, w1, x1, x2)
            SS_TRIP(2, w2, x2, x3)
            SS_TRIP(3, w3, x3, x0)
        }
    } else {
        for (int it = 0; it < part_len; it += 2) {
            SS_TRIP(0, w0, x0, x1)
            SS_TRIP(1, w1, x1, x0)
        }
    }
#undef SS_WLOAD
#undef SS_XLOAD
#undef SS_XSTORE
#undef SS_COMPUTE
#undef SS_TRIP

    if (KP > 1) {
        if (part == 1) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int m = 0; m < TMS; ++m) red[i * TMS + m][tid] = acc[i][m];
        }
        __syncthreads();
        if (part == 1) return;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int m = 0; m < TMS; ++m) acc[i][m] += red[i * TMS + m][tid];
    }

    const int col4 = (lane >> 4) * 4;
#pragma unroll
    for (int m = 0; m < TMS; ++m) {
        const int row = (mb0 + m) * 16 + (lane & 15);
        if (row >= a.m_rows) continue;
        if (EPI == EPI_PARTIAL) {
            float* o = a.out + ((size_t)ks * a.m_stride + row) * a.N;
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (nb0 + i < NBT)
                    *(float4*)(o + (nb0 + i) * 16 + col4) = make_float4(acc[i][m][0], acc[i][m][1], acc[i][m][2], acc[i][m][3]);
        } else {
#pragma unroll
            for (int i = 0; i < 4; i += 2)
                if (nb0 + i + 1 < NBT) {
                    const int f = ((nb0 + i) >> 1) * 16 + col4;
                    f16_t o[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) o[e] = f2h(silu_f(acc[i][m][e]) * acc[i + 1][m][e]);
                    const size_t at = pk_index(row, f, a.kp_out);
                    *(uint2*)(a.out_packed + at) = *(const uint2*)o;
                }
        }
    }
}

// SwiGLU over k-sliced partial sums: the gate|up projection was run with k-slices (its output columns are
// in strip order: strip 2j = gate columns 16j.., strip 2j+1 = the matching up columns); this adds the
// slices and writes silu(gate)*up as packed activations.  One thread per 4 MLP columns of a row.
__global__ __launch_bounds__(256) void k_swiglu_reduce(const float* __restrict__ part, int ksplit, size_t part_stride,
                                                       int m_rows, int F, int kp_out, f16_t* __restrict__ out)
{
    const int row = blockIdx.y;
    const int f = (blockIdx.x * 256 + threadIdx.x) * 4;
    if (row >= m_rows || f >= F) return;
    const size_t g_at = (size_t)row * 2 * F + (size_t)(f >> 4) * 32 + (f & 15);
    float4 g = make_float4(0.f, 0.f, 0.f, 0.f), u = g;
    for (int s = 0; s < ksplit; ++s) {
        const float4 a = *(const float4*)(part + (size_t)s * part_stride + g_at);
        const float4 b = *(const float4*)(part + (size_t)s * part_stride + g_at + 16);
        g.x += a.x; g.y += a.y; g.z += a.z; g.w += a.w;
        u.x += b.x; u.y += b.y; u.z += b.z; u.w += b.w;
    }
    const f16_t o[4] = {f2h(silu_f(g.x) * u.x), f2h(silu_f(g.y) * u.y), f2h(silu_f(g.z) * u.z), f2h(silu_f(g.w) * u.w)};
    const size_t at = pk_index(row, f, kp_out);
    *(uint2*)(out + at) = *(const uint2*)o;
}

// ------------------------------------------------------------------------------------------ RoPE + KV append
// Token-row j: sums the k-slices of its [q | k | v] projection, rotates q and k at the row's position
// (pairs e, e + hd/2; cos/sin from a table indexed [pos][e]), stores q as fp32 and k, v as IEEE half (kv_t) into the
// row's key/value slab: element (head h, slot s, e) of row i lives at so[i]*d + (h*cap[i] + s)*hd + e.
__global__ __launch_bounds__(256) void k_rope_append(MbState st, const float* __restrict__ part, int ksplit,
                                                     size_t part_stride, float* __restrict__ qrot,
                                                     kv_t* __restrict__ kc, kv_t* __restrict__ vc,
                                                     const float* __restrict__ rcos, const float* __restrict__ rsin,
                                                     int d, int H, int hd)
{
    const int j = blockIdx.x;
    if (j >= *st.d_n) return;
    const int row = st.tr_row[j], pos = st.tr_pos[j];
    const int half = hd >> 1;
    const size_t slab = (size_t)st.row_so[row] * d;
    const int cap = st.row_cap[row];
    const float* p0 = part + (size_t)j * 3 * d;
    for (int idx = threadIdx.x; idx < (d >> 1); idx += 256) {
        const int h = idx / half, e = idx - h * half;
        const int c = h * hd + e;
        float q1 = 0.f, q2 = 0.f, k1 = 0.f, k2 = 0.f, v1 = 0.f, v2 = 0.f;
        for (int s = 0; s < ksplit; ++s) {
            const float* p = p0 + (size_t)s * part_stride;
            q1 += p[c]; q2 += p[c + half];
            k1 += p[d + c]; k2 += p[d + c + half];
            v1 += p[2 * d + c]; v2 += p[2 * d + c + half];
        }
        const float cs = rcos[(size_t)pos * half + e], sn = rsin[(size_t)pos * half + e];
        qrot[(size_t)j * d + c] = q1 * cs - q2 * sn;
        qrot[(size_t)j * d + c + half] = q1 * sn + q2 * cs;
        const size_t o = slab + ((size_t)h * cap + pos) * hd + e;
        kc[o] = f2kv(k1 * cs - k2 * sn);
        kc[o + half] = f2kv(k1 * sn + k2 * cs);
        vc[o] = f2kv(v1);
        vc[o + half] = f2kv(v2);
    }
}

// ------------------------------------------------------------------------------------------ attention
// One workgroup per (token-row, head): softmax(q.K^T / sqrt(hd)) V over the row's own slots 0..pos.
// Two passes, exactly the max-subtracted definition: scores to LDS, block max and sum, then the weighted
// sum of V.  A wave's load covers 64/LPK consecutive keys (LPK = hd/8 lanes of 16 bytes per key), so K
// and V are each streamed once, fully coalesced; a wave issues AU such loads before it consumes them, so
// a context of a few hundred slots costs two or three memory round trips, not one per load.
constexpr int kAttnUnroll = 8;
constexpr int kAttnWideMaxGroups = 512;   // decode attention: (row, head) workgroups up to which 8 waves each are used

template <int HD, int NW>
__device__ __forceinline__ void attend(const float* __restrict__ qs, float* __restrict__ sc, float* __restrict__ red,
                                       float (*__restrict__ oacc)[HD], const kv_t* __restrict__ kbase,
                                       const kv_t* __restrict__ vbase, int ctx, f16_t* __restrict__ out, int out_r,
                                       int out_k0, int out_kp)
{
    constexpr int LPK = HD / 8;       // lanes per key
    constexpr int KPW = 64 / LPK;     // keys per wave load
    constexpr int AU = kAttnUnroll;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int sub = lane % LPK, kin = lane / LPK;
    const float scale = rsqrtf((float)HD);
    float q[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) q[e] = qs[sub * 8 + e];

    float mx = -3.0e38f;
    for (int c0 = wave * KPW; c0 < ctx; c0 += NW * KPW * AU) {
        uint4 raw[AU];
#pragma unroll
        for (int u = 0; u < AU; ++u) {
            const int s = c0 + u * NW * KPW + kin;
            raw[u] = s < ctx ? *(const uint4*)(kbase + (size_t)s * HD + sub * 8) : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int u = 0; u < AU; ++u) {
            const int s = c0 + u * NW * KPW + kin;
            const kv_t* kv = (const kv_t*)&raw[u];
            float part = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) part += q[e] * kv2f(kv[e]);
#pragma unroll
            for (int m = 1; m < LPK; m <<= 1) part += __shfl_xor(part, m, 64);
            part *= scale;
            if (s < ctx) {
                if (sub == 0) sc[s] = part;
                mx = fmaxf(mx, part);
            }
        }
    }
    // the first chunk of V does not depend on the scores: get it moving before the reductions
    uint4 vraw[AU];
#pragma unroll
    for (int u = 0; u < AU; ++u) {
        const int s = wave * KPW + u * NW * KPW + kin;
        vraw[u] = s < ctx ? *(const uint4*)(vbase + (size_t)s * HD + sub * 8) : make_uint4(0, 0, 0, 0);
    }
    mx = wave_max(mx);
    if (lane == 0) red[wave] = mx;
    __syncthreads();
    mx = red[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) mx = fmaxf(mx, red[w]);
    float sum = 0.f;
    for (int s = tid; s < ctx; s += 64 * NW) {
        const float p = __expf(sc[s] - mx);
        sc[s] = p;
        sum += p;
    }
    sum = wave_sum(sum);
    if (lane == 0) red[NW + wave] = sum;
    __syncthreads();
    float tot = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) tot += red[NW + w];
    const float inv = 1.f / tot;

    float o[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int c0 = wave * KPW; c0 < ctx; c0 += NW * KPW * AU) {
        uint4 raw[AU];
#pragma unroll
        for (int u = 0; u < AU; ++u) {
            const int s = c0 + u * NW * KPW + kin;
            if (c0 == wave * KPW)
                raw[u] = vraw[u];
            else
                raw[u] = s < ctx ? *(const uint4*)(vbase + (size_t)s * HD + sub * 8) : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int u = 0; u < AU; ++u) {
            const int s = c0 + u * NW * KPW + kin;
            const float p = s < ctx ? sc[s] : 0.f;
            const kv_t* vv = (const kv_t*)&raw[u];
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] += p * kv2f(vv[e]);
        }
    }
#pragma unroll
    for (int m = LPK; m < 64; m <<= 1)
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] += __shfl_xor(o[e], m, 64);
    if (kin == 0)
#pragma unroll
        for (int e = 0; e < 8; ++e) oacc[wave][sub * 8 + e] = o[e];
    __syncthreads();
    if (tid < HD / 4) {
        f16_t r[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int c = tid * 4 + e;
            float t = 0.f;
#pragma unroll
            for (int w = 0; w < NW; ++w) t += oacc[w][c];
            r[e] = f2h(t * inv);
        }
        const size_t at = pk_index(out_r, out_k0 + tid * 4, out_kp);
        *(uint2*)(out + at) = *(const uint2*)r;
    }
}

// Prompt forwards: q was rotated and K, V appended for every token-row by k_rope_append before this runs.
// Causal attention of one (row, head, tile of 64 queries) per workgroup; each of its 4 waves owns 16 queries.
// The row's keys and values are visited in tiles of 32 slots that are staged once in LDS for all 64 queries
// (K as stored, V transposed), the next tile's global loads in flight while the current one is used.
// Both contractions run on the matrix cores in half precision, the cache's own format:
//   S^T = K Q^T   A = K tile (16 keys x 32 head elements), B = Q^T; q is carried as the sum of two halves
//                 (hi + lo), so the scores see q to ~22 bits like the decode kernel's fp32 dot product;
//                 D: lane holds, for query lane%16, keys 4*(lane/16)..+3 of a 16-key tile.
//   O^T = V^T P^T two score tiles (32 keys) form one B operand as they lie in the registers: contraction slot
//                 8*(lane/16) + j is key 4*(lane/16) + j of the first tile for j < 4, of the second for j >= 4;
//                 the A operand reads V^T in the same slot order (two 8-byte LDS reads);
//                 D: lane holds, for query lane%16, output elements 16t + 4*(lane/16)..+3.
// So a query's running maximum, sum and rescale factor stay in its own lanes: fp32 online softmax with no
// transposition of the probabilities.  Slots above a query's position are masked before the exponential.
template <int HD>
__global__ __launch_bounds__(256) void k_attention_prompt(MbState st, const float* __restrict__ qrot,
                                                          const kv_t* __restrict__ kc, const kv_t* __restrict__ vc,
                                                          f16_t* __restrict__ out, int d)
{
    constexpr int KS = HD / 32;          // steps of the score contraction
    constexpr int ET = HD / 16;          // 16-element tiles of the output
    constexpr int OCT = HD / 8;          // 16-byte pieces per key
    constexpr int KROW = HD + 8;         // halves per staged key row (16 bytes of padding: conflict-free operand reads)
    constexpr int VROW = 32 + 4;         // halves per row of the transposed value tile (8 bytes of padding)
    constexpr int PIECES = 32 * OCT;     // 16-byte pieces of a tile
    constexpr int PPT = PIECES / 256;    // pieces per thread
    static_assert(PIECES % 256 == 0, "tile pieces per thread");
    __shared__ __attribute__((aligned(16))) _Float16 k_lds[32 * KROW];
    __shared__ __attribute__((aligned(16))) _Float16 v_lds[HD * VROW];
    const int qt = blockIdx.x, h = blockIdx.y, row = blockIdx.z;
    const int p = st.row_plen[row];      // tokens of this row in the forward: positions 0..p-1
    const int q0 = qt * 64;
    if (q0 >= p) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int ql = lane & 15, g = lane >> 4;
    const int j0 = st.row_j0[row];
    const size_t base = (size_t)st.row_so[row] * d + (size_t)h * st.row_cap[row] * HD;
    const u32x4* Kg = (const u32x4*)(kc + base);
    const u32x4* Vg = (const u32x4*)(vc + base);
    const int qpos = min(q0 + wave * 16 + ql, p - 1);   // queries past the row's end repeat its last one (never stored)
    const bool q_valid = q0 + wave * 16 + ql < p;
    const int wave_last = min(q0 + wave * 16 + 15, p - 1);
    const int n_keys = min(p, q0 + 64);
    const int n_tiles = (n_keys + 31) >> 5;
    const float scale = rsqrtf((float)HD);

    // this lane's query: head elements 32*ks + 8*g .. +7 for every step, split into two halves
    f16x8 qh[KS], qlo[KS];
    {
        const float* qp = qrot + (size_t)(j0 + qpos) * d + h * HD + 8 * g;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const float4 a = *(const float4*)(qp + 32 * ks), b = *(const float4*)(qp + 32 * ks + 4);
            const float v[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const _Float16 hi = (_Float16)v[e];
                qh[ks][e] = hi;
                qlo[ks][e] = (_Float16)(v[e] - (float)hi);
            }
        }
    }
    f32x4 o[ET];
#pragma unroll
    for (int t = 0; t < ET; ++t) o[t] = (f32x4){0.f, 0.f, 0.f, 0.f};
    float m_run = -3.0e38f, l_run = 0.f;

    u32x4 kreg[PPT], vreg[PPT];
    const u32x4 zero4 = {0u, 0u, 0u, 0u};
    auto load_tile = [&](int t) {
#pragma unroll
        for (int i = 0; i < PPT; ++i) {
            const int c = tid + i * 256;
            const int key = t * 32 + c / OCT, oct = c % OCT;
            const bool live = key < n_keys;
            const size_t at = (size_t)min(key, n_keys - 1) * OCT + oct;
            const u32x4 kv = Kg[at], vv = Vg[at];
            kreg[i] = live ? kv : zero4;
            vreg[i] = live ? vv : zero4;
        }
    };
    load_tile(0);
    for (int t = 0; t < n_tiles; ++t) {
        // stage tile t: K rows as stored, V transposed
#pragma unroll
        for (int i = 0; i < PPT; ++i) {
            const int c = tid + i * 256;
            const int key = c / OCT, oct = c % OCT;
            *(u32x4*)&k_lds[key * KROW + oct * 8] = kreg[i];
            const f16x8 vv = __builtin_bit_cast(f16x8, vreg[i]);
#pragma unroll
            for (int e = 0; e < 8; ++e) v_lds[(oct * 8 + e) * VROW + key] = vv[e];
        }
        __syncthreads();
        if (t + 1 < n_tiles) load_tile(t + 1);
        const int k0 = t * 32;
        if (k0 <= wave_last) {   // wave-uniform: tiles wholly above this wave's queries are skipped
            f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const f16x8 a0 = *(const f16x8*)&k_lds[ql * KROW + ks * 32 + 8 * g];
                const f16x8 a1 = *(const f16x8*)&k_lds[(16 + ql) * KROW + ks * 32 + 8 * g];
                s0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(a0, qlo[ks], s0, 0, 0, 0);
                s0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(a0, qh[ks], s0, 0, 0, 0);
                s1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(a1, qlo[ks], s1, 0, 0, 0);
                s1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(a1, qh[ks], s1, 0, 0, 0);
            }
            float sc[8];
            float mt = -3.0e38f;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                sc[i] = (k0 + 4 * g + i <= qpos) ? s0[i] * scale : -3.0e38f;
                sc[4 + i] = (k0 + 16 + 4 * g + i <= qpos) ? s1[i] * scale : -3.0e38f;
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) mt = fmaxf(mt, sc[i]);
            mt = fmaxf(mt, __shfl_xor(mt, 16, 64));
            mt = fmaxf(mt, __shfl_xor(mt, 32, 64));
            const float m_new = fmaxf(m_run, mt);
            const float alpha = __expf(m_run - m_new);
            float ps = 0.f;
            f16x8 pb;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const float pv = sc[i] > -1.0e38f ? __expf(sc[i] - m_new) : 0.f;
                ps += pv;
                pb[i] = (_Float16)pv;
            }
            ps += __shfl_xor(ps, 16, 64);
            ps += __shfl_xor(ps, 32, 64);
            l_run = l_run * alpha + ps;
            m_run = m_new;
#pragma unroll
            for (int tt = 0; tt < ET; ++tt) {
                const _Float16* vr = &v_lds[(tt * 16 + ql) * VROW];
                const f16x4 lo4 = *(const f16x4*)(vr + 4 * g), hi4 = *(const f16x4*)(vr + 16 + 4 * g);
                const f16x8 av = {lo4[0], lo4[1], lo4[2], lo4[3], hi4[0], hi4[1], hi4[2], hi4[3]};
                o[tt] *= alpha;
                o[tt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(av, pb, o[tt], 0, 0, 0);
            }
        }
        __syncthreads();   // the tile is rewritten next trip
    }
    if (!q_valid) return;
    const float inv = 1.f / l_run;
    const int j = j0 + qpos;
#pragma unroll
    for (int tt = 0; tt < ET; ++tt) {
        f16_t r[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) r[e] = f2h(o[tt][e] * inv);
        const size_t at = pk_index(j, h * HD + tt * 16 + 4 * g, d);
        *(uint2*)(out + at) = *(const uint2*)r;
    }
}

// Decode forwards: the (token-row, head) workgroup first finishes its own slice of the q|k|v projection
// (sums the k-slices, rotates q and k at the row's position, appends k and v to the row's slab), then
// attends.  Saves a launch and the round trip of q through HBM for every layer of every step.
// NW waves per workgroup: 8 (256 cache slots per round trip) when the grid is small enough for every workgroup to
// be resident with room to spare, 4 (128 slots) for larger batches, whose many workgroups already fill the chip.
template <int HD, int NW>
__global__ __launch_bounds__(64 * NW) void k_attention_decode(MbState st, const float* __restrict__ part, int ksplit,
                                                          size_t part_stride, kv_t* __restrict__ kc,
                                                          kv_t* __restrict__ vc, const float* __restrict__ rcos,
                                                          const float* __restrict__ rsin, f16_t* __restrict__ out,
                                                          int d)
{
    __shared__ float sc[kMaxPos];
    __shared__ float red[2 * NW];
    __shared__ float oacc[NW][HD];
    __shared__ float qs[HD];
    constexpr int HALF = HD / 2;
    const int j = blockIdx.x, h = blockIdx.y;
    // count, row and position are requested together (the tables are sized for the grid); only the loads that
    // are indexed by the row wait for the count check
    const int count = *st.d_n;
    const int row = st.tr_row[j], pos = st.tr_pos[j];
    if (j >= count) return;
    const size_t base = (size_t)st.row_so[row] * d + (size_t)h * st.row_cap[row] * HD;
    const int which = threadIdx.x / HALF, e = threadIdx.x % HALF;   // 0 q, 1 k, 2 v
    if (which < 3) {
        const float* p = part + (size_t)j * 3 * d + (size_t)which * d + h * HD + e;
        float pa[kNormMaxSplit], pb[kNormMaxSplit];   // every k-slice load issued before the first add
#pragma unroll
        for (int s = 0; s < kNormMaxSplit; ++s) {
            pa[s] = s < ksplit ? p[(size_t)s * part_stride] : 0.f;
            pb[s] = s < ksplit ? p[(size_t)s * part_stride + HALF] : 0.f;
        }
        float a = 0.f, b = 0.f;
#pragma unroll
        for (int s = 0; s < kNormMaxSplit; ++s) {
            a += pa[s];
            b += pb[s];
        }
        if (which < 2) {
            const float cs = rcos[(size_t)pos * HALF + e], sn = rsin[(size_t)pos * HALF + e];
            const float ra = a * cs - b * sn, rb = a * sn + b * cs;
            a = ra;
            b = rb;
        }
        if (which == 0) {
            qs[e] = a;
            qs[e + HALF] = b;
        } else {
            kv_t* dst = (which == 1 ? kc : vc) + base + (size_t)pos * HD + e;
            dst[0] = f2kv(a);
            dst[HALF] = f2kv(b);
        }
    }
    __syncthreads();   // the new key/value slot and q are visible to the whole workgroup
    attend<HD, NW>(qs, sc, red, oacc, kc + base, vc + base, pos + 1, out, j, h * HD, d);
}

// ------------------------------------------------------------------------------------------ argmax
// Greedy choice per selected row: index of the largest logit, lowest index on exact ties.
// 1024 threads per row, all of a thread's loads issued before the first compare.
__global__ __launch_bounds__(1024) void k_argmax(const float* __restrict__ logits, int vocab,
                                                 const int32_t* __restrict__ d_count, int32_t* __restrict__ am)
{
    const int j = blockIdx.x;
    if (j >= *d_count) return;
    const float* lg = logits + (size_t)j * vocab;
    float best = -3.4e38f;
    int bi = 0x7fffffff;
    for (int c0 = threadIdx.x * 4; c0 < vocab; c0 += 4096 * 4) {
        float4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int c = c0 + u * 4096;
            v[u] = c < vocab ? *(const float4*)(lg + c) : make_float4(-3.4e38f, -3.4e38f, -3.4e38f, -3.4e38f);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int c = c0 + u * 4096;
            const float vv[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (c < vocab && (vv[e] > best || (vv[e] == best && c + e < bi))) { best = vv[e]; bi = c + e; }
        }
    }
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) {
        const float ob = __shfl_xor(best, m, 64);
        const int oi = __shfl_xor(bi, m, 64);
        if (ob > best || (ob == best && oi < bi)) { best = ob; bi = oi; }
    }
    __shared__ float sb[16];
    __shared__ int si[16];
    if ((threadIdx.x & 63) == 0) { sb[threadIdx.x >> 6] = best; si[threadIdx.x >> 6] = bi; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < 16; ++w)
            if (sb[w] > best || (sb[w] == best && si[w] < bi)) { best = sb[w]; bi = si[w]; }
        // no logit compared greater than the start value (a row of NaN or -inf): id 0, never an id outside the
        // vocabulary, which the next step would use as an embedding row
        am[j] = (unsigned)bi < (unsigned)vocab ? bi : 0;
    }
}

// ------------------------------------------------------------------------------------------ sampling
// Temperature sampling per selected row (Sec. 4.2, Experimental Setting: responses are sampled at a temperature):
// token = smallest v with  sum_{v' <= v} e_v'  >  u * sum_v' e_v',  e_v = exp((logit_v - max) * inv_temp),
// u being the draw for (row, token number): supplied by the caller, or generated from a counter (below).  The CDF runs in vocabulary order, so thread t owns
// the contiguous chunk [t*c, (t+1)*c): it sums its chunk in index order, a workgroup scan of the 1024
// chunk sums finds the first chunk whose running total exceeds the target, and that chunk's owner walks
// it again in the same order (same additions, same roundings) to the token.  V-1 when rounding leaves no
// chunk above the target.  1024 threads per row; the row's logits (just written by the LM head) are read
// three times from L2.
// Counter-based draw in [0,1): Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC 2011) on the counter
// (token number, row id, 0, 0) under the 64-bit key; the top 24 bits of the first output word, scaled by 2^-24.
__device__ inline float philox_draw(uint32_t k0, uint32_t k1, uint32_t id, uint32_t t)
{
    uint32_t c0 = t, c1 = id, c2 = 0u, c3 = 0u;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
        const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
        c0 = hi1 ^ c1 ^ k0;
        c1 = lo1;
        c2 = hi0 ^ c3 ^ k1;
        c3 = lo0;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return (float)(c0 >> 8) * (1.0f / 16777216.0f);
}

__global__ __launch_bounds__(1024) void k_sample(const float* __restrict__ logits, int vocab,
                                                 const int32_t* __restrict__ d_count, MbState st,
                                                 const float* __restrict__ draws, const int32_t* __restrict__ ids,
                                                 uint32_t key0, uint32_t key1, float inv_temp)
{
    const int j = blockIdx.x;
    if (j >= *d_count) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int row = st.live_row[j];
    const int t = *st.d_step;
    const float u = draws ? draws[(size_t)row * st.max_new + t] : philox_draw(key0, key1, (uint32_t)ids[row], (uint32_t)t);
    const float* lg = logits + (size_t)j * vocab;
    const int c = (((vocab + 1023) >> 10) + 3) & ~3;   // floats per thread, a multiple of 4 (vocab % 16 == 0)
    const int lo = tid * c;
    const int hi = lo + c < vocab ? lo + c : vocab;    // lo >= vocab: empty chunk

    __shared__ float s_red[16];
    __shared__ float s_tot[17];
    __shared__ int s_owner[16];

    float m = -3.4e38f;
    for (int v = lo; v < hi; v += 4) {
        const float4 q = *(const float4*)(lg + v);
        m = fmaxf(fmaxf(m, fmaxf(q.x, q.y)), fmaxf(q.z, q.w));
    }
#pragma unroll
    for (int k = 32; k >= 1; k >>= 1) m = fmaxf(m, __shfl_xor(m, k, 64));
    if (lane == 0) s_red[wave] = m;
    __syncthreads();
    m = s_red[0];
#pragma unroll
    for (int w = 1; w < 16; ++w) m = fmaxf(m, s_red[w]);

    float csum = 0.f;
    for (int v = lo; v < hi; v += 4) {
        const float4 q = *(const float4*)(lg + v);
        csum += expf((q.x - m) * inv_temp);
        csum += expf((q.y - m) * inv_temp);
        csum += expf((q.z - m) * inv_temp);
        csum += expf((q.w - m) * inv_temp);
    }
    // inclusive scan of the chunk sums: within the wave, then over the 16 wave totals
    float incl = csum;
#pragma unroll
    for (int k = 1; k < 64; k <<= 1) {
        const float o = __shfl_up(incl, k, 64);
        if (lane >= k) incl += o;
    }
    if (lane == 63) s_tot[wave + 1] = incl;
    __syncthreads();
    if (tid == 0) {
        float a = 0.f;
        s_tot[0] = 0.f;
        for (int w = 1; w <= 16; ++w) { a += s_tot[w]; s_tot[w] = a; }
    }
    __syncthreads();
    const float base = s_tot[wave];
    const float target = u * s_tot[16];
    const float before = base + (incl - csum);   // running total ahead of this chunk
    const float upto = base + incl;
    const unsigned long long hit = __ballot(upto > target);
    if (lane == 0) s_owner[wave] = hit ? (wave << 6) + __ffsll((long long)hit) - 1 : 0x7fffffff;
    __syncthreads();
    int owner = 0x7fffffff;
#pragma unroll
    for (int w = 0; w < 16; ++w) owner = s_owner[w] < owner ? s_owner[w] : owner;
    if (owner == 0x7fffffff) {
        if (tid == 0) st.am[j] = vocab - 1;
        return;
    }
    if (tid != owner) return;
    const float want = target - before;
    float acc = 0.f;
    int pick = hi - 1;
    for (int v = lo; v < hi; ++v) {
        acc += expf((lg[v] - m) * inv_temp);
        if (acc > want) { pick = v; break; }
    }
    st.am[j] = pick;
}

// ------------------------------------------------------------------------------------------ bookkeeping
// After a forward: slot j's chosen token is the row's token number s (s = tokens generated so far).  Emit it
// if the row still owes tokens, then build the next forward: every surviving slot feeds its token back at
// position prompt_len + s.  With `compact` a row leaves the live batch once it has emitted its last token;
// without it the row stays and keeps running on its own output (its later tokens are never emitted).
// A row that emits `eos_id` (never matched when it is -1) has emitted its last token: its limit drops to
// s + 1, which is also where the host reads the row's length afterwards.  *st.d_active counts the rows that
// still owe tokens, for a host that does not know the lengths and polls.
__global__ __launch_bounds__(1024) void k_step_update(MbState st, int compact, int eos_id)
{
    __shared__ int wave_cnt[16];
    __shared__ int wave_act[16];
    __shared__ int wave_off[17];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = *st.d_nlive;
    const int s = *st.d_step;
    int row = -1, tok = 0, keep = 0, owes = 0;
    if (tid < n) {
        row = st.live_row[tid];
        tok = st.am[tid];
        int lim = st.row_limit[row];
        if (s < lim) {
            st.out_tok[(size_t)row * st.max_new + s] = tok;
            if (tok == eos_id && s + 1 < lim) {
                lim = s + 1;
                st.row_limit[row] = lim;
            }
        }
        owes = s + 1 < lim;
        keep = compact ? owes : 1;
    }
    const unsigned long long bal = __ballot(keep);
    const unsigned long long act = __ballot(owes);
    const int before = __popcll(bal & ((1ull << lane) - 1ull));
    if (lane == 0) { wave_cnt[wave] = __popcll(bal); wave_act[wave] = __popcll(act); }
    __syncthreads();
    if (tid == 0) {
        int a = 0, b = 0;
        for (int w = 0; w < 16; ++w) { wave_off[w] = a; a += wave_cnt[w]; b += wave_act[w]; }
        wave_off[16] = a;
        *st.d_active = b;
    }
    __syncthreads();
    if (keep) {
        const int jn = wave_off[wave] + before;
        st.tr_tok[jn] = tok;
        st.tr_row[jn] = row;
        st.tr_pos[jn] = st.row_plen[row] + s;
        st.live_row[jn] = row;
    }
    if (tid == 0) {
        *st.d_n = wave_off[16];
        *st.d_nlive = wave_off[16];
        *st.d_step = s + 1;
    }
}

// ------------------------------------------------------------------------------------------ read probe
// Measurement aid: a plain read stream over a packed weight matrix, one wave per 64 KiB chunk, 8 non-temporal
// 16-byte loads per lane in flight, nothing computed.  The rate it reaches at a projection's size is the
// ceiling that the projection kernels are compared with.
__global__ __launch_bounds__(256) void k_read_stream(const u32x4* __restrict__ p, int n_chunks, uint32_t* __restrict__ sink)
{
    const int lane = threadIdx.x & 63;
    const int w = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (w >= n_chunks) return;
    const u32x4* q = p + (size_t)w * 4096 + lane;   // 64 KiB = 4096 vectors of 16 bytes
    u32x4 acc = {0u, 0u, 0u, 0u};
    for (int i = 0; i < 4096; i += 512) {
        u32x4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = __builtin_nontemporal_load(q + i + u * 64);
#pragma unroll
        for (int u = 0; u < 8; ++u) acc ^= v[u];
    }
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9E3779B9u) sink[0] = 1u;   // keeps the loads alive; bf16 weights never hit it in practice
}

// ------------------------------------------------------------------------------------------ launchers
static inline int grid_for(size_t n, int block)
{
    const size_t g = (n + block - 1) / block;
    return (int)(g > (1u << 20) ? (1u << 20) : (g < 1 ? 1 : g));
}

void launch_pack_weight(const void* src, int src_f32, f16_t* dst, int n_src, int k, int kp, int blk_stride,
                        int blk_off, hipStream_t s)
{
    const size_t total = (size_t)n_src * (k / 8);
    hipLaunchKernelGGL(k_pack_weight, dim3(grid_for(total, 256)), dim3(256), 0, s, src, src_f32, dst, n_src, k, kp,
                       blk_stride, blk_off);
}

void launch_cast_rows(const void* src, int src_f32, bf16_t* dst, size_t count, hipStream_t s)
{
    hipLaunchKernelGGL(k_cast_rows, dim3(grid_for(count, 256)), dim3(256), 0, s, src, src_f32, dst, count);
}

void launch_fill_i32(int32_t* p, int32_t v, size_t n, hipStream_t s)
{
    if (n == 0) return;
    hipLaunchKernelGGL(k_fill_i32, dim3(grid_for(n, 256)), dim3(256), 0, s, p, v, n);
}

void launch_embed(const MbState& st, const bf16_t* embed, float* x, int d, int n_max, hipStream_t s)
{
    hipLaunchKernelGGL(k_embed, dim3(n_max), dim3(256), 0, s, st, embed, x, d);
}

void launch_rmsnorm(const MbState& st, float* x, const float* part, int ksplit, size_t part_stride,
                    const bf16_t* w, float eps, const int32_t* sel, const int32_t* d_nsel, f16_t* h_packed, int d,
                    int n_max, hipStream_t s)
{
    // Few rows: 1024 threads per row, the whole row in one round trip.  Many rows (prompt forwards): 256 threads per
    // row, so that eight rows share a compute unit and the launch is bound by bytes rather than by workgroup
    // start-up (measured at the 7B width: a prompt forward of 640 token-rows takes 13.8 ms, against 15.8 with 1024
    // threads per row, whose norm launches took 47 us each there; up to 256 rows the wide form is the faster one:
    // 24 rows 3.29 against 3.37 ms per decode step, 256 rows equal).
    if (n_max >= kNormNarrowFrom)
        hipLaunchKernelGGL((k_rmsnorm<256, 8>), dim3(n_max), dim3(256), 0, s, d_nsel ? d_nsel : st.d_n, x, part,
                           part ? ksplit : 0, part_stride, w, eps, sel, h_packed, d);
    else
        hipLaunchKernelGGL((k_rmsnorm<1024, 2>), dim3(n_max), dim3(1024), 0, s, d_nsel ? d_nsel : st.d_n, x, part,
                           part ? ksplit : 0, part_stride, w, eps, sel, h_packed, d);
}

void launch_swiglu_reduce(const float* part, int ksplit, size_t part_stride, int m_rows, int F, int kp_out,
                          f16_t* out, hipStream_t s)
{
    hipLaunchKernelGGL(k_swiglu_reduce, dim3((F / 4 + 255) / 256, m_rows), dim3(256), 0, s, part, ksplit, part_stride,
                       m_rows, F, kp_out, out);
}

template <int MT, int NB, int KD, int EPI>
static void launch_skinny_inst(const GemmArgs& a, hipStream_t s)
{
    const int KB = a.Kp / 32;
    const int groups = (a.N / 16 + NB - 1) / NB;
    const int kbs = (KB + a.ksplit - 1) / a.ksplit;
    hipLaunchKernelGGL((k_gemm_skinny<MT, NB, KD, EPI>), dim3(groups * a.ksplit), dim3(256), 0, s, a, groups, kbs);
}

template <int MT, int EPI>
static void launch_skinny_mt(const GemmArgs& a, hipStream_t s)
{
    if (a.nb == 2) {
        if (a.kd == 2) launch_skinny_inst<MT, 2, 2, EPI>(a, s);
        else launch_skinny_inst<MT, 2, 4, EPI>(a, s);
    } else {
        if (a.kd == 2 || MT > 2) launch_skinny_inst<MT, 4, 2, EPI>(a, s);
        else launch_skinny_inst<MT, 4, 4, EPI>(a, s);
    }
}

template <int P, int MT, int NBW, int EPI, int KH>
static void launch_sweep_inst(const GemmArgs& a, int units, hipStream_t s)
{
    const int KB = a.Kp / 32;
    const int kbs = (KB + a.ksplit - 1) / a.ksplit;
    hipLaunchKernelGGL((k_gemm_sweep<P, MT, NBW, EPI, KH>), dim3(a.sweep_gn * a.ksplit), dim3(64 * P), 0, s, a, units,
                       a.sweep_gn, kbs);
}

template <int P, int MT, int EPI, int KH>
static void launch_sweep_mt(const GemmArgs& a, int units, hipStream_t s)
{
    // strips per wave (sweep_nbw): a gate/up pair with the SwiGLU epilogue, otherwise one
    launch_sweep_inst<P, MT, EPI == EPI_SWIGLU ? 2 : 1, EPI, KH>(a, units, s);
}

template <int P, int EPI, int KH>
static void launch_sweep_p(const GemmArgs& a, int units, hipStream_t s)
{
    switch ((a.m_rows + 15) / 16) {
        case 1: launch_sweep_mt<P, 1, EPI, 1>(a, units, s); break;   // one row strip: never split
        case 2: launch_sweep_mt<P, 2, EPI, KH>(a, units, s); break;
        case 3: launch_sweep_mt<P, 3, EPI, KH>(a, units, s); break;
        case 4: launch_sweep_mt<P, 4, EPI, KH>(a, units, s); break;
        case 5: launch_sweep_mt<P, 5, EPI, KH>(a, units, s); break;
        case 6: launch_sweep_mt<P, 6, EPI, KH>(a, units, s); break;
        case 7: launch_sweep_mt<P, 7, EPI, KH>(a, units, s); break;
        case 8: launch_sweep_mt<P, 8, EPI, KH>(a, units, s); break;
        case 9: launch_sweep_mt<P, 9, EPI, KH>(a, units, s); break;
        case 10: launch_sweep_mt<P, 10, EPI, KH>(a, units, s); break;
        case 11: launch_sweep_mt<P, 11, EPI, KH>(a, units, s); break;
        case 12: launch_sweep_mt<P, 12, EPI, KH>(a, units, s); break;
        case 13: launch_sweep_mt<P, 13, EPI, KH>(a, units, s); break;
        case 14: launch_sweep_mt<P, 14, EPI, KH>(a, units, s); break;
        case 15: launch_sweep_mt<P, 15, EPI, KH>(a, units, s); break;
        default: launch_sweep_mt<P, 16, EPI, KH>(a, units, s); break;
    }
}

template <int TMS, int KP, int EPI>
static void launch_tiled(const GemmArgs& a, hipStream_t s)
{
    const int KB = a.Kp / 32;
    const int kbs = (KB + a.ksplit - 1) / a.ksplit;
    const int n_ntiles = (a.N + 255) / 256, n_mtiles = (a.m_rows + TMS * 16 - 1) / (TMS * 16);
    const int grid = (n_ntiles + 7) / 8 * 8 * n_mtiles * a.ksplit;
    hipLaunchKernelGGL((k_gemm_tiled<TMS, KP, EPI>), dim3(grid), dim3(256 * KP), 0, s, a, kbs, n_ntiles, n_mtiles);
}

template <int EPI>
static void launch_gemm_epi(const GemmArgs& a, hipStream_t s)
{
    if (a.m_rows <= kSweepMaxRows && a.sweep_p > 0 && a.sweep_gn > 0 && a.zero_blk) {
        const int nbw = sweep_nbw(EPI, a.m_rows);
        const int units = (a.N / 16 + nbw - 1) / nbw;
        const int per = (units + a.sweep_gn - 1) / a.sweep_gn;   // most units any workgroup owns
        if (a.sweep_p == 4 && per <= 4) {
            // where the plan asks for it (above 96 rows): 8 waves, two per unit (see SweepSlot)
            if (a.m_rows > 16 && a.sweep_kh == 2) return launch_sweep_p<8, EPI, 2>(a, units, s);
            return launch_sweep_p<4, EPI, 1>(a, units, s);
        }
        if (per <= 8) return launch_sweep_p<8, EPI, 1>(a, units, s);
        // a plan this kernel cannot run falls through to the other kernels
    }
    if (a.m_rows <= 64) {
        const int mt = (a.m_rows + 15) / 16;
        switch (mt) {
            case 1: launch_skinny_mt<1, EPI>(a, s); break;
            case 2: launch_skinny_mt<2, EPI>(a, s); break;
            case 3: launch_skinny_mt<3, EPI>(a, s); break;
            default: launch_skinny_mt<4, EPI>(a, s); break;
        }
        return;
    }
    if (a.tms == 8 && a.kp != 2) return launch_tiled<8, 1, EPI>(a, s);
    if (a.kp == 2) return launch_tiled<4, 2, EPI>(a, s);
    launch_tiled<4, 1, EPI>(a, s);
}

void launch_gemm(const GemmArgs& a, int epilogue, hipStream_t s)
{
    if (epilogue == EPI_SWIGLU)
        launch_gemm_epi<EPI_SWIGLU>(a, s);
    else
        launch_gemm_epi<EPI_PARTIAL>(a, s);
}

void launch_rope_append(const MbState& st, const float* qkv_part, int ksplit, size_t part_stride, float* qrot,
                        kv_t* kcache, kv_t* vcache, const float* rope_cos, const float* rope_sin, int d, int H,
                        int hd, int n_max, hipStream_t s)
{
    hipLaunchKernelGGL(k_rope_append, dim3(n_max), dim3(256), 0, s, st, qkv_part, ksplit, part_stride, qrot, kcache,
                       vcache, rope_cos, rope_sin, d, H, hd);
}

template <int HD, int NW>
static void launch_attention_decode_inst(const MbState& st, const float* qkv_part, int ksplit, size_t part_stride,
                                         kv_t* kcache, kv_t* vcache, const float* rope_cos, const float* rope_sin,
                                         f16_t* out_packed, int d, int H, int n_max, hipStream_t s)
{
    hipLaunchKernelGGL((k_attention_decode<HD, NW>), dim3(n_max, H), dim3(64 * NW), 0, s, st, qkv_part, ksplit, part_stride,
                       kcache, vcache, rope_cos, rope_sin, out_packed, d);
}

void launch_attention_decode(const MbState& st, const float* qkv_part, int ksplit, size_t part_stride,
                             kv_t* kcache, kv_t* vcache, const float* rope_cos, const float* rope_sin,
                             f16_t* out_packed, int d, int H, int hd, int n_max, hipStream_t s)
{
    // measured at the 7B shape: 8 waves win at 16 rows (512 workgroups: 14.1 against 14.9 us per layer at context
    // 200), 4 waves win at 64 rows (2048 workgroups: 25.7 against 36.1 us at context 100)
    const bool wide = n_max * H <= kAttnWideMaxGroups;
#define SS_ATTN_ARGS st, qkv_part, ksplit, part_stride, kcache, vcache, rope_cos, rope_sin, out_packed, d, H, n_max, s
    if (hd == 128) {
        if (wide) launch_attention_decode_inst<128, 8>(SS_ATTN_ARGS);
        else launch_attention_decode_inst<128, 4>(SS_ATTN_ARGS);
    } else {
        if (wide) launch_attention_decode_inst<64, 8>(SS_ATTN_ARGS);
        else launch_attention_decode_inst<64, 4>(SS_ATTN_ARGS);
    }
#undef SS_ATTN_ARGS
}

void launch_attention_prompt(const MbState& st, const float* qrot, const kv_t* kcache, const kv_t* vcache,
                             f16_t* out_packed, int d, int H, int hd, int B, int max_len, hipStream_t s)
{
    const dim3 grid((max_len + 63) / 64, H, B);
    if (hd == 128)
        hipLaunchKernelGGL((k_attention_prompt<128>), grid, dim3(256), 0, s, st, qrot, kcache, vcache, out_packed, d);
    else
        hipLaunchKernelGGL((k_attention_prompt<64>), grid, dim3(256), 0, s, st, qrot, kcache, vcache, out_packed, d);
}

void launch_argmax(const float* logits, int vocab, const int32_t* d_nsel, int32_t* am, int n_max, hipStream_t s)
{
    hipLaunchKernelGGL(k_argmax, dim3(n_max), dim3(1024), 0, s, logits, vocab, d_nsel, am);
}

void launch_read_stream(const f16_t* p, size_t bytes, uint32_t* sink, hipStream_t s)
{
    const int n_chunks = (int)(bytes >> 16);
    if (n_chunks < 1) return;
    hipLaunchKernelGGL(k_read_stream, dim3((n_chunks + 3) / 4), dim3(256), 0, s, (const u32x4*)p, n_chunks, sink);
}

void launch_sample(const float* logits, int vocab, const int32_t* d_nsel, const MbState& st, const float* draws,
                   const int32_t* ids, uint64_t seed, float inv_temp, int n_max, hipStream_t s)
{
    hipLaunchKernelGGL(k_sample, dim3(n_max), dim3(1024), 0, s, logits, vocab, d_nsel, st, draws, ids,
                       (uint32_t)(seed & 0xffffffffu), (uint32_t)(seed >> 32), inv_temp);
}

void launch_step_update(const MbState& st, int compact, int eos_id, hipStream_t s)
{
    hipLaunchKernelGGL(k_step_update, dim3(1), dim3(1024), 0, s, st, compact, eos_id);
}

}  // namespace ss
