// Launch wrappers of the gfx950 kernels (host side).  All pointers are device pointers.
#ifndef SS_KERNELS_H
#define SS_KERNELS_H

#include <hip/hip_runtime.h>

#include <cstdint>

#include "ss_plan.h"

namespace ss {

typedef uint16_t bf16_t;  // bf16 bit pattern (source tensors, embedding rows, norm gains)
typedef uint16_t f16_t;   // IEEE half bit pattern: both operands of every projection (packed weights, packed activations)
typedef uint16_t kv_t;    // key/value cache slot: IEEE half bit pattern

// Packed weight matrix: N output rows (multiple of 16), K inputs padded to Kp (multiple of 64).
struct PackedMat {
    f16_t* p = nullptr;
    int N = 0, K = 0, Kp = 0;
};

// Per-micro-batch device state read and written by the kernels, so that one decode step can be
// replayed without any host-side scalar changing.
struct MbState {
    int32_t* d_n;        // [1] token-rows of the next forward
    int32_t* d_step;     // [1] tokens generated so far by every live row (rows advance in lockstep)
    int32_t* tr_tok;     // [n_max] token id fed by token-row j
    int32_t* tr_row;     // [n_max] micro-batch row of token-row j
    int32_t* tr_pos;     // [n_max] position of token-row j inside its row
    int32_t* live_row;   // [B]     rows still in the live batch, in slot order
    int32_t* d_nlive;    // [1]
    int32_t* d_active;   // [1] rows that still owe tokens after the last bookkeeping step
    int32_t* row_plen;   // [B] prompt length
    int32_t* row_j0;     // [B] first token-row of the row in a prompt forward
    int32_t* row_limit;  // [B] min(target, cap): tokens the row emits; lowered by the device when the row emits its end id
    int64_t* row_so;     // [B] first key/value slot of the row's slab
    int32_t* row_cap;    // [B] slots in the row's slab (prompt + cap)
    int32_t* am;         // [n_sel_max] argmax of the selected rows' logits
    int32_t* out_tok;    // [B][max_new]
    int32_t max_new;
};

struct GemmArgs {
    const f16_t* W;      // packed [N, Kp]
    const f16_t* X;      // packed [rows, Kp] activations
    float* out;          // EPI_PARTIAL: [ksplit][m_stride][N] fp32
    f16_t* out_packed;   // EPI_SWIGLU: packed [rows, kp_out], column f = silu(gate_f) * up_f
    int N, Kp, m_rows;   // m_rows: rows to compute (stores are guarded by it)
    int m_stride;        // row stride (in rows) between k-slices of `out`
    int kp_out;          // padded K of out_packed
    int ksplit;          // outer k-slices (gemm_plan)
    int nb, kd;          // skinny kernel shape (gemm_plan)
    int kp;              // tiled kernel: k-parts inside the workgroup (gemm_plan)
    int tms;             //      row strips per tile, 4 or 8 (gemm_plan)
    int sweep_p;         // > 0: sweep kernel with this many waves per workgroup (gemm_plan)
    int sweep_gn;        //      its workgroups per k-slice
    int sweep_kh;        //      2: two waves per unit, each half of every chunk's k-blocks (gemm_plan)
    const f16_t* zero_blk;   // 1 KiB of zeros: operand block read in place of weights beyond a range (sweep kernel)
};

void launch_pack_weight(const void* src, int src_f32, f16_t* dst, int n_src, int k, int kp, int blk_stride,
                        int blk_off, hipStream_t s);
void launch_cast_rows(const void* src, int src_f32, bf16_t* dst, size_t count, hipStream_t s);
void launch_embed(const MbState& st, const bf16_t* embed, float* x, int d, int n_max, hipStream_t s);
void launch_rmsnorm(const MbState& st, float* x, const float* part, int ksplit, size_t part_stride,
                    const bf16_t* w, float eps, const int32_t* sel, const int32_t* d_nsel, f16_t* h_packed, int d,
                    int n_max, hipStream_t s);
void launch_gemm(const GemmArgs& a, int epilogue, hipStream_t s);
void launch_swiglu_reduce(const float* part, int ksplit, size_t part_stride, int m_rows, int F, int kp_out,
                          f16_t* out, hipStream_t s);
void launch_rope_append(const MbState& st, const float* qkv_part, int ksplit, size_t part_stride, float* qrot,
                        kv_t* kcache, kv_t* vcache, const float* rope_cos, const float* rope_sin, int d, int H,
                        int hd, int n_max, hipStream_t s);
// Causal attention of a prompt forward: B rows, row i holding st.row_plen[i] token-rows that start at token-row
// st.row_j0[i]; max_len = the longest row (sizes the grid).
void launch_attention_prompt(const MbState& st, const float* qrot, const kv_t* kcache, const kv_t* vcache,
                             f16_t* out_packed, int d, int H, int hd, int B, int max_len, hipStream_t s);
void launch_attention_decode(const MbState& st, const float* qkv_part, int ksplit, size_t part_stride,
                             kv_t* kcache, kv_t* vcache, const float* rope_cos, const float* rope_sin,
                             f16_t* out_packed, int d, int H, int hd, int n_max, hipStream_t s);
void launch_argmax(const float* logits, int vocab, const int32_t* d_nsel, int32_t* am, int n_max, hipStream_t s);
// Temperature sampling in place of the argmax: st.am[j] for the first *d_nsel selected rows.  The draw of slot j
// (row r = st.live_row[j], token number t = *st.d_step) is draws[r * st.max_new + t], or with draws == nullptr
// the counter-based generator's draw for (ids[r], t) under `seed`.
void launch_sample(const float* logits, int vocab, const int32_t* d_nsel, const MbState& st, const float* draws,
                   const int32_t* ids, uint64_t seed, float inv_temp, int n_max, hipStream_t s);
// eos_id: -1 when rows end only at their limit.
void launch_step_update(const MbState& st, int compact, int eos_id, hipStream_t s);
// Reads the first bytes/65536 chunks of 64 KiB at p and discards them (bandwidth probe).
void launch_read_stream(const f16_t* p, size_t bytes, uint32_t* sink, hipStream_t s);
void launch_fill_i32(int32_t* p, int32_t v, size_t n, hipStream_t s);

}  // namespace ss

#endif
