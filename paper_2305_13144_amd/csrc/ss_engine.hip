// Host side of the decode engine: weight upload/packing, the grow-only device workspace, one
// forward over a list of token-rows, and the C-ABI entry points built on it (Sec. 4.1 of the paper:
// micro-batch generation with a cap, failure collection and recomputation after the group).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <chrono>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <numeric>
#include <thread>
#include <vector>

#include "ss_internal.h"
#include "ss_kernels.h"

using ss::bf16_t;
using ss::f16_t;
using ss::GemmArgs;
using ss::MbState;
using ss::PackedMat;

#define HIPCHK(expr)                                                                              \
    do {                                                                                          \
        hipError_t e_ = (expr);                                                                   \
        if (e_ != hipSuccess)                                                                     \
            return ss::fail(e_ == hipErrorOutOfMemory ? SS_ENOMEM : SS_EDEVICE, "%s: %s", #expr, \
                            hipGetErrorString(e_));                                               \
    } while (0)

// Workspace of ss_decode_microbatch_static: one array per GPU, held until the process ends.  In host code the
// array's name is only a handle for hipGetSymbolAddress; the device address it returns (per device) is what the
// kernels and fills get.
constexpr size_t kStaticScratchBytes = (size_t)SS_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices] = {};        // device address of `scratch` on each device, once looked up
std::atomic<int> g_scratch_busy[kMaxDevices];  // 1 while a static call runs on that device

// Device address of this device's copy of `scratch`; `device` must be the current device.
int scratch_address(int device, void** out)
{
    if (device < 0 || device >= kMaxDevices) return ss::fail(SS_EDEVICE, "device ordinal %d not supported", device);
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[device]) {
        void* ptr = nullptr;
        hipError_t e = hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr)
            return ss::fail(SS_EDEVICE, "hipGetSymbolAddress(scratch) on device %d: %s", device, hipGetErrorString(e));
        g_scratch_ptr[device] = ptr;
    }
    *out = g_scratch_ptr[device];
    return SS_OK;
}

}  // namespace

namespace {

struct Layer {
    bf16_t *attn_norm = nullptr, *mlp_norm = nullptr;
    PackedMat wqkv, wo, wgu, wd;
};

// A grow-only device buffer.
struct Buf {
    void* p = nullptr;
    size_t bytes = 0;
    bool borrowed = false;   // a view into memory owned elsewhere (the static scratch array): never grown or freed
    int ensure(size_t need, bool zero)
    {
        if (need <= bytes) return SS_OK;
        if (borrowed) return ss::fail(SS_ESTATE, "a borrowed buffer of %zu bytes cannot grow to %zu", bytes, need);
        if (p) (void)hipFree(p);
        p = nullptr;
        bytes = 0;
        const size_t want = need + need / 8;
        hipError_t e = hipMalloc(&p, want);
        if (e != hipSuccess) {
            p = nullptr;
            return ss::fail(SS_ENOMEM, "hipMalloc(%zu bytes): %s", want, hipGetErrorString(e));
        }
        bytes = want;
        if (zero) {
            e = hipMemset(p, 0, want);
            if (e != hipSuccess) return ss::fail(SS_EDEVICE, "hipMemset: %s", hipGetErrorString(e));
        }
        return SS_OK;
    }
    void release()
    {
        if (p && !borrowed) (void)hipFree(p);
        p = nullptr;
        bytes = 0;
        borrowed = false;
    }
    template <class T>
    T* as() const { return (T*)p; }
};

struct Workspace {
    Buf x, h, ao, act, qrot, pqkv, pd, pgu, hsel, logits, kv, ints, i64s, draws;
    // Non-null: every buffer is carved out of [arena, arena + arena_bytes) instead of being allocated.
    char* arena = nullptr;
    size_t arena_bytes = 0;
    void release()
    {
        for (Buf* b : {&x, &h, &ao, &act, &qrot, &pqkv, &pd, &pgu, &hsel, &logits, &kv, &ints, &i64s, &draws})
            b->release();
    }
};

}  // namespace

// What one micro-batch in flight owns: its stream, workspace, device state and the token choice of its forwards.
// A handle has kLanes of them; every entry point works on lane 0, and a group pass may run further micro-batches
// on the other lanes at the same time (the weights are shared and only read).
namespace {
constexpr int kLanes = SS_IN_FLIGHT_MAX;
struct Lane {
    hipStream_t stream = nullptr;
    Workspace ws;
    int32_t* d_sel = nullptr;  // carved from ws.ints
    MbState st{};
    size_t kv_layer_stride = 0;  // elements between a layer's K and V, and 2x that between layers
    // token choice of the forward in flight: cur_inv_temp == 0 selects the argmax; otherwise sampling with the
    // draws in cur_draws, or (cur_draws == nullptr) generated from (cur_seed, cur_ids[row], token number)
    const float* cur_draws = nullptr;
    const int32_t* cur_ids = nullptr;
    uint64_t cur_seed = 0;
    float cur_inv_temp = 0.f;
    int32_t* h_poll = nullptr;   // pinned host copy of the 4-int device header (d_n, d_step, d_nlive, d_active)
    hipEvent_t ev[3] = {nullptr, nullptr, nullptr};   // start, end of the prompt forward, end of a micro-batch
    int prompt_rows = 0, prompt_max_len = 0;   // shape of the prompt forward whose state was uploaded last
};
}  // namespace

struct ss_weights {
    ss_model_cfg cfg{};
    int device = 0;
    std::vector<void*> allocs;
    bf16_t* embed = nullptr;
    std::vector<Layer> layers;
    bf16_t* final_norm = nullptr;
    PackedMat lm_head;
    float *rope_cos = nullptr, *rope_sin = nullptr;
    f16_t* zero_blk = nullptr;    // 1 KiB of zeros (see GemmArgs::zero_blk)
    int n_cu = 256;               // compute units of the device
    Lane lane[kLanes];
    std::atomic<int> busy{0};
    void* scratch_ptr = nullptr;   // device address of this device's static scratch array
    int in_flight = SS_IN_FLIGHT_DEFAULT;       // micro-batches a group pass keeps in flight (1 to kLanes)
};

namespace {

struct BusyGuard {
    ss_weights* w;
    bool ok;
    explicit BusyGuard(ss_weights* w_) : w(w_), ok(w_->busy.exchange(1) == 0) {}
    ~BusyGuard()
    {
        if (ok) w->busy.store(0);
    }
};

int dev_alloc(ss_weights* w, void** out, size_t bytes, bool zero)
{
    void* p = nullptr;
    hipError_t e = hipMalloc(&p, bytes);
    if (e != hipSuccess) return ss::fail(SS_ENOMEM, "hipMalloc(%zu bytes): %s", bytes, hipGetErrorString(e));
    w->allocs.push_back(p);
    if (zero) HIPCHK(hipMemset(p, 0, bytes));
    *out = p;
    return SS_OK;
}

// Uploads a row-major host matrix through a staging buffer and packs it into dst (Sec. of ss_internal.h
// on the operand layout).  Source row r -> packed row (r/16*blk_stride + blk_off)*16 + r%16.
int upload_pack(ss_weights* w, Buf& staging, const void* host, int src_f32, int n_src, int k, f16_t* dst, int kp,
                int blk_stride, int blk_off)
{
    const size_t bytes = (size_t)n_src * k * (src_f32 ? 4 : 2);
    if (int rc = staging.ensure(bytes, false)) return rc;
    HIPCHK(hipMemcpy(staging.p, host, bytes, hipMemcpyHostToDevice));
    ss::launch_pack_weight(staging.p, src_f32, dst, n_src, k, kp, blk_stride, blk_off, w->lane[0].stream);
    HIPCHK(hipStreamSynchronize(w->lane[0].stream));
    return SS_OK;
}

int upload_vec(ss_weights* w, Buf& staging, const void* host, int src_f32, size_t count, bf16_t** out)
{
    void* p = nullptr;
    if (int rc = dev_alloc(w, &p, count * 2, false)) return rc;
    const size_t bytes = count * (src_f32 ? 4 : 2);
    if (int rc = staging.ensure(bytes, false)) return rc;
    HIPCHK(hipMemcpy(staging.p, host, bytes, hipMemcpyHostToDevice));
    ss::launch_cast_rows(staging.p, src_f32, (bf16_t*)p, count, w->lane[0].stream);
    HIPCHK(hipStreamSynchronize(w->lane[0].stream));
    *out = (bf16_t*)p;
    return SS_OK;
}

int alloc_packed(ss_weights* w, PackedMat* m, int n, int k)
{
    m->N = n;
    m->K = k;
    m->Kp = ss::padded_k(k);
    void* p = nullptr;
    if (int rc = dev_alloc(w, &p, (size_t)n * m->Kp * 2, m->Kp != k)) return rc;
    m->p = (f16_t*)p;
    return SS_OK;
}

int check_cfg(const ss_model_cfg* c)
{
    if (!c) return ss::fail(SS_EINVAL, "cfg is NULL");
    if (c->n_layers < 1 || c->d_model < 64 || c->n_heads < 1 || c->d_ffn < 16 || c->vocab < 16)
        return ss::fail(SS_EINVAL, "non-positive model dimension");
    if (c->n_heads * c->head_dim != c->d_model) return ss::fail(SS_EINVAL, "n_heads*head_dim != d_model");
    if (c->head_dim != 64 && c->head_dim != 128) return ss::fail(SS_EINVAL, "head_dim must be 64 or 128");
    if (c->d_model % 64 || c->d_model > 8192) return ss::fail(SS_EINVAL, "d_model must be a multiple of 64, <= 8192");
    if (c->d_ffn % 16) return ss::fail(SS_EINVAL, "d_ffn must be a multiple of 16");
    if (c->vocab % 16) return ss::fail(SS_EINVAL, "vocab must be a multiple of 16");
    if (!(c->rope_base > 1.f) || !(c->rms_eps > 0.f)) return ss::fail(SS_EINVAL, "bad rope_base / rms_eps");
    return SS_OK;
}

// ---------------------------------------------------------------------------------------- workspace
// n_max token-rows in a forward, B micro-batch rows, n_sel rows whose logits are wanted,
// slots = total key/value slots of the micro-batch.
int ensure_workspace(const ss_weights* w, Lane& ln, int n_max, int B, int n_sel, size_t slots, int max_new, hipStream_t s)
{
    const ss_model_cfg& c = w->cfg;
    const int d = c.d_model, F = c.d_ffn, V = c.vocab;
    Workspace& ws = ln.ws;
    const size_t nr = (size_t)ss::round_up(n_max, 128);
    const size_t Bp = ss::round_up(B, 4), np = ss::round_up(n_max, 4), sp = ss::round_up(n_sel, 4);
    const size_t n_i32 = 4 + 3 * np + 5 * Bp + 2 * sp + (size_t)B * max_new;
    ln.kv_layer_stride = slots * d;
    // Partial-sum buffers hold [ksplit][rows][N] for whatever plan a forward over 1..n_max rows gets.
    // gate|up partial sums exist only when that projection runs with k-slices (never in the sweep kernel).
    struct Item { Buf* b; size_t bytes; bool zero; };
    const Item items[] = {
        {&ws.x, nr * d * 4, false},
        {&ws.h, nr * d * 2, true},
        {&ws.ao, nr * d * 2, true},
        {&ws.act, nr * ss::padded_k(F) * 2, true},
        {&ws.qrot, nr * d * 4, false},
        {&ws.pqkv, ss::gemm_partial_rows_bound(3 * d, n_max) * 3 * d * 4, false},
        {&ws.pd, ss::gemm_partial_rows_bound(d, n_max) * d * 4, false},
        {&ws.pgu, ss::gemm_partial_rows_bound(2 * F, n_max, true) * 2 * F * 4, false},
        {&ws.hsel, (size_t)ss::round_up(n_sel, 128) * d * 2, true},
        {&ws.logits, (size_t)ss::round_up(n_sel, 16) * V * 4, false},
        {&ws.kv, (size_t)c.n_layers * 2 * slots * d * 2, false},
        {&ws.ints, n_i32 * 4, false},
        {&ws.i64s, Bp * 8, false},
    };
    if (ws.arena) {
        // Carve the buffers out of the arena.  It keeps the last call's bytes in a different layout, so what
        // must read as zero (padding columns and rows of the packed activations) is cleared by a kernel.
        size_t at = 0;
        for (const Item& it : items) at += (it.bytes + 255) & ~(size_t)255;
        if (at > ws.arena_bytes)
            return ss::fail(SS_EINVAL, "this call needs %zu bytes of workspace; the static scratch array holds %zu", at,
                            ws.arena_bytes);
        at = 0;
        for (const Item& it : items) {
            it.b->p = ws.arena + at;
            it.b->bytes = it.bytes;
            it.b->borrowed = true;
            if (it.zero) ss::launch_fill_i32((int32_t*)it.b->p, 0, it.bytes / 4, s);
            at += (it.bytes + 255) & ~(size_t)255;
        }
    } else {
        for (const Item& it : items)
            if (int rc = it.b->ensure(it.bytes, it.zero)) return rc;
    }
    // int32 arena: d_n d_step d_nlive d_active | tr_tok tr_row tr_pos [n_max] | live_row plen j0 limit cap [B] | am sel [n_sel] | out_tok
    int32_t* q = ws.ints.as<int32_t>();
    MbState& st = ln.st;
    st.d_n = q; st.d_step = q + 1; st.d_nlive = q + 2; st.d_active = q + 3; q += 4;
    st.tr_tok = q; q += np;
    st.tr_row = q; q += np;
    st.tr_pos = q; q += np;
    st.live_row = q; q += Bp;
    st.row_plen = q; q += Bp;
    st.row_j0 = q; q += Bp;
    st.row_limit = q; q += Bp;
    st.row_cap = q; q += Bp;
    st.am = q; q += sp;
    ln.d_sel = q; q += sp;
    st.out_tok = q;
    st.max_new = max_new;
    st.row_so = ws.i64s.as<int64_t>();
    return SS_OK;
}

// Launch plans of the five projections of a forward over n token-rows with n_sel logit rows.
struct Plans {
    ss::GemmPlan qkv, o, gu, down, lm;
};

Plans make_plans(const ss_weights* w, int n, int n_sel)
{
    const ss_model_cfg& c = w->cfg;
    const int d = c.d_model, F = c.d_ffn, V = c.vocab, Fp = ss::padded_k(F), cu = w->n_cu;
    Plans p;
    p.qkv = ss::gemm_plan(3 * d, d, n, ss::EPI_PARTIAL, cu);
    p.o = ss::gemm_plan(d, d, n, ss::EPI_PARTIAL, cu);
    p.gu = ss::gemm_plan(2 * F, d, n, ss::EPI_SWIGLU, cu);
    p.down = ss::gemm_plan(d, Fp, n, ss::EPI_PARTIAL, cu);
    p.lm = ss::gemm_plan(V, d, n_sel, ss::EPI_PARTIAL, cu, 1);   // logits are read directly: no k-slices
    return p;
}

GemmArgs gemm_args(const ss_weights* w, const f16_t* W, const f16_t* X, float* out, f16_t* outp, int N, int Kp, int rows,
                   int kp_out, const ss::GemmPlan& p)
{
    GemmArgs g{};
    g.W = W; g.X = X; g.out = out; g.out_packed = outp; g.N = N; g.Kp = Kp;
    g.m_rows = rows; g.m_stride = rows; g.kp_out = kp_out; g.ksplit = p.ksplit; g.nb = p.nb; g.kd = p.kd;
    g.kp = p.kp; g.tms = p.tms; g.sweep_p = p.sweep_p; g.sweep_gn = p.sweep_gn; g.sweep_kh = p.sweep_kh; g.zero_blk = w->zero_blk;
    return g;
}

// ---------------------------------------------------------------------------------------- one forward
// Runs the decoder over the token-rows described by the device state (st.d_n of them, at most n of
// them: n sizes the grids and picks the kernel variants).  Logits are produced for n_sel rows:
// the rows listed in d_sel, or the first *d_nsel rows when d_sel is null.  Ends with the token choice:
// the argmax, or a draw from the softmax when the lane carries a temperature (cur_inv_temp).
void forward(const ss_weights* w, Lane& ln, int n, int n_sel, const int32_t* d_sel, const int32_t* d_nsel, bool decode, hipStream_t s)
{
    const ss_model_cfg& c = w->cfg;
    const int d = c.d_model, H = c.n_heads, hd = c.head_dim, F = c.d_ffn, V = c.vocab;
    Workspace& ws = ln.ws;
    const MbState& st = ln.st;
    float* x = ws.x.as<float>();
    f16_t *h = ws.h.as<f16_t>(), *ao = ws.ao.as<f16_t>(), *act = ws.act.as<f16_t>();
    float* qrot = ws.qrot.as<float>();
    float* pqkv = ws.pqkv.as<float>();
    float* pd = ws.pd.as<float>();
    const int Fp = ss::padded_k(F);

    const Plans pl = make_plans(w, n, n_sel);
    const ss::GemmPlan &p_qkv = pl.qkv, &p_o = pl.o, &p_gu = pl.gu, &p_d = pl.down, &p_lm = pl.lm;
    const int ks_qkv = p_qkv.ksplit, ks_o = p_o.ksplit, ks_d = p_d.ksplit;
    const size_t st_qkv = (size_t)n * 3 * d, st_d = (size_t)n * d;
    auto mk = [w](const f16_t* W, const f16_t* X, float* out, f16_t* outp, int N, int Kp, int rows, int kp_out,
                  const ss::GemmPlan& p) { return gemm_args(w, W, X, out, outp, N, Kp, rows, kp_out, p); };

    ss::launch_embed(st, w->embed, x, d, n, s);
    for (int l = 0; l < c.n_layers; ++l) {
        const Layer& L = w->layers[l];
        ss::kv_t* kc = ws.kv.as<ss::kv_t>() + (size_t)l * 2 * ln.kv_layer_stride;
        ss::kv_t* vc = kc + ln.kv_layer_stride;
        ss::launch_rmsnorm(st, x, l ? pd : nullptr, ks_d, st_d, L.attn_norm, c.rms_eps, nullptr, nullptr, h, d, n, s);
        ss::launch_gemm(mk(L.wqkv.p, h, pqkv, nullptr, 3 * d, d, n, 0, p_qkv), ss::EPI_PARTIAL, s);
        if (decode) {   // one token-row per row: rotation and append are fused into the attention kernel
            ss::launch_attention_decode(st, pqkv, ks_qkv, st_qkv, kc, vc, w->rope_cos, w->rope_sin, ao, d, H, hd, n, s);
        } else {        // prompt: every key of a row must be in place before any of its queries attends
            ss::launch_rope_append(st, pqkv, ks_qkv, st_qkv, qrot, kc, vc, w->rope_cos, w->rope_sin, d, H, hd, n, s);
            ss::launch_attention_prompt(st, qrot, kc, vc, ao, d, H, hd, ln.prompt_rows, ln.prompt_max_len, s);
        }
        ss::launch_gemm(mk(L.wo.p, ao, pd, nullptr, d, d, n, 0, p_o), ss::EPI_PARTIAL, s);
        ss::launch_rmsnorm(st, x, pd, ks_o, st_d, L.mlp_norm, c.rms_eps, nullptr, nullptr, h, d, n, s);
        if (p_gu.ksplit == 1) {
            ss::launch_gemm(mk(L.wgu.p, h, nullptr, act, 2 * F, d, n, Fp, p_gu), ss::EPI_SWIGLU, s);
        } else {   // k-sliced: partial sums, then one small kernel adds them and applies SwiGLU
            ss::launch_gemm(mk(L.wgu.p, h, ws.pgu.as<float>(), nullptr, 2 * F, d, n, 0, p_gu), ss::EPI_PARTIAL, s);
            ss::launch_swiglu_reduce(ws.pgu.as<float>(), p_gu.ksplit, (size_t)n * 2 * F, n, F, Fp, act, s);
        }
        ss::launch_gemm(mk(L.wd.p, act, pd, nullptr, d, Fp, n, 0, p_d), ss::EPI_PARTIAL, s);
    }
    f16_t* hsel = ws.hsel.as<f16_t>();
    ss::launch_rmsnorm(st, x, pd, ks_d, st_d, w->final_norm, c.rms_eps, d_sel, d_nsel, hsel, d, n_sel, s);
    ss::launch_gemm(mk(w->lm_head.p, hsel, ws.logits.as<float>(), nullptr, V, d, n_sel, 0, p_lm), ss::EPI_PARTIAL, s);
    if (ln.cur_inv_temp > 0.f)
        ss::launch_sample(ws.logits.as<float>(), V, d_nsel ? d_nsel : st.d_n, st, ln.cur_draws, ln.cur_ids, ln.cur_seed,
                          ln.cur_inv_temp, n_sel, s);
    else
        ss::launch_argmax(ws.logits.as<float>(), V, d_nsel ? d_nsel : st.d_n, st.am, n_sel, s);
}

int check_prompts(const ss_weights* w, const int32_t* toks, const int32_t* offs, int B)
{
    if (!w) return ss::fail(SS_EINVAL, "weights handle is NULL");
    if (B <= 0) return ss::fail(SS_EINVAL, "B must be > 0");
    if (B > ss::kMaxBatch) return ss::fail(SS_EINVAL, "B = %d exceeds %d rows", B, ss::kMaxBatch);
    if (!toks || !offs) return ss::fail(SS_EINVAL, "NULL prompt arrays");
    if (offs[0] != 0) return ss::fail(SS_EINVAL, "prompt_offsets[0] must be 0");
    for (int i = 0; i < B; ++i)
        if (offs[i + 1] <= offs[i]) return ss::fail(SS_EINVAL, "empty prompt or non-monotone offsets at row %d", i);
    for (int t = 0; t < offs[B]; ++t)
        if (toks[t] < 0 || toks[t] >= w->cfg.vocab) return ss::fail(SS_EINVAL, "token id %d out of range", toks[t]);
    return SS_OK;
}

struct Upload {
    std::vector<int32_t> v;
    hipStream_t s;
    int put(int32_t* dst, const int32_t* src, size_t n)
    {
        HIPCHK(hipMemcpyAsync(dst, src, n * 4, hipMemcpyHostToDevice, s));
        return SS_OK;
    }
};

// Uploads the state of a prompt forward: token-rows are the concatenated prompt positions.
//   lens[i]   tokens of row i processed by this forward (positions 0..lens[i]-1)
//   slab[i]   key/value slots reserved for row i
int upload_prompt_state(Lane& ln, const int32_t* toks, const int32_t* offs, const int32_t* lens, int B,
                        const int32_t* slab, const int32_t* limit, const std::vector<int32_t>& sel, hipStream_t s)
{
    const MbState& st = ln.st;
    int n = 0;
    for (int i = 0; i < B; ++i) n += lens[i];
    std::vector<int32_t> tok(n), row(n), pos(n), live(B), plen(B), first(B);
    std::vector<int64_t> so(B);
    int at = 0;
    int64_t slot = 0;
    for (int i = 0; i < B; ++i) {
        first[i] = at;
        for (int t = 0; t < lens[i]; ++t, ++at) {
            tok[at] = toks[offs[i] + t];
            row[at] = i;
            pos[at] = t;
        }
        live[i] = i;
        plen[i] = lens[i];
        so[i] = slot;
        slot += slab[i];
    }
    const int32_t hdr[4] = {n, 0, B, B};
    HIPCHK(hipMemcpyAsync(st.d_n, hdr, 16, hipMemcpyHostToDevice, s));
    HIPCHK(hipMemcpyAsync(st.tr_tok, tok.data(), (size_t)n * 4, hipMemcpyHostToDevice, s));
    HIPCHK(hipMemcpyAsync(st.tr_row, row.data(), (size_t)n * 4, hipMemcpyHostToDevice, s));
    HIPCHK(hipMemcpyAsync(st.tr_pos, pos.data(), (size_t)n * 4, hipMemcpyHostToDevice, s));
    HIPCHK(hipMemcpyAsync(st.live_row, live.data(), (size_t)B * 4, hipMemcpyHostToDevice, s));
    HIPCHK(hipMemcpyAsync(st.row_plen, plen.data(), (size_t)B * 4, hipMemcpyHostToDevice, s));
    HIPCHK(hipMemcpyAsync(st.row_j0, first.data(), (size_t)B * 4, hipMemcpyHostToDevice, s));
    ln.prompt_rows = B;
    ln.prompt_max_len = *std::max_element(plen.begin(), plen.end());
    HIPCHK(hipMemcpyAsync(st.row_limit, limit, (size_t)B * 4, hipMemcpyHostToDevice, s));
    HIPCHK(hipMemcpyAsync(st.row_cap, slab, (size_t)B * 4, hipMemcpyHostToDevice, s));
    HIPCHK(hipMemcpyAsync(st.row_so, so.data(), (size_t)B * 8, hipMemcpyHostToDevice, s));
    if (!sel.empty()) HIPCHK(hipMemcpyAsync(ln.d_sel, sel.data(), sel.size() * 4, hipMemcpyHostToDevice, s));
    HIPCHK(hipStreamSynchronize(s));   // the host vectors above die with this frame
    return SS_OK;
}

int check_gen_opts(const ss_weights* w, const ss_gen_opts* g, int rows, int need_stride)
{
    if (!g) return ss::fail(SS_EINVAL, "opts is NULL");
    if (g->eos_id < -1 || g->eos_id >= w->cfg.vocab) return ss::fail(SS_EINVAL, "eos_id outside [-1, vocab)");
    if (!(g->temperature >= 0.f) || !std::isfinite(g->temperature))
        return ss::fail(SS_EINVAL, "temperature must be finite and >= 0");
    if (g->sync_every < 1) return ss::fail(SS_EINVAL, "sync_every must be >= 1");
    if (g->temperature > 0.f && g->draws) {
        if (g->draws_stride < need_stride)
            return ss::fail(SS_EINVAL, "draws_stride %d < %d", g->draws_stride, need_stride);
        for (int i = 0; i < rows; ++i)
            for (int t = 0; t < need_stride; ++t) {
                const float u = g->draws[(size_t)i * g->draws_stride + t];
                if (!(u >= 0.f && u < 1.f)) return ss::fail(SS_EINVAL, "draw [%d][%d] outside [0,1)", i, t);
            }
    }
    if (g->draw_ids)
        for (int i = 0; i < rows; ++i)
            if (g->draw_ids[i] < 0) return ss::fail(SS_EINVAL, "draw_ids[%d] < 0", i);
    if (g->target_lens)
        for (int i = 0; i < rows; ++i)
            if (g->target_lens[i] < 1) return ss::fail(SS_EINVAL, "target_lens[%d] < 1", i);
    return SS_OK;
}

// iters + 1 HIP events that are destroyed however the call ends.
struct EventList {
    std::vector<hipEvent_t> e;
    int create(int count)
    {
        e.assign((size_t)count, nullptr);
        for (auto& x : e) HIPCHK(hipEventCreate(&x));
        return SS_OK;
    }
    ~EventList()
    {
        for (auto& x : e)
            if (x) (void)hipEventDestroy(x);
    }
};

// Clears the handle's token-choice state however the call ends.
struct ChoiceGuard {
    Lane& ln;
    ~ChoiceGuard()
    {
        ln.cur_draws = nullptr;
        ln.cur_ids = nullptr;
        ln.cur_seed = 0;
        ln.cur_inv_temp = 0.f;
    }
};

// One micro-batch.  gen == nullptr: greedy, rows end at target_lens (known to the host, which therefore
// knows the number of forwards and the live rows of each).  gen != nullptr: token choice and row ends per
// gen (checked by the caller), target_lens ignored; the host learns how many rows are left by polling.
int decode_microbatch_impl(const ss_weights* w, Lane& ln, const int32_t* prompt_tokens, const int32_t* prompt_offsets, int32_t B,
                           int32_t max_new, const int32_t* target_lens, const ss_gen_opts* gen, uint32_t flags,
                           int32_t* out_tokens, int32_t* out_lens, uint8_t* out_failed, ss_stats* stats, hipStream_t s)
{
    if (int rc = check_prompts(w, prompt_tokens, prompt_offsets, B)) return rc;
    if (max_new < 1) return ss::fail(SS_EINVAL, "max_new must be >= 1");
    if (!out_tokens || !out_lens || !out_failed) return ss::fail(SS_EINVAL, "NULL argument");
    if (!gen && !target_lens) return ss::fail(SS_EINVAL, "NULL argument");
    if (flags & ~SS_COMPACT) return ss::fail(SS_EINVAL, "unknown flag");
    const int32_t* tl = gen ? gen->target_lens : target_lens;
    std::vector<int32_t> lens(B), slab(B), limit(B), sel(B);
    int n_prompt = prompt_offsets[B], steps = 0;
    size_t slots = 0;
    for (int i = 0; i < B; ++i) {
        if (tl && tl[i] < 1) return ss::fail(SS_EINVAL, "target_lens[%d] < 1", i);
        lens[i] = prompt_offsets[i + 1] - prompt_offsets[i];
        if (lens[i] + max_new > ss::kMaxPos)
            return ss::fail(SS_EINVAL, "row %d: prompt %d + max_new %d exceeds %d positions", i, lens[i], max_new,
                            ss::kMaxPos);
        slab[i] = lens[i] + max_new;
        slots += (size_t)slab[i];
        limit[i] = tl ? std::min(tl[i], max_new) : max_new;
        steps = std::max(steps, limit[i]);
        sel[i] = prompt_offsets[i + 1] - 1;
    }
    HIPCHK(hipSetDevice(w->device));
    if (int rc = ensure_workspace(w, ln, std::max(n_prompt, B), B, B, slots, max_new, s)) return rc;
    const MbState& st = ln.st;
    const int compact = (flags & SS_COMPACT) ? 1 : 0;
    const int eos_id = gen ? gen->eos_id : -1;

    if (int rc = upload_prompt_state(ln, prompt_tokens, prompt_offsets, lens.data(), B, slab.data(), limit.data(), sel, s))
        return rc;
    ChoiceGuard choice{ln};
    if (gen && gen->temperature > 0.f) {
        if (gen->draws) {
            if (int rc = ln.ws.draws.ensure((size_t)B * max_new * 4, false)) return rc;
            HIPCHK(hipMemcpy2DAsync(ln.ws.draws.p, (size_t)max_new * 4, gen->draws, (size_t)gen->draws_stride * 4,
                                    (size_t)max_new * 4, B, hipMemcpyHostToDevice, s));
            HIPCHK(hipStreamSynchronize(s));
            ln.cur_draws = ln.ws.draws.as<float>();
        } else {   // generated on the device from (seed, row id, token number)
            std::vector<int32_t> ids(B);
            for (int i = 0; i < B; ++i) ids[i] = gen->draw_ids ? gen->draw_ids[i] : i;
            if (int rc = ln.ws.draws.ensure((size_t)B * 4, false)) return rc;
            HIPCHK(hipMemcpyAsync(ln.ws.draws.p, ids.data(), (size_t)B * 4, hipMemcpyHostToDevice, s));
            HIPCHK(hipStreamSynchronize(s));
            ln.cur_ids = ln.ws.draws.as<int32_t>();
            ln.cur_seed = gen->seed;
        }
        ln.cur_inv_temp = 1.f / gen->temperature;
    }
    ss::launch_fill_i32(st.out_tok, -1, (size_t)B * max_new, s);

    const hipEvent_t e0 = ln.ev[0], e1 = ln.ev[1], e2 = ln.ev[2];   // created with the handle: nothing is created per call
    HIPCHK(hipEventRecord(e0, s));
    forward(w, ln, n_prompt, B, ln.d_sel, st.d_nlive, false, s);
    ss::launch_step_update(st, compact, eos_id, s);
    HIPCHK(hipEventRecord(e1, s));

    int64_t row_steps = B, kv_tokens = 0;
    int forwards = 1, polls = 0;
    if (!gen) {
        std::vector<int32_t> sorted_limit(limit);
        std::sort(sorted_limit.begin(), sorted_limit.end());
        for (int g = 1; g < steps; ++g) {
            // rows alive for forward g: all of them, or with compaction those that owe more than g tokens
            int n_live = B;
            if (compact)
                n_live = (int)(sorted_limit.end() - std::upper_bound(sorted_limit.begin(), sorted_limit.end(), g));
            forward(w, ln, n_live, n_live, nullptr, nullptr, true, s);
            ss::launch_step_update(st, compact, eos_id, s);
            row_steps += n_live;
        }
        forwards = steps;
    } else {
        // The device ends rows and shrinks the live batch by itself; the host sizes the launches by the last
        // count it has read (an upper bound: the kernels take the true count from device memory) and stops
        // when a read shows no unfinished row.
        auto poll = [&](int* n_live, int* active) -> int {
            HIPCHK(hipMemcpyAsync(ln.h_poll, st.d_n, 16, hipMemcpyDeviceToHost, s));
            HIPCHK(hipStreamSynchronize(s));
            ++polls;
            if (compact) *n_live = ln.h_poll[2];
            *active = ln.h_poll[3];
            return SS_OK;
        };
        int n_live = B, active = B;
        if (int rc = poll(&n_live, &active)) return rc;
        for (int g = 1; g < max_new && active > 0; ++g) {
            forward(w, ln, n_live, n_live, nullptr, nullptr, true, s);
            ss::launch_step_update(st, compact, eos_id, s);
            row_steps += n_live;
            ++forwards;
            if (g % gen->sync_every == 0 && g + 1 < max_new)
                if (int rc = poll(&n_live, &active)) return rc;
        }
    }
    HIPCHK(hipEventRecord(e2, s));
    HIPCHK(hipMemcpyAsync(out_tokens, st.out_tok, (size_t)B * max_new * 4, hipMemcpyDeviceToHost, s));
    if (gen) HIPCHK(hipMemcpyAsync(limit.data(), st.row_limit, (size_t)B * 4, hipMemcpyDeviceToHost, s));
    HIPCHK(hipStreamSynchronize(s));
    HIPCHK(hipGetLastError());
    int longest = 0;
    for (int i = 0; i < B; ++i) {
        out_lens[i] = limit[i];
        longest = std::max(longest, limit[i]);
        if (!gen) {
            out_failed[i] = target_lens[i] > max_new;
        } else {   // unfinished: ran into the cap without its end id and short of its simulated end
            const bool hit_cap = limit[i] == max_new;
            const bool ended = out_tokens[(size_t)i * max_new + limit[i] - 1] == eos_id || (tl && tl[i] <= max_new);
            out_failed[i] = hit_cap && !ended;
        }
    }
    if (stats) {
        for (int g = 1; g < forwards; ++g)
            for (int i = 0; i < B; ++i)
                if (!compact || limit[i] > g) kv_tokens += lens[i] + g;
        float ms01 = 0.f, ms12 = 0.f;
        HIPCHK(hipEventElapsedTime(&ms01, e0, e1));
        HIPCHK(hipEventElapsedTime(&ms12, e1, e2));
        stats->steps = forwards;
        stats->rows = B;
        stats->row_steps = row_steps;
        stats->prompt_tokens = n_prompt;
        stats->decode_kv_tokens = kv_tokens;
        stats->prefill_ms = ms01;
        stats->decode_ms = ms12;
        stats->polls = polls;
        stats->idle_steps = forwards - longest;
    }
    return SS_OK;
}

// Fills a fresh handle: streams and events of every lane, the packed weights, the rotary tables.  Whatever it
// has created when it fails (or throws) is released by the caller through ss_weights_destroy.
int weights_create_impl(ss_weights* w, const void* const* tensors, int32_t src_dtype)
{
    const ss_model_cfg* cfg = &w->cfg;
    if (hipGetDevice(&w->device) != hipSuccess) return ss::fail(SS_EDEVICE, "hipGetDevice failed");
    if (int rc_s = scratch_address(w->device, &w->scratch_ptr)) return rc_s;
    for (Lane& ln : w->lane) {
        if (hipStreamCreate(&ln.stream) != hipSuccess) return ss::fail(SS_EDEVICE, "hipStreamCreate failed");
        if (hipHostMalloc((void**)&ln.h_poll, 16, hipHostMallocDefault) != hipSuccess)
            return ss::fail(SS_ENOMEM, "hipHostMalloc failed");
        for (auto& e : ln.ev)
            if (hipEventCreate(&e) != hipSuccess) return ss::fail(SS_EDEVICE, "hipEventCreate failed");
    }

    const int d = cfg->d_model, F = cfg->d_ffn, V = cfg->vocab, f32 = (src_dtype == SS_F32);
    struct Staging {   // the upload buffer goes however the function ends
        Buf b;
        ~Staging() { b.release(); }
    } staging_owner;
    Buf& staging = staging_owner.b;
    int rc = SS_OK;
    int ti = 0;
    if ((rc = upload_vec(w, staging, tensors[ti++], f32, (size_t)V * d, &w->embed))) return rc;
    w->layers.resize(cfg->n_layers);
    for (int l = 0; l < cfg->n_layers; ++l) {
        Layer& L = w->layers[l];
        if ((rc = upload_vec(w, staging, tensors[ti++], f32, d, &L.attn_norm))) return rc;
        if ((rc = alloc_packed(w, &L.wqkv, 3 * d, d))) return rc;
        for (int part = 0; part < 3; ++part)   // q, k, v stacked along the output dimension
            if ((rc = upload_pack(w, staging, tensors[ti++], f32, d, d, L.wqkv.p, L.wqkv.Kp, 1, part * d / 16)))
                return rc;
        if ((rc = alloc_packed(w, &L.wo, d, d))) return rc;
        if ((rc = upload_pack(w, staging, tensors[ti++], f32, d, d, L.wo.p, L.wo.Kp, 1, 0))) return rc;
        if ((rc = upload_vec(w, staging, tensors[ti++], f32, d, &L.mlp_norm))) return rc;
        if ((rc = alloc_packed(w, &L.wgu, 2 * F, d))) return rc;
        for (int part = 0; part < 2; ++part)   // gate and up strips interleaved: strip 2j = gate, 2j+1 = up
            if ((rc = upload_pack(w, staging, tensors[ti++], f32, F, d, L.wgu.p, L.wgu.Kp, 2, part))) return rc;
        if ((rc = alloc_packed(w, &L.wd, d, F))) return rc;
        if ((rc = upload_pack(w, staging, tensors[ti++], f32, d, F, L.wd.p, L.wd.Kp, 1, 0))) return rc;
    }
    if ((rc = upload_vec(w, staging, tensors[ti++], f32, d, &w->final_norm))) return rc;
    if ((rc = alloc_packed(w, &w->lm_head, V, d))) return rc;
    if ((rc = upload_pack(w, staging, tensors[ti++], f32, V, d, w->lm_head.p, w->lm_head.Kp, 1, 0))) return rc;

    // rotary tables: cos/sin(pos * base^(-2e/hd)) evaluated in double, stored as fp32 [pos][e]
    const int half = cfg->head_dim / 2;
    std::vector<float> tc((size_t)ss::kMaxPos * half), tsn((size_t)ss::kMaxPos * half);
    for (int e = 0; e < half; ++e) {
        const double inv = std::pow((double)cfg->rope_base, -2.0 * e / (double)cfg->head_dim);
        for (int p = 0; p < ss::kMaxPos; ++p) {
            tc[(size_t)p * half + e] = (float)std::cos(p * inv);
            tsn[(size_t)p * half + e] = (float)std::sin(p * inv);
        }
    }
    void* p = nullptr;
    if ((rc = dev_alloc(w, &p, 1024, true))) return rc;
    w->zero_blk = (f16_t*)p;
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, w->device) != hipSuccess || prop.multiProcessorCount <= 0)
        return ss::fail(SS_EDEVICE, "cannot read the device's compute unit count");
    w->n_cu = prop.multiProcessorCount;
    if ((rc = dev_alloc(w, &p, tc.size() * 4, false))) return rc;
    w->rope_cos = (float*)p;
    if ((rc = dev_alloc(w, &p, tsn.size() * 4, false))) return rc;
    w->rope_sin = (float*)p;
    if (hipMemcpy(w->rope_cos, tc.data(), tc.size() * 4, hipMemcpyHostToDevice) != hipSuccess ||
        hipMemcpy(w->rope_sin, tsn.data(), tsn.size() * 4, hipMemcpyHostToDevice) != hipSuccess)
        return ss::fail(SS_EDEVICE, "rotary table upload failed");
    return SS_OK;
}

}  // namespace

// ============================================================================================ C ABI
// No entry point lets a C++ exception out: host allocations that fail are reported as SS_ENOMEM (ss::no_throw).
extern "C" int ss_weights_create(const ss_model_cfg* cfg, const void* const* tensors, int32_t src_dtype,
                                 ss_weights** out)
{
    ss::clear_error();
    if (!out || !tensors) return ss::fail(SS_EINVAL, "NULL argument");
    if (int rc = check_cfg(cfg)) return rc;
    if (src_dtype != SS_BF16 && src_dtype != SS_F32) return ss::fail(SS_EINVAL, "unknown src_dtype");
    const int nt = 3 + 9 * cfg->n_layers;
    for (int i = 0; i < nt; ++i)
        if (!tensors[i]) return ss::fail(SS_EINVAL, "tensors[%d] is NULL", i);
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || ndev < 1) return ss::fail(SS_EDEVICE, "no HIP device available");

    ss_weights* w = new (std::nothrow) ss_weights();
    if (!w) return ss::fail(SS_ENOMEM, "host allocation failed");
    w->cfg = *cfg;
    const int rc = ss::no_throw([&] { return weights_create_impl(w, tensors, src_dtype); });
    if (rc != SS_OK) {
        ss_weights_destroy(w);
        return rc;
    }
    *out = w;
    return SS_OK;
}

extern "C" int ss_set_option(ss_weights* w, int32_t option, int32_t value)
{
    ss::clear_error();
    if (!w) return ss::fail(SS_EINVAL, "weights handle is NULL");
    BusyGuard guard(w);
    if (!guard.ok) return ss::fail(SS_ESTATE, "another call is in flight on this handle");
    if (option == SS_OPT_IN_FLIGHT) {
        if (value < 1 || value > kLanes) return ss::fail(SS_EINVAL, "SS_OPT_IN_FLIGHT takes 1 to %d", kLanes);
        w->in_flight = value;
        return SS_OK;
    }
    return ss::fail(SS_EINVAL, "unknown option %d", option);
}

extern "C" void ss_set_gemm_mode(int32_t mode)
{
    if (mode >= 0 && mode <= 14 && (mode & 3) != 3) ss::set_gemm_mode(mode);
}

extern "C" void ss_weights_destroy(ss_weights* w)
{
    if (!w) return;
    (void)hipSetDevice(w->device);
    for (Lane& ln : w->lane) {
        if (ln.stream) (void)hipStreamSynchronize(ln.stream);
        ln.ws.release();
        if (ln.stream) (void)hipStreamDestroy(ln.stream);
        if (ln.h_poll) (void)hipHostFree(ln.h_poll);
        for (auto& e : ln.ev)
            if (e) (void)hipEventDestroy(e);
    }
    for (void* p : w->allocs) (void)hipFree(p);
    delete w;
}

extern "C" int ss_decode_microbatch(ss_weights* w, const int32_t* prompt_tokens, const int32_t* prompt_offsets,
                                    int32_t B, int32_t max_new, const int32_t* target_lens, uint32_t flags,
                                    int32_t* out_tokens, int32_t* out_lens, uint8_t* out_failed, ss_stats* stats,
                                    void* hip_stream)
{
    ss::clear_error();
    if (!w) return ss::fail(SS_EINVAL, "weights handle is NULL");
    BusyGuard guard(w);
    if (!guard.ok) return ss::fail(SS_ESTATE, "another call is in flight on this handle");
    Lane& ln = w->lane[0];
    hipStream_t s = hip_stream ? (hipStream_t)hip_stream : ln.stream;
    return ss::no_throw([&] {
        return decode_microbatch_impl(w, ln, prompt_tokens, prompt_offsets, B, max_new, target_lens, nullptr, flags,
                                      out_tokens, out_lens, out_failed, stats, s);
    });
}

extern "C" int ss_decode_microbatch_static(ss_weights* w, const int32_t* prompt_tokens, const int32_t* prompt_offsets,
                                           int32_t B, int32_t max_new, const int32_t* target_lens, uint32_t flags,
                                           int32_t* out_tokens, int32_t* out_lens, uint8_t* out_failed,
                                           ss_stats* stats, void* hip_stream)
{
    ss::clear_error();
    if (!w) return ss::fail(SS_EINVAL, "weights handle is NULL");
    BusyGuard guard(w);
    if (!guard.ok) return ss::fail(SS_ESTATE, "another call is in flight on this handle");
    if (!w->scratch_ptr) return ss::fail(SS_ESTATE, "the static scratch array was not located on this device");
    // every static call on a GPU shares that GPU's array: overlapping calls (other handles) are refused
    struct ScratchGuard {
        std::atomic<int>& f;
        bool ok;
        explicit ScratchGuard(std::atomic<int>& f_) : f(f_), ok(f_.exchange(1) == 0) {}
        ~ScratchGuard()
        {
            if (ok) f.store(0);
        }
    } sg(g_scratch_busy[w->device]);
    if (!sg.ok) return ss::fail(SS_ESTATE, "another static call is using this GPU's scratch array");
    Lane& ln = w->lane[0];
    hipStream_t s = hip_stream ? (hipStream_t)hip_stream : ln.stream;
    // The handle's own (allocated, growable) workspace steps aside for the call; every buffer is a view into the
    // scratch array instead.  decode_microbatch_impl allocates nothing else on the device: its events belong to
    // the handle, its host staging lives on the host heap.
    struct View {   // swaps the lane's workspace for the view, and back however the call ends
        Lane& ln;
        Workspace ws;
        explicit View(Lane& l) : ln(l) {}
        void in() { std::swap(ln.ws, ws); }
        ~View()
        {
            std::swap(ln.ws, ws);
            ln.st = MbState{};   // pointed into the scratch array; the next call lays its own state out
        }
    } view(ln);
    view.ws.arena = (char*)w->scratch_ptr;
    view.ws.arena_bytes = kStaticScratchBytes;
    view.in();
    return ss::no_throw([&] {
        return decode_microbatch_impl(w, ln, prompt_tokens, prompt_offsets, B, max_new, target_lens, nullptr, flags,
                                      out_tokens, out_lens, out_failed, stats, s);
    });
}

extern "C" int ss_generate_microbatch(ss_weights* w, const int32_t* prompt_tokens, const int32_t* prompt_offsets,
                                      int32_t B, int32_t max_new, const ss_gen_opts* opts, uint32_t flags,
                                      int32_t* out_tokens, int32_t* out_lens, uint8_t* out_failed, ss_stats* stats,
                                      void* hip_stream)
{
    ss::clear_error();
    if (!w) return ss::fail(SS_EINVAL, "weights handle is NULL");
    if (B <= 0 || B > ss::kMaxBatch) return ss::fail(SS_EINVAL, "B = %d outside [1, %d]", B, ss::kMaxBatch);
    if (max_new < 1) return ss::fail(SS_EINVAL, "max_new must be >= 1");
    if (int rc = check_gen_opts(w, opts, B, max_new)) return rc;
    BusyGuard guard(w);
    if (!guard.ok) return ss::fail(SS_ESTATE, "another call is in flight on this handle");
    Lane& ln = w->lane[0];
    hipStream_t s = hip_stream ? (hipStream_t)hip_stream : ln.stream;
    return ss::no_throw([&] {
        return decode_microbatch_impl(w, ln, prompt_tokens, prompt_offsets, B, max_new, nullptr, opts, flags, out_tokens,
                                      out_lens, out_failed, stats, s);
    });
}

namespace {

int forward_logits_impl(const ss_weights* w, Lane& ln, hipStream_t s, const int32_t* tokens, const int32_t* offsets,
                        int32_t B, const int32_t* n_prompt, int32_t all_prompt_logits, float* logits_out)
{
    const int V = w->cfg.vocab;
    std::vector<int32_t> len(B), slab(B), limit(B, 1), np(n_prompt, n_prompt + B), sel;
    std::vector<size_t> out_base(B);
    int n_p = 0, max_extra = 0;
    size_t slots = 0, out_rows = 0;
    for (int i = 0; i < B; ++i) {
        len[i] = offsets[i + 1] - offsets[i];
        if (len[i] > ss::kMaxPos) return ss::fail(SS_EINVAL, "row %d longer than %d positions", i, ss::kMaxPos);
        if (np[i] < 1 || np[i] > len[i]) return ss::fail(SS_EINVAL, "n_prompt[%d] out of range", i);
        if (all_prompt_logits && np[i] != len[i]) return ss::fail(SS_EINVAL, "all_prompt_logits needs n_prompt == len");
        slab[i] = len[i];
        slots += (size_t)len[i];
        out_base[i] = out_rows;
        if (all_prompt_logits) {
            for (int t = 0; t < len[i]; ++t) sel.push_back(n_p + t);
            out_rows += (size_t)len[i];
        } else {
            sel.push_back(n_p + np[i] - 1);
            out_rows += (size_t)(len[i] - np[i] + 1);
        }
        n_p += np[i];
        max_extra = std::max(max_extra, len[i] - np[i]);
    }
    const int n_sel = (int)sel.size();
    HIPCHK(hipSetDevice(w->device));
    if (int rc = ensure_workspace(w, ln, std::max(n_p, B), B, std::max(n_sel, B), slots, 1, s)) return rc;
    const MbState& st = ln.st;
    // prompt forward over the first n_prompt[i] tokens of every row
    std::vector<int32_t> ptoks, poffs(B + 1, 0);
    for (int i = 0; i < B; ++i) {
        ptoks.insert(ptoks.end(), tokens + offsets[i], tokens + offsets[i] + np[i]);
        poffs[i + 1] = (int32_t)ptoks.size();
    }
    if (int rc = upload_prompt_state(ln, ptoks.data(), poffs.data(), np.data(), B, slab.data(), limit.data(), sel, s))
        return rc;
    const int32_t nsel32 = n_sel;
    HIPCHK(hipMemcpyAsync(st.d_nlive, &nsel32, 4, hipMemcpyHostToDevice, s));
    forward(w, ln, n_p, n_sel, ln.d_sel, st.d_nlive, false, s);
    std::vector<float> lg((size_t)std::max(n_sel, B) * V);
    HIPCHK(hipMemcpyAsync(lg.data(), ln.ws.logits.p, (size_t)n_sel * V * 4, hipMemcpyDeviceToHost, s));
    HIPCHK(hipStreamSynchronize(s));
    if (all_prompt_logits) {
        std::memcpy(logits_out, lg.data(), (size_t)n_sel * V * 4);
    } else {
        for (int i = 0; i < B; ++i) std::memcpy(logits_out + out_base[i] * V, lg.data() + (size_t)i * V, (size_t)V * 4);
    }
    // decode steps: rows that still have a forced token feed it at their next position
    for (int g = 1; g <= max_extra; ++g) {
        std::vector<int32_t> tok, row, pos;
        for (int i = 0; i < B; ++i)
            if (len[i] - np[i] >= g) {
                tok.push_back(tokens[offsets[i] + np[i] + g - 1]);
                row.push_back(i);
                pos.push_back(np[i] + g - 1);
            }
        const int n = (int)tok.size();
        const int32_t n32 = n;
        HIPCHK(hipMemcpyAsync(st.d_n, &n32, 4, hipMemcpyHostToDevice, s));
        HIPCHK(hipMemcpyAsync(st.tr_tok, tok.data(), (size_t)n * 4, hipMemcpyHostToDevice, s));
        HIPCHK(hipMemcpyAsync(st.tr_row, row.data(), (size_t)n * 4, hipMemcpyHostToDevice, s));
        HIPCHK(hipMemcpyAsync(st.tr_pos, pos.data(), (size_t)n * 4, hipMemcpyHostToDevice, s));
        forward(w, ln, n, n, nullptr, nullptr, true, s);
        HIPCHK(hipMemcpyAsync(lg.data(), ln.ws.logits.p, (size_t)n * V * 4, hipMemcpyDeviceToHost, s));
        HIPCHK(hipStreamSynchronize(s));
        for (int j = 0; j < n; ++j)
            std::memcpy(logits_out + (out_base[row[j]] + g) * V, lg.data() + (size_t)j * V, (size_t)V * 4);
    }
    HIPCHK(hipGetLastError());
    return SS_OK;
}

}  // namespace

extern "C" int ss_forward_logits(ss_weights* w, const int32_t* tokens, const int32_t* offsets, int32_t B,
                                 const int32_t* n_prompt, int32_t all_prompt_logits, float* logits_out,
                                 void* hip_stream)
{
    ss::clear_error();
    if (int rc = check_prompts(w, tokens, offsets, B)) return rc;
    if (!n_prompt || !logits_out) return ss::fail(SS_EINVAL, "NULL argument");
    BusyGuard guard(w);
    if (!guard.ok) return ss::fail(SS_ESTATE, "another call is in flight on this handle");
    Lane& ln = w->lane[0];
    hipStream_t s = hip_stream ? (hipStream_t)hip_stream : ln.stream;
    return ss::no_throw(
        [&] { return forward_logits_impl(w, ln, s, tokens, offsets, B, n_prompt, all_prompt_logits, logits_out); });
}

namespace {

// The group pipeline shared by ss_run_group (gen == nullptr, lengths known) and ss_run_group_generate.
// A pass over a plan hands its micro-batches out one at a time, longest cap first, to the lanes at work: the
// calling thread on lane 0 and up to kLanes - 1 further host threads, each on a lane with its own stream and
// workspace, so that one micro-batch's kernels fill the gaps between the others'.  What a query receives does not depend on the
// lane or the order: micro-batches are independent, failures are sorted before they are rescheduled.
int run_group_impl(ss_weights* w, const int32_t* prompt_tokens, const int32_t* prompt_offsets, int32_t n,
                   const int32_t* target_lens, const int32_t* pred_lens, int32_t bin, const ss_policy* policy,
                   const ss_gen_opts* gen, int32_t* out_tokens, int32_t* out_lens, ss_group_stats* stats, hipStream_t s)
{
    using clk = std::chrono::steady_clock;
    const auto t_plan0 = clk::now();
    struct PlanOwner {   // frees the plan however the call ends
        ss_plan* p = nullptr;
        ~PlanOwner() { ss_plan_free(p); }
    };
    PlanOwner first_plan;
    if (int rc = ss_schedule(pred_lens, n, bin, policy, &first_plan.p)) return rc;
    const ss_plan* plan = first_plan.p;
    double plan_ms = std::chrono::duration<double, std::milli>(clk::now() - t_plan0).count();

    ss_group_stats gs{};
    const int L = policy->base_len;
    const uint32_t eflags = policy->flags & SS_COMPACT;
    std::vector<int32_t> failed;
    for (size_t i = 0; i < (size_t)n * L; ++i) out_tokens[i] = -1;

    // state shared by the lanes of one pass
    struct Pass {
        const ss_plan* pl = nullptr;
        bool first = true;
        std::vector<int> order;        // micro-batch indices in the order they are handed out
        std::atomic<int> next{0};
        std::atomic<int> stop{0};
        std::mutex mu;                 // guards gs, failed, rc/err and the progress lines
        int rc = SS_OK;
        char err[512] = "";            // fixed storage: recording an error allocates nothing
    };

    // One lane's share of a pass.  Runs on the calling thread (lane 0) or on a thread of its own (the other lanes).
    auto work = [&](Pass& ps, Lane& ln, hipStream_t ls) {
        std::vector<int32_t> mb_toks, mb_offs, mb_tl, mb_out, mb_lens, mb_ids;
        std::vector<float> mb_draws;
        std::vector<uint8_t> mb_failed;
        const ss_plan* pl = ps.pl;
        auto give_up = [&](int rc) {
            std::lock_guard<std::mutex> lock(ps.mu);
            if (ps.rc == SS_OK) {
                ps.rc = rc;
                std::snprintf(ps.err, sizeof(ps.err), "%s", ss_last_error());
            }
            ps.stop.store(1);
        };
        if (hipSetDevice(w->device) != hipSuccess) return give_up(ss::fail(SS_EDEVICE, "hipSetDevice failed"));
        while (!ps.stop.load()) {
            const int at = ps.next.fetch_add(1);
            if (at >= pl->n_mb) break;
            const int k = ps.order[at];
            const int b0 = pl->mb_offsets[k], B = pl->mb_offsets[k + 1] - b0, cap = pl->mb_cap[k];
            const int32_t* src_tl = gen ? gen->target_lens : target_lens;
            mb_toks.clear();
            mb_offs.assign(1, 0);
            mb_tl.resize(B);
            const bool given_draws = gen && gen->temperature > 0.f && gen->draws;
            if (given_draws) mb_draws.resize((size_t)B * cap);
            mb_ids.resize(B);
            for (int r = 0; r < B; ++r) {
                const int qi = pl->query_idx[b0 + r];
                mb_toks.insert(mb_toks.end(), prompt_tokens + prompt_offsets[qi], prompt_tokens + prompt_offsets[qi + 1]);
                mb_offs.push_back((int32_t)mb_toks.size());
                if (src_tl) mb_tl[r] = src_tl[qi];
                if (given_draws)
                    std::memcpy(mb_draws.data() + (size_t)r * cap, gen->draws + (size_t)qi * gen->draws_stride,
                                (size_t)cap * 4);
                mb_ids[r] = gen && gen->draw_ids ? gen->draw_ids[qi] : qi;
            }
            mb_out.resize((size_t)B * cap);
            mb_lens.resize(B);
            mb_failed.resize(B);
            ss_stats st{};
            ss_gen_opts mbg{};
            if (gen) {
                mbg = *gen;
                mbg.draws = given_draws ? mb_draws.data() : nullptr;
                mbg.draws_stride = cap;
                mbg.draw_ids = mb_ids.data();
                mbg.target_lens = src_tl ? mb_tl.data() : nullptr;
            }
            if (int rc = decode_microbatch_impl(w, ln, mb_toks.data(), mb_offs.data(), B, cap, mb_tl.data(),
                                                gen ? &mbg : nullptr, eflags, mb_out.data(), mb_lens.data(),
                                                mb_failed.data(), &st, ls))
                return give_up(rc);
            std::lock_guard<std::mutex> lock(ps.mu);
            for (int r = 0; r < B; ++r) {
                const int qi = pl->query_idx[b0 + r];
                // unfinished below the global limit: partial output and key/value state are dropped, the
                // query is recomputed later; unfinished at the global limit is simply the truncated result
                if (mb_failed[r] && cap < L) {
                    failed.push_back(qi);
                    continue;
                }
                std::memcpy(out_tokens + (size_t)qi * L, mb_out.data() + (size_t)r * cap, (size_t)mb_lens[r] * 4);
                out_lens[qi] = mb_lens[r];
            }
            gs.steps += st.steps;
            gs.padded_row_steps += (int64_t)B * st.steps;
            gs.computed_row_steps += st.row_steps;
            gs.prompt_tokens += st.prompt_tokens;
            gs.prefill_ms += st.prefill_ms;
            gs.decode_ms += st.decode_ms;
            gs.polls += st.polls;
            gs.idle_steps += st.idle_steps;
            (ps.first ? gs.n_mb_first : gs.n_mb_failure) += 1;
            if (ss::verbose() > 0) {
                std::fprintf(stderr, "[ss] %s micro-batch %d/%d: %d rows, cap %d, %d steps, %.0f ms\n",
                             ps.first ? "first-pass" : "recompute", k + 1, pl->n_mb, B, cap, st.steps,
                             st.prefill_ms + st.decode_ms);
                std::fflush(stderr);
            }
        }
    };
    // A lane's share with nothing escaping the thread it runs on.
    auto work_noexcept = [&](Pass& ps, Lane& ln, hipStream_t ls) {
        try {
            work(ps, ln, ls);
        } catch (...) {
            std::lock_guard<std::mutex> lock(ps.mu);
            if (ps.rc == SS_OK) {
                ps.rc = SS_ENOMEM;
                std::snprintf(ps.err, sizeof(ps.err), "host allocation failed in a micro-batch");
            }
            ps.stop.store(1);
        }
    };

    auto run_plan = [&](const ss_plan* pl, bool first) -> int {
        Pass ps;
        ps.pl = pl;
        ps.first = first;
        ps.order.resize((size_t)pl->n_mb);
        std::iota(ps.order.begin(), ps.order.end(), 0);
        const int lanes = std::min({w->in_flight, kLanes, (int)pl->n_mb});
        if (lanes > 1)   // longest first, so that the pass does not end with one lane idle behind a long micro-batch
            std::stable_sort(ps.order.begin(), ps.order.end(), [&](int a, int b) {
                const int64_t ca = (int64_t)pl->mb_cap[a] * (64 + pl->mb_offsets[a + 1] - pl->mb_offsets[a]);
                const int64_t cb = (int64_t)pl->mb_cap[b] * (64 + pl->mb_offsets[b + 1] - pl->mb_offsets[b]);
                return ca > cb;
            });
        std::thread others[kLanes];   // fixed storage: from here on nothing can throw past the joins
        int n_others = 0;
        for (int l = 1; l < lanes; ++l) {
            try {
                others[n_others] = std::thread([&, l] { work_noexcept(ps, w->lane[l], w->lane[l].stream); });
                ++n_others;
            } catch (...) {   // no further thread to be had: the pass runs on those it has
                break;
            }
        }
        work_noexcept(ps, w->lane[0], s);
        for (int i = 0; i < n_others; ++i) others[i].join();
        if (ps.rc != SS_OK) return ss::fail(ps.rc, "%s", ps.err);
        return SS_OK;
    };

    const auto t0 = clk::now();
    int rc = run_plan(plan, true);
    if (rc) return rc;
    gs.n_failed = (int32_t)failed.size();
    if (!failed.empty()) {
        std::sort(failed.begin(), failed.end());
        const auto tp = clk::now();
        PlanOwner fplan;
        if ((rc = ss_schedule_failures(pred_lens, n, failed.data(), (int32_t)failed.size(), bin, policy, &fplan.p)))
            return rc;
        plan_ms += std::chrono::duration<double, std::milli>(clk::now() - tp).count();
        failed.clear();
        rc = run_plan(fplan.p, false);
        if (rc) return rc;
        if (!failed.empty()) return ss::fail(SS_ESTATE, "a query failed in the recomputation pass");
    }
    gs.wall_ms = std::chrono::duration<double, std::milli>(clk::now() - t0).count();
    gs.plan_ms = plan_ms;
    for (int i = 0; i < n; ++i) gs.useful_tokens += gen ? out_lens[i] : target_lens[i];
    if (stats) *stats = gs;
    return SS_OK;
}

}  // namespace

extern "C" int ss_run_group(ss_weights* w, const int32_t* prompt_tokens, const int32_t* prompt_offsets, int32_t n,
                            const int32_t* target_lens, const int32_t* pred_lens, int32_t bin, const ss_policy* policy,
                            int32_t* out_tokens, int32_t* out_lens, ss_group_stats* stats, void* hip_stream)
{
    ss::clear_error();
    if (!w) return ss::fail(SS_EINVAL, "weights handle is NULL");
    if (n <= 0 || !prompt_tokens || !prompt_offsets || !target_lens || !policy || !out_tokens || !out_lens)
        return ss::fail(SS_EINVAL, "NULL or empty argument");
    BusyGuard guard(w);
    if (!guard.ok) return ss::fail(SS_ESTATE, "another call is in flight on this handle");
    Lane& ln = w->lane[0];
    hipStream_t s = hip_stream ? (hipStream_t)hip_stream : ln.stream;
    for (int i = 0; i < n; ++i)
        if (target_lens[i] < 1 || target_lens[i] > policy->base_len)
            return ss::fail(SS_EINVAL, "target_lens[%d] outside [1, base_len]", i);
    return ss::no_throw([&] {
        return run_group_impl(w, prompt_tokens, prompt_offsets, n, target_lens, pred_lens, bin, policy, nullptr,
                              out_tokens, out_lens, stats, s);
    });
}

extern "C" int ss_run_group_generate(ss_weights* w, const int32_t* prompt_tokens, const int32_t* prompt_offsets,
                                     int32_t n, const int32_t* pred_lens, int32_t bin, const ss_policy* policy,
                                     const ss_gen_opts* opts, int32_t* out_tokens, int32_t* out_lens,
                                     ss_group_stats* stats, void* hip_stream)
{
    ss::clear_error();
    if (!w) return ss::fail(SS_EINVAL, "weights handle is NULL");
    if (n <= 0 || !prompt_tokens || !prompt_offsets || !policy || !out_tokens || !out_lens)
        return ss::fail(SS_EINVAL, "NULL or empty argument");
    if (policy->base_len < 1) return ss::fail(SS_EINVAL, "base_len must be >= 1");
    if (int rc = check_gen_opts(w, opts, n, policy->base_len)) return rc;
    BusyGuard guard(w);
    if (!guard.ok) return ss::fail(SS_ESTATE, "another call is in flight on this handle");
    Lane& ln = w->lane[0];
    hipStream_t s = hip_stream ? (hipStream_t)hip_stream : ln.stream;
    return ss::no_throw([&] {
        return run_group_impl(w, prompt_tokens, prompt_offsets, n, nullptr, pred_lens, bin, policy, opts, out_tokens,
                              out_lens, stats, s);
    });
}

namespace {

// Prefills B rows of ctx tokens on a lane, then times iters decode forwards on it.  `gate`, when given, is
// counted up after the prefill has finished and waited on until it reaches `parties`, so that several lanes
// start their timed forwards together.
int bench_decode_step_lane(const ss_weights* w, Lane& ln, hipStream_t s, const int32_t* prompt_tokens, int32_t B,
                           int32_t ctx, int32_t iters, double* ms_out, std::atomic<int>* gate, int parties)
{
    struct Arrive {   // a lane that fails before the gate must not leave the others waiting
        std::atomic<int>* g;
        bool done = false;
        void now()
        {
            if (g && !done) g->fetch_add(1);
            done = true;
        }
        ~Arrive() { now(); }
    } arrive{gate};
    std::vector<int32_t> offs(B + 1), lens(B, ctx), slab(B, ctx + 1), limit(B, 2), sel(B);
    for (int i = 0; i <= B; ++i) offs[i] = i * ctx;
    for (int i = 0; i < B; ++i) sel[i] = (i + 1) * ctx - 1;
    HIPCHK(hipSetDevice(w->device));
    if (int rc = ensure_workspace(w, ln, B * ctx, B, B, (size_t)B * (ctx + 1), 2, s)) return rc;
    const MbState& st = ln.st;
    if (int rc = upload_prompt_state(ln, prompt_tokens, offs.data(), lens.data(), B, slab.data(), limit.data(), sel, s))
        return rc;
    forward(w, ln, B * ctx, B, ln.d_sel, st.d_nlive, false, s);
    ss::launch_step_update(st, 0, -1, s);   // token-rows of the decode step: every row at position ctx
    EventList evl;
    if (int rc = evl.create(iters + 1)) return rc;
    const std::vector<hipEvent_t>& ev = evl.e;
    if (gate) {
        HIPCHK(hipStreamSynchronize(s));
        arrive.now();
        while (gate->load() < parties) std::this_thread::yield();
    }
    HIPCHK(hipEventRecord(ev[0], s));
    for (int it = 0; it < iters; ++it) {
        forward(w, ln, B, B, nullptr, nullptr, true, s);
        HIPCHK(hipEventRecord(ev[it + 1], s));
    }
    HIPCHK(hipStreamSynchronize(s));
    HIPCHK(hipGetLastError());
    for (int it = 0; it < iters; ++it) {
        float ms = 0.f;
        HIPCHK(hipEventElapsedTime(&ms, ev[it], ev[it + 1]));
        ms_out[it] = ms;
    }
    return SS_OK;
}

int check_bench_decode_step(const ss_weights* w, const int32_t* prompt_tokens, int32_t B, int32_t ctx, int32_t iters,
                            const double* ms_out)
{
    if (!w || !prompt_tokens || !ms_out) return ss::fail(SS_EINVAL, "NULL argument");
    if (B <= 0 || B > ss::kMaxBatch || ctx < 1 || ctx + 1 > ss::kMaxPos || iters < 1)
        return ss::fail(SS_EINVAL, "bad B / ctx / iters");
    for (size_t t = 0; t < (size_t)B * ctx; ++t)
        if (prompt_tokens[t] < 0 || prompt_tokens[t] >= w->cfg.vocab) return ss::fail(SS_EINVAL, "token id out of range");
    return SS_OK;
}

}  // namespace

extern "C" int ss_bench_decode_step(ss_weights* w, const int32_t* prompt_tokens, int32_t B, int32_t ctx,
                                    int32_t iters, double* ms_out, void* hip_stream)
{
    ss::clear_error();
    if (int rc = check_bench_decode_step(w, prompt_tokens, B, ctx, iters, ms_out)) return rc;
    BusyGuard guard(w);
    if (!guard.ok) return ss::fail(SS_ESTATE, "another call is in flight on this handle");
    Lane& ln = w->lane[0];
    hipStream_t s = hip_stream ? (hipStream_t)hip_stream : ln.stream;
    return ss::no_throw(
        [&] { return bench_decode_step_lane(w, ln, s, prompt_tokens, B, ctx, iters, ms_out, nullptr, 0); });
}

extern "C" int ss_bench_decode_steps_in_flight(ss_weights* w, const int32_t* prompt_tokens, int32_t B, int32_t ctx,
                                               int32_t iters, int32_t lanes, double* ms_out)
{
    ss::clear_error();
    if (int rc = check_bench_decode_step(w, prompt_tokens, B, ctx, iters, ms_out)) return rc;
    if (lanes < 1 || lanes > kLanes) return ss::fail(SS_EINVAL, "lanes outside [1, %d]", kLanes);
    BusyGuard guard(w);
    if (!guard.ok) return ss::fail(SS_ESTATE, "another call is in flight on this handle");
    std::atomic<int> gate{0};
    int rc[kLanes] = {};
    char err[kLanes][256] = {};
    auto run = [&](int l) {   // a lane's thread lets no exception out; its error text is copied for the caller
        rc[l] = ss::no_throw([&] {
            return bench_decode_step_lane(w, w->lane[l], w->lane[l].stream, prompt_tokens, B, ctx, iters,
                                          ms_out + (size_t)l * iters, &gate, lanes);
        });
        if (rc[l]) std::snprintf(err[l], sizeof(err[l]), "%s", ss_last_error());
    };
    std::thread others[kLanes];   // fixed storage: only starting a thread can fail below
    int n_others = 0;
    auto join_all = [&] {
        for (int i = 0; i < n_others; ++i) others[i].join();
    };
    for (int l = 1; l < lanes; ++l) {
        try {
            others[n_others] = std::thread(run, l);
            ++n_others;
        } catch (...) {
            // the lanes already started (1 .. l-1) wait at the gate for `lanes` arrivals: stand in for the ones
            // that will not come (l .. lanes-1, and lane 0, which this thread would have run)
            gate.fetch_add(lanes - l + 1);
            join_all();
            return ss::fail(SS_ESTATE, "could not start host thread %d", l);
        }
    }
    run(0);
    join_all();
    for (int l = 0; l < lanes; ++l)
        if (rc[l]) return ss::fail(rc[l], "%s", err[l]);
    return SS_OK;
}

namespace {

int bench_weight_stream_impl(const ss_weights* w, Lane& ln, hipStream_t s, int32_t B, int32_t iters, double* ms_out,
                             int32_t* launches_out)
{
    HIPCHK(hipSetDevice(w->device));
    if (int rc = ensure_workspace(w, ln, B, B, B, (size_t)B, 1, s)) return rc;
    const ss_model_cfg& c = w->cfg;
    const int d = c.d_model, F = c.d_ffn, V = c.vocab, Fp = ss::padded_k(F), n = B;
    Workspace& ws = ln.ws;
    const Plans pl = make_plans(w, n, n);
    const ss::GemmPlan &p_qkv = pl.qkv, &p_o = pl.o, &p_gu = pl.gu, &p_d = pl.down, &p_lm = pl.lm;
    auto mk = [w](const f16_t* W, const f16_t* X, float* out, f16_t* outp, int N, int Kp, int rows, int kp_out,
                  const ss::GemmPlan& p) { return gemm_args(w, W, X, out, outp, N, Kp, rows, kp_out, p); };
    f16_t *h = ws.h.as<f16_t>(), *ao = ws.ao.as<f16_t>(), *act = ws.act.as<f16_t>();
    float *pqkv = ws.pqkv.as<float>(), *pd = ws.pd.as<float>();
    EventList evl;
    if (int rc = evl.create(iters + 1)) return rc;
    const std::vector<hipEvent_t>& ev = evl.e;
    HIPCHK(hipEventRecord(ev[0], s));
    int launches = 0;
    for (int it = 0; it < iters; ++it) {
        launches = 0;
        for (int l = 0; l < c.n_layers; ++l) {
            const Layer& L = w->layers[l];
            ss::launch_gemm(mk(L.wqkv.p, h, pqkv, nullptr, 3 * d, d, n, 0, p_qkv), ss::EPI_PARTIAL, s);
            ss::launch_gemm(mk(L.wo.p, ao, pd, nullptr, d, d, n, 0, p_o), ss::EPI_PARTIAL, s);
            if (p_gu.ksplit == 1)
                ss::launch_gemm(mk(L.wgu.p, h, nullptr, act, 2 * F, d, n, Fp, p_gu), ss::EPI_SWIGLU, s);
            else
                ss::launch_gemm(mk(L.wgu.p, h, ws.pgu.as<float>(), nullptr, 2 * F, d, n, 0, p_gu), ss::EPI_PARTIAL, s);
            ss::launch_gemm(mk(L.wd.p, act, pd, nullptr, d, Fp, n, 0, p_d), ss::EPI_PARTIAL, s);
            launches += 4;
        }
        ss::launch_gemm(mk(w->lm_head.p, ws.hsel.as<f16_t>(), ws.logits.as<float>(), nullptr, V, d, n, 0, p_lm),
                        ss::EPI_PARTIAL, s);
        launches += 1;
        HIPCHK(hipEventRecord(ev[it + 1], s));
    }
    HIPCHK(hipStreamSynchronize(s));
    HIPCHK(hipGetLastError());
    for (int it = 0; it < iters; ++it) {
        float ms = 0.f;
        HIPCHK(hipEventElapsedTime(&ms, ev[it], ev[it + 1]));
        ms_out[it] = ms;
    }
    if (launches_out) *launches_out = launches;
    return SS_OK;
}

int bench_read_stream_impl(const ss_weights* w, Lane& ln, hipStream_t s, int32_t iters, double* ms_out,
                           int64_t* bytes_out)
{
    HIPCHK(hipSetDevice(w->device));
    if (int rc = ln.ws.ints.ensure(64, false)) return rc;
    uint32_t* sink = ln.ws.ints.as<uint32_t>();
    auto mat_bytes = [](const PackedMat& m) { return ((size_t)m.N * m.Kp * 2) & ~(size_t)0xffff; };
    EventList evl;
    if (int rc = evl.create(iters + 1)) return rc;
    const std::vector<hipEvent_t>& ev = evl.e;
    HIPCHK(hipEventRecord(ev[0], s));
    size_t bytes = 0;
    for (int it = 0; it < iters; ++it) {
        bytes = 0;
        for (const Layer& L : w->layers)
            for (const PackedMat* m : {&L.wqkv, &L.wo, &L.wgu, &L.wd}) {
                ss::launch_read_stream(m->p, mat_bytes(*m), sink, s);
                bytes += mat_bytes(*m);
            }
        ss::launch_read_stream(w->lm_head.p, mat_bytes(w->lm_head), sink, s);
        bytes += mat_bytes(w->lm_head);
        HIPCHK(hipEventRecord(ev[it + 1], s));
    }
    HIPCHK(hipStreamSynchronize(s));
    HIPCHK(hipGetLastError());
    for (int it = 0; it < iters; ++it) {
        float ms = 0.f;
        HIPCHK(hipEventElapsedTime(&ms, ev[it], ev[it + 1]));
        ms_out[it] = ms;
    }
    if (bytes_out) *bytes_out = (int64_t)bytes;
    return SS_OK;
}

}  // namespace

extern "C" int ss_bench_weight_stream(ss_weights* w, int32_t B, int32_t iters, double* ms_out, int32_t* launches_out,
                                      void* hip_stream)
{
    ss::clear_error();
    if (!w || !ms_out) return ss::fail(SS_EINVAL, "NULL argument");
    if (B <= 0 || B > ss::kMaxBatch || iters < 1) return ss::fail(SS_EINVAL, "bad B / iters");
    BusyGuard guard(w);
    if (!guard.ok) return ss::fail(SS_ESTATE, "another call is in flight on this handle");
    Lane& ln = w->lane[0];
    hipStream_t s = hip_stream ? (hipStream_t)hip_stream : ln.stream;
    return ss::no_throw([&] { return bench_weight_stream_impl(w, ln, s, B, iters, ms_out, launches_out); });
}

extern "C" int ss_bench_read_stream(ss_weights* w, int32_t iters, double* ms_out, int64_t* bytes_out, void* hip_stream)
{
    ss::clear_error();
    if (!w || !ms_out) return ss::fail(SS_EINVAL, "NULL argument");
    if (iters < 1) return ss::fail(SS_EINVAL, "bad iters");
    BusyGuard guard(w);
    if (!guard.ok) return ss::fail(SS_ESTATE, "another call is in flight on this handle");
    Lane& ln = w->lane[0];
    hipStream_t s = hip_stream ? (hipStream_t)hip_stream : ln.stream;
    return ss::no_throw([&] { return bench_read_stream_impl(w, ln, s, iters, ms_out, bytes_out); });
}
