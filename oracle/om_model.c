/*
 * CPU oracle for the batched greedy decode of a LLaMA-style decoder.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * HIP path is checked against.  Only the tests, the smoke check and the
 * benchmark's cpu_baseline leg may build or call it; the product library never
 * links, loads or falls back to it, and the two share no source.
 *
 * What it computes.  The paper (Sec. 4.1, Method) batches queries into
 * micro-batches and generates token by token until every row has finished or
 * the cap on newly generated tokens is reached (FCR paragraph); the decoder
 * under it is the stock LLaMA-family model named in Sec. 4.2 (Experimental
 * Setting).  The paper prints no formula for the decoder, so the definition
 * here is the family's standard one with the free choices fixed as follows
 * (both sides of every parity test use the same choices):
 *   - pre-norm residual blocks; RMSNorm y = x * rsqrt(mean(x^2) + eps) * w;
 *   - projections y = x W^T with W stored [out, in], no bias anywhere;
 *   - rotary embedding on q and k, pairing element j with j + hd/2,
 *     angle = pos * base^(-2j/hd), positions start at 0 for every row, no BOS;
 *   - causal softmax attention with scale 1/sqrt(hd), max-subtracted;
 *   - MLP  down( silu(gate(h)) * up(h) ), silu(z) = z / (1 + exp(-z));
 *   - final RMSNorm, untied LM head, greedy argmax with the lowest index on ties;
 *   - end of sequence is simulated: row i is finished exactly when it has
 *     emitted target_len[i] tokens (or the cap, whichever is smaller); a row
 *     whose target exceeds the cap is a failure (Sec. 4.1, FCR).
 *   - prompts are ragged: no pad token is ever computed or attended, so a
 *     query's tokens do not depend on which micro-batch it ran in.
 *
 * Precision.  Weights are bf16 bit patterns widened exactly.  All arithmetic
 * is done in om_real, which is double unless the file is compiled with
 * -DOM_REAL_FLOAT (an fp32 build of the same text, used to show what plain
 * fp32 evaluation gives and as the timed CPU baseline).
 *
 * Every loop nest below is the definition written out: no blocking, no fusion,
 * no reordering other than the OpenMP "simd reduction" on the innermost dot
 * product and "parallel for" over independent outputs.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef OM_REAL_FLOAT
typedef float om_real;
#else
typedef double om_real;
#endif

typedef struct {
    int32_t n_layers, d_model, n_heads, head_dim, d_ffn, vocab;
    float rope_base, rms_eps;
} om_cfg;

typedef struct {
    om_cfg cfg;
    const uint16_t **t; /* borrowed tensor pointers, fixed order (see tensor index helpers) */
} om_model;

/* One sequence's key/value history: k, v are [n_layers][cap][d_model]. */
typedef struct {
    int32_t cap, len;
    om_real *k, *v;
} om_seq;

/* ------------------------------------------------------------------ tensor order */
/* embed, then per layer: attn_norm wq wk wv wo mlp_norm wg wu wd, then final_norm, lm_head */
enum { T_ATTN_NORM = 0, T_WQ, T_WK, T_WV, T_WO, T_MLP_NORM, T_WG, T_WU, T_WD, T_PER_LAYER };
static const uint16_t *layer_t(const om_model *m, int l, int which) { return m->t[1 + l * T_PER_LAYER + which]; }
static const uint16_t *embed_t(const om_model *m) { return m->t[0]; }
static const uint16_t *final_norm_t(const om_model *m) { return m->t[1 + m->cfg.n_layers * T_PER_LAYER]; }
static const uint16_t *lm_head_t(const om_model *m) { return m->t[2 + m->cfg.n_layers * T_PER_LAYER]; }

static inline om_real bf16_widen(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, 4);
    return (om_real)f;
}

int om_real_size(void) { return (int)sizeof(om_real); }

/* ------------------------------------------------------------------ components
 * Each is exported so the tests can pin it on its own against a library routine
 * or a closed form; the model below calls exactly these functions. */

/* RMSNorm: out_j = x_j * w_j / sqrt(mean_j x_j^2 + eps). */
void om_c_rmsnorm(const om_real *x, const uint16_t *w, int d, float eps, om_real *out)
{
    om_real ss = 0;
    for (int j = 0; j < d; ++j) ss += x[j] * x[j];
    om_real r = (om_real)1 / (om_real)sqrt((double)(ss / (om_real)d + (om_real)eps));
    for (int j = 0; j < d; ++j) out[j] = x[j] * r * bf16_widen(w[j]);
}

/* y_o = sum_k x_k W[o][k], W is [n_out][n_in] bf16. */
static inline om_real dot_bf16(const om_real *x, const uint16_t *w, int n)
{
    om_real acc = 0;
#pragma omp simd reduction(+ : acc)
    for (int k = 0; k < n; ++k) acc += x[k] * bf16_widen(w[k]);
    return acc;
}

void om_c_matvec(const om_real *x, const uint16_t *W, int n_out, int n_in, om_real *y)
{
    for (int o = 0; o < n_out; ++o) y[o] = dot_bf16(x, W + (size_t)o * n_in, n_in);
}

/* Rows of x are [n][n_in], rows of y are [n][n_out]; the weight row is reused across the n rows. */
static void matmul_rows(const om_real *x, int n, const uint16_t *W, int n_out, int n_in, om_real *y)
{
#pragma omp parallel for schedule(static)
    for (int o = 0; o < n_out; ++o) {
        const uint16_t *wrow = W + (size_t)o * n_in;
        for (int j = 0; j < n; ++j) y[(size_t)j * n_out + o] = dot_bf16(x + (size_t)j * n_in, wrow, n_in);
    }
}

/* Rotary embedding of one head vector in place: pairs (j, j + hd/2), angle pos * base^(-2j/hd). */
void om_c_rope(om_real *v, int hd, int pos, float base)
{
    int half = hd / 2;
    for (int j = 0; j < half; ++j) {
        double ang = (double)pos * pow((double)base, -2.0 * (double)j / (double)hd);
        om_real c = (om_real)cos(ang), s = (om_real)sin(ang);
        om_real a = v[j], b = v[j + half];
        v[j] = a * c - b * s;
        v[j + half] = a * s + b * c;
    }
}

/* out = sum_u softmax_u(q.k_u / sqrt(hd)) v_u over u in [0, T); K and V rows are `stride` apart. */
void om_c_attention(const om_real *q, const om_real *K, const om_real *V, int T, int hd, int stride, om_real *out)
{
    om_real *s = (om_real *)malloc(sizeof(om_real) * (size_t)T);
    om_real scale = (om_real)1 / (om_real)sqrt((double)hd);
    om_real mx = 0;
    for (int u = 0; u < T; ++u) {
        om_real acc = 0;
        for (int e = 0; e < hd; ++e) acc += q[e] * K[(size_t)u * stride + e];
        s[u] = acc * scale;
        if (u == 0 || s[u] > mx) mx = s[u];
    }
    om_real den = 0;
    for (int u = 0; u < T; ++u) {
        s[u] = (om_real)exp((double)(s[u] - mx));
        den += s[u];
    }
    for (int e = 0; e < hd; ++e) out[e] = 0;
    for (int u = 0; u < T; ++u) {
        om_real p = s[u] / den;
        for (int e = 0; e < hd; ++e) out[e] += p * V[(size_t)u * stride + e];
    }
    free(s);
}

om_real om_c_silu(om_real z) { return z / ((om_real)1 + (om_real)exp((double)-z)); }

/* Greedy choice: index of the maximum, lowest index on exact ties; margin = top1 - top2 (0 on a tie). */
int om_c_argmax(const om_real *logits, int n, double *margin_out)
{
    int best = 0;
    for (int i = 1; i < n; ++i)
        if (logits[i] > logits[best]) best = i;
    if (margin_out) {
        int have = 0;
        om_real second = 0;
        for (int i = 0; i < n; ++i) {
            if (i == best) continue;
            if (!have || logits[i] > second) { second = logits[i]; have = 1; }
        }
        *margin_out = have ? (double)(logits[best] - second) : INFINITY;
    }
    return best;
}

/* ------------------------------------------------------------------ model / sequences */
om_model *om_model_create(const om_cfg *cfg, const uint16_t *const *tensors)
{
    if (!cfg || !tensors) return NULL;
    if (cfg->n_heads * cfg->head_dim != cfg->d_model || (cfg->head_dim & 1)) return NULL;
    om_model *m = (om_model *)calloc(1, sizeof(om_model));
    m->cfg = *cfg;
    int nt = 3 + cfg->n_layers * T_PER_LAYER;
    m->t = (const uint16_t **)malloc(sizeof(void *) * (size_t)nt);
    for (int i = 0; i < nt; ++i) m->t[i] = tensors[i];
    return m;
}

void om_model_free(om_model *m)
{
    if (!m) return;
    free((void *)m->t);
    free(m);
}

om_seq *om_seq_create(const om_model *m, int cap)
{
    om_seq *s = (om_seq *)calloc(1, sizeof(om_seq));
    size_t n = (size_t)m->cfg.n_layers * (size_t)cap * (size_t)m->cfg.d_model;
    s->cap = cap;
    s->len = 0;
    s->k = (om_real *)malloc(sizeof(om_real) * n);
    s->v = (om_real *)malloc(sizeof(om_real) * n);
    return s;
}

void om_seq_reset(om_seq *s) { s->len = 0; }

void om_seq_free(om_seq *s)
{
    if (!s) return;
    free(s->k);
    free(s->v);
    free(s);
}

/*
 * Forward n token-rows.  Row j feeds token tok[j] at position pos[j] of sequence
 * seqs[seq_of[j]].  Several rows may belong to one sequence (a prompt processed
 * at once) provided their positions are consecutive, increasing, and start at
 * the sequence's current length; attention of a row sees positions <= its own.
 * want[j] != 0 asks for that row's logits, written densely in row order into
 * logits_out as double [n_want][vocab].  Returns 0, or -1 on a bad argument.
 */
int om_forward_rows(const om_model *m, om_seq **seqs, int n, const int32_t *seq_of, const int32_t *tok,
                    const int32_t *pos, const uint8_t *want, double *logits_out)
{
    const om_cfg *c = &m->cfg;
    const int d = c->d_model, H = c->n_heads, hd = c->head_dim, F = c->d_ffn, V = c->vocab;
    if (n <= 0) return -1;
    for (int j = 0; j < n; ++j) {
        if (tok[j] < 0 || tok[j] >= V) return -1;
        om_seq *s = seqs[seq_of[j]];
        if (pos[j] < 0 || pos[j] >= s->cap) return -1;
    }
    om_real *x = (om_real *)malloc(sizeof(om_real) * (size_t)n * d);
    om_real *h = (om_real *)malloc(sizeof(om_real) * (size_t)n * d);
    om_real *q = (om_real *)malloc(sizeof(om_real) * (size_t)n * d);
    om_real *kk = (om_real *)malloc(sizeof(om_real) * (size_t)n * d);
    om_real *vv = (om_real *)malloc(sizeof(om_real) * (size_t)n * d);
    om_real *a = (om_real *)malloc(sizeof(om_real) * (size_t)n * d);
    om_real *o = (om_real *)malloc(sizeof(om_real) * (size_t)n * d);
    om_real *g = (om_real *)malloc(sizeof(om_real) * (size_t)n * F);
    om_real *u = (om_real *)malloc(sizeof(om_real) * (size_t)n * F);

    /* token embedding */
    for (int j = 0; j < n; ++j)
        for (int e = 0; e < d; ++e) x[(size_t)j * d + e] = bf16_widen(embed_t(m)[(size_t)tok[j] * d + e]);

    for (int l = 0; l < c->n_layers; ++l) {
        /* attention block */
        for (int j = 0; j < n; ++j)
            om_c_rmsnorm(x + (size_t)j * d, layer_t(m, l, T_ATTN_NORM), d, c->rms_eps, h + (size_t)j * d);
        matmul_rows(h, n, layer_t(m, l, T_WQ), d, d, q);
        matmul_rows(h, n, layer_t(m, l, T_WK), d, d, kk);
        matmul_rows(h, n, layer_t(m, l, T_WV), d, d, vv);
        /* rotate q, k; append k, v to each row's own history (all rows before any attention) */
        for (int j = 0; j < n; ++j) {
            om_seq *s = seqs[seq_of[j]];
            for (int hh = 0; hh < H; ++hh) {
                om_c_rope(q + (size_t)j * d + hh * hd, hd, pos[j], c->rope_base);
                om_c_rope(kk + (size_t)j * d + hh * hd, hd, pos[j], c->rope_base);
            }
            size_t off = ((size_t)l * s->cap + (size_t)pos[j]) * d;
            memcpy(s->k + off, kk + (size_t)j * d, sizeof(om_real) * d);
            memcpy(s->v + off, vv + (size_t)j * d, sizeof(om_real) * d);
        }
#pragma omp parallel for schedule(dynamic)
        for (int jh = 0; jh < n * H; ++jh) {
            int j = jh / H, hh = jh % H;
            om_seq *s = seqs[seq_of[j]];
            size_t base = (size_t)l * s->cap * d + (size_t)hh * hd;
            om_c_attention(q + (size_t)j * d + hh * hd, s->k + base, s->v + base, pos[j] + 1, hd, d,
                           a + (size_t)j * d + hh * hd);
        }
        matmul_rows(a, n, layer_t(m, l, T_WO), d, d, o);
        for (size_t i = 0; i < (size_t)n * d; ++i) x[i] += o[i];
        /* MLP block */
        for (int j = 0; j < n; ++j)
            om_c_rmsnorm(x + (size_t)j * d, layer_t(m, l, T_MLP_NORM), d, c->rms_eps, h + (size_t)j * d);
        matmul_rows(h, n, layer_t(m, l, T_WG), F, d, g);
        matmul_rows(h, n, layer_t(m, l, T_WU), F, d, u);
        for (size_t i = 0; i < (size_t)n * F; ++i) g[i] = om_c_silu(g[i]) * u[i];
        matmul_rows(g, n, layer_t(m, l, T_WD), d, F, o);
        for (size_t i = 0; i < (size_t)n * d; ++i) x[i] += o[i];
    }

    /* final norm + LM head for the rows that asked */
    int nw = 0;
    for (int j = 0; j < n; ++j) {
        if (want && !want[j]) continue;
        if (logits_out) {
            om_c_rmsnorm(x + (size_t)j * d, final_norm_t(m), d, c->rms_eps, h);
            om_real *lg = (om_real *)malloc(sizeof(om_real) * (size_t)V);
            matmul_rows(h, 1, lm_head_t(m), V, d, lg);
            for (int t = 0; t < V; ++t) logits_out[(size_t)nw * V + t] = (double)lg[t];
            free(lg);
        }
        ++nw;
    }
    for (int j = 0; j < n; ++j) {
        om_seq *s = seqs[seq_of[j]];
        if (pos[j] + 1 > s->len) s->len = pos[j] + 1;
    }
    free(x); free(h); free(q); free(kk); free(vv); free(a); free(o); free(g); free(u);
    return 0;
}

/*
 * Greedy decode of one micro-batch (Sec. 4.1): the prompts are processed, then one
 * token per live row is generated per step until every row has emitted
 * min(target_len, max_new) tokens.  Row i fails iff target_len[i] > max_new.
 * The token produced by the prompt forward counts as the first generated token,
 * so a micro-batch costs steps = min(max_new, max_i target_len[i]) forwards.
 *
 * out_tokens  [B][max_new] emitted ids, -1 after the emitted length
 * out_lens    [B]          min(target, max_new)
 * out_failed  [B]          target > max_new
 * out_margin  [B][max_new] top-1 minus top-2 logit at each emitted position (nullable)
 * steps_out                number of forwards (nullable)
 * A finished row is simply not computed any more: what a padded engine feeds
 * such a row never reaches an output.
 */
int om_greedy_microbatch(const om_model *m, const int32_t *prompt_tokens, const int32_t *prompt_offsets, int B,
                         int max_new, const int32_t *target_lens, int32_t *out_tokens, int32_t *out_lens,
                         uint8_t *out_failed, double *out_margin, int32_t *steps_out)
{
    const int V = m->cfg.vocab;
    if (B <= 0 || max_new < 1) return -1;
    om_seq **seqs = (om_seq **)malloc(sizeof(om_seq *) * (size_t)B);
    int total = prompt_offsets[B], steps = 0;
    for (int i = 0; i < B; ++i) {
        int p = prompt_offsets[i + 1] - prompt_offsets[i];
        if (p < 1 || target_lens[i] < 1) return -1;
        seqs[i] = om_seq_create(m, p + max_new);
        out_lens[i] = target_lens[i] < max_new ? target_lens[i] : max_new;
        out_failed[i] = target_lens[i] > max_new;
        if (out_lens[i] > steps) steps = out_lens[i];
        for (int g = 0; g < max_new; ++g) {
            out_tokens[(size_t)i * max_new + g] = -1;
            if (out_margin) out_margin[(size_t)i * max_new + g] = 0.0;
        }
    }
    int32_t *seq_of = (int32_t *)malloc(sizeof(int32_t) * (size_t)(total > B ? total : B));
    int32_t *pos = (int32_t *)malloc(sizeof(int32_t) * (size_t)(total > B ? total : B));
    int32_t *tok = (int32_t *)malloc(sizeof(int32_t) * (size_t)(total > B ? total : B));
    uint8_t *want = (uint8_t *)malloc((size_t)(total > B ? total : B));
    double *logits = (double *)malloc(sizeof(double) * (size_t)B * V);
    om_real *row = (om_real *)malloc(sizeof(om_real) * (size_t)V);
    int32_t *last = (int32_t *)malloc(sizeof(int32_t) * (size_t)B);
    int32_t *who = (int32_t *)malloc(sizeof(int32_t) * (size_t)B);

    /* step 0: prompt forward; logits at each row's last prompt position give its first token */
    for (int i = 0; i < B; ++i)
        for (int t = prompt_offsets[i]; t < prompt_offsets[i + 1]; ++t) {
            seq_of[t] = i;
            pos[t] = t - prompt_offsets[i];
            tok[t] = prompt_tokens[t];
            want[t] = (t == prompt_offsets[i + 1] - 1);
        }
    int rc = om_forward_rows(m, seqs, total, seq_of, tok, pos, want, logits);
    int n_live = B;
    for (int i = 0; i < B; ++i) who[i] = i;
    for (int g = 0; rc == 0 && g < steps; ++g) {
        /* read the choice of every row that was forwarded, emit it */
        for (int j = 0; j < n_live; ++j) {
            int i = who[j];
            for (int t = 0; t < V; ++t) row[t] = (om_real)logits[(size_t)j * V + t];
            double mg;
            last[i] = om_c_argmax(row, V, &mg);
            out_tokens[(size_t)i * max_new + g] = last[i];
            if (out_margin) out_margin[(size_t)i * max_new + g] = mg;
        }
        if (g + 1 == steps) break;
        /* rows that still owe tokens feed their last token back */
        int nl = 0;
        for (int i = 0; i < B; ++i)
            if (g + 1 < out_lens[i]) {
                who[nl] = i;
                seq_of[nl] = i;
                tok[nl] = last[i];
                pos[nl] = (prompt_offsets[i + 1] - prompt_offsets[i]) + g;
                want[nl] = 1;
                ++nl;
            }
        n_live = nl;
        rc = om_forward_rows(m, seqs, n_live, seq_of, tok, pos, want, logits);
    }
    if (steps_out) *steps_out = steps;
    for (int i = 0; i < B; ++i) om_seq_free(seqs[i]);
    free(seqs); free(seq_of); free(pos); free(tok); free(want); free(logits); free(row); free(last); free(who);
    return rc;
}
