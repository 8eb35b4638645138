/*
 * libss - sequence-scheduled batched greedy decoding on one MI355X (gfx950).
 *
 * C ABI.  Every pointer argument says "host" or "device" below; nothing in a
 * signature is a framework type.  All functions are synchronous on return.
 * Every function that returns int returns SS_OK (0) or a negative ss_status;
 * ss_last_error() then gives a thread-local message.  No exception or abort
 * crosses this boundary; outputs are untouched when an error is returned
 * before any work was started.
 *
 * The operations follow the paper's Sec. 4.1 (Method): a group of queries is
 * ordered by predicted response length and split into micro-batches (binning,
 * variable batch size), every micro-batch is generated token by token with a
 * cap on newly generated tokens, rows that overrun the cap are failures that
 * are collected and recomputed after the group (FCR).  Sec. 4.2 gives the
 * constants (bin cell 50, baseline batch 16, group 256).
 */
#ifndef SS_H
#define SS_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { SS_OK = 0, SS_EINVAL = -1, SS_ENOMEM = -2, SS_EDEVICE = -3, SS_ESTATE = -4 } ss_status;

/* Thread-local text of the last error on this thread ("" if none).  Host pointer, library-owned. */
const char* ss_last_error(void);

/* Progress lines: level 1 makes ss_run_group print one line per finished micro-batch to stderr (long groups
 * take minutes); level 0 (default) prints nothing.  Process-wide. */
void ss_set_verbose(int32_t level);

/* Testing aid: which kernel runs the projections of small batches.  0 (default): chosen per shape and row
 * count; 1: never the kernel that stages activations once per workgroup (then: the k-splitting kernel up to 64
 * token-rows, the tiled kernel above); 2: that kernel for every projection of at most 256 token-rows.
 * Adding 4 to a mode (4, 5, 6) keeps that kernel from sharing a strip's k-blocks between two wavefronts (what it
 * does above 96 token-rows when a workgroup has few strips); adding 8 keeps the tiled kernel at 64-row tiles where
 * it would use 128-row tiles (prompt forwards of 896 token-rows and more); both for A/B measurements.
 * Results agree to the rounding differences between launch shapes (about 1e-3 of the largest logit).  Process-wide (atomic integers, read when a forward is planned: set it
 * between calls, not during one); other values are ignored. */
void ss_set_gemm_mode(int32_t mode);

/* ------------------------------------------------------------------ scheduler (host only) */

/* Policy flags.  0 = vanilla batching: arrival order, fixed batch, cap = base_len (Sec. 4.2 baseline). */
#define SS_SORT    1u  /* order the group by scheduled length (Sec. 4.1, sort-and-split)                  */
#define SS_BIN     2u  /* schedule by the upper edge of the prediction's bin (Sec. 4.1, Binning); needs SS_SORT */
#define SS_FCR     4u  /* cap = largest scheduled length in the micro-batch; overruns fail (Sec. 4.1, FCR) */
#define SS_VBS     8u  /* batch size inversely proportional to the scheduled length (Sec. 4.1, VBS); needs SS_SORT */
#define SS_COMPACT 16u /* engine flag: finished rows leave the live batch (not in the paper; outputs unchanged) */

#define SS_VBS_CLAMP_FLOOR 0 /* B = clamp(floor(base_batch*base_len/L), base_batch, max_batch)               */
#define SS_VBS_PAPER_POW2  1 /* Sec. 4.2: 16 if L >= 300, else 256*50/L rounded to the nearest power of two  */

typedef struct {
    uint32_t flags;      /* SS_SORT | SS_BIN | SS_FCR | SS_VBS | SS_COMPACT */
    int32_t  base_batch; /* B0: vanilla / minimum batch size, >= 1 (16 in the paper)            */
    int32_t  base_len;   /* L0 = global limit on generated tokens per query (L_max), >= 1       */
    int32_t  max_batch;  /* upper bound of the variable batch size, >= base_batch               */
    int32_t  vbs_rule;   /* SS_VBS_CLAMP_FLOOR or SS_VBS_PAPER_POW2                             */
} ss_policy;

/* A plan: micro-batch k holds queries query_idx[mb_offsets[k] .. mb_offsets[k+1]) and may generate at
 * most mb_cap[k] tokens per row.  query_idx lists each scheduled query exactly once.  All arrays are
 * host memory owned by the plan and immutable; free with ss_plan_free. */
typedef struct {
    int32_t        n;          /* number of scheduled queries       */
    int32_t        n_mb;       /* number of micro-batches           */
    const int32_t* mb_offsets; /* host, [n_mb + 1]                  */
    const int32_t* query_idx;  /* host, [n]                         */
    const int32_t* mb_cap;     /* host, [n_mb]                      */
} ss_plan;

/*
 * First-pass plan of a group (Sec. 4.1).  Pure host integer work, deterministic, no GPU needed.
 *   pred_lens  host, int32[n], predicted response length of each query (>= 1); may be NULL when
 *              SS_SORT is not set (vanilla: arrival order, chunks of base_batch, cap base_len).
 *   bin        bin cell size (50 in the paper); 0 = schedule by the raw prediction; must be > 0 with SS_BIN.
 * Scheduled length of a query = min(bin*ceil(pred/bin), bin*ceil(base_len/bin)) with SS_BIN, else pred.
 * Order: stable by (scheduled length, arrival index).  With SS_BIN every bin is chunked on its own
 * (batch size from the bin's edge; only a bin's last chunk is short).  Without SS_BIN the sorted list
 * is cut into chunks of base_batch, or with SS_VBS into the longest chunks whose size does not exceed
 * the batch size allowed for their largest prediction.  cap = min(largest scheduled length in the
 * micro-batch, base_len) with SS_FCR, else base_len.
 * Errors: SS_EINVAL for n <= 0, NULL out/policy, pred < 1, bin < 0, SS_BIN without SS_SORT or with bin 0,
 * SS_VBS without SS_SORT, base_batch < 1, max_batch < base_batch, base_len < 1, unknown vbs_rule; SS_ENOMEM when
 * the host cannot hold the plan.  *out is written only on success.
 */
int ss_schedule(const int32_t* pred_lens, int32_t n, int32_t bin, const ss_policy* policy, ss_plan** out);

/*
 * Plan of the recomputation pass (Sec. 4.1, FCR: failures are collected and recomputed at the end of
 * the group).  failed_idx (host, int32[n_failed], query indices < n) is ordered stably by
 * (scheduled length, index), cut into chunks of base_batch, cap = base_len, so nothing fails twice.
 * n_failed == 0 gives an empty plan.
 */
int ss_schedule_failures(const int32_t* pred_lens, int32_t n, const int32_t* failed_idx, int32_t n_failed,
                         int32_t bin, const ss_policy* policy, ss_plan** out);

void ss_plan_free(ss_plan* plan);

/* ------------------------------------------------------------------ model weights (device resident) */

typedef struct {
    int32_t n_layers, d_model, n_heads, head_dim, d_ffn, vocab;
    float   rope_base, rms_eps;
} ss_model_cfg;

typedef struct ss_weights ss_weights; /* opaque; owns packed bf16 weights and a grow-only device workspace */

#define SS_BF16 0 /* source tensors are bf16 bit patterns (uint16)            */
#define SS_F32  1 /* source tensors are fp32; rounded to bf16, nearest-even    */

/*
 * Upload and pack a LLaMA-style decoder (pre-norm, RMSNorm, rotary embedding pairing j with j+head_dim/2,
 * SwiGLU MLP, untied LM head, no biases; the model family of Sec. 4.2).
 *   tensors  host array of 3 + 9*n_layers host pointers, matrices [out, in] row-major, in this order:
 *            embed[vocab,d]; per layer attn_norm[d], wq[d,d], wk[d,d], wv[d,d], wo[d,d], mlp_norm[d],
 *            wg[ffn,d], wu[ffn,d], wd[d,ffn]; final_norm[d]; lm_head[vocab,d].
 *            The caller keeps ownership; the data is copied.
 * Requires n_heads*head_dim == d_model, head_dim in {64, 128}, d_model % 64 == 0 and <= 8192, d_ffn % 16 == 0,
 * vocab % 16 == 0.
 * Precision: weights are bf16 values (fp32 sources are rounded to bf16, nearest-even), held on the device as
 * IEEE half: the same number for 2^-17 <= |w| <= 65504, rounded to a multiple of 2^-24 below that, saturated
 * above.  An activation that feeds a projection is rounded to IEEE half once (11 significand bits); accumulation,
 * softmax, normalisation and the residual stream are fp32; key/value cache slots are IEEE half (2 bytes per
 * element).  Everything stored as half saturates at +-65504.  Source values must be finite: they are not checked.
 * A row whose logits are all NaN or -inf yields token id 0, never an id outside the vocabulary.
 * Errors: SS_EINVAL (shape), SS_EDEVICE (no usable GPU / HIP error), SS_ENOMEM.
 */
int  ss_weights_create(const ss_model_cfg* cfg, const void* const* tensors, int32_t src_dtype, ss_weights** out);
void ss_weights_destroy(ss_weights* w);

/*
 * Per-handle options.
 *   option SS_OPT_IN_FLIGHT, value = 1 .. SS_IN_FLIGHT_MAX: how many micro-batches of a group pass (ss_run_group,
 *   ss_run_group_generate) are generated at the same time.  The micro-batches of a pass (Sec. 4.1) are independent
 *   of each other, and a decode step of a few rows leaves the memory system idle between its kernels; with more than
 *   one the call hands the pass's micro-batches, longest cap first, to that many host threads, each with a stream, a
 *   workspace and a key/value cache of its own, so that one micro-batch's kernels run in the others' gaps (measured
 *   at the 7B shape, 16-row steps: 58 % of the HBM peak with one in flight, 69 % with two, 70 % with three, 72 %
 *   with four; on a whole group the third and fourth also shorten the tail at the end of a pass).  Every query's tokens
 *   are the same as with 1; only the order in which micro-batches finish changes.  The stream argument of the call
 *   is used for one of them; the others run on streams the handle owns.  The call returns when all are done.  Device
 *   time in the statistics is summed per micro-batch and so can exceed the wall time.  Device memory: one workspace
 *   and key/value cache per lane in use, each as large as the largest micro-batch that lane has run.
 * Errors: SS_EINVAL (NULL handle, unknown option, value out of range), SS_ESTATE (a call is in flight).
 */
#define SS_OPT_IN_FLIGHT 2
#define SS_IN_FLIGHT_MAX 4
#define SS_IN_FLIGHT_DEFAULT 4
int ss_set_option(ss_weights* w, int32_t option, int32_t value);

/* ------------------------------------------------------------------ generation */

typedef struct {
    int32_t steps;            /* forwards run: 1 prompt forward + steps-1 decode forwards                    */
    int32_t rows;             /* B                                                                            */
    int64_t row_steps;        /* rows actually computed, summed over forwards (B*steps without SS_COMPACT)   */
    int64_t prompt_tokens;    /* sum of prompt lengths                                                       */
    int64_t decode_kv_tokens; /* key/value slots read by decode attention, summed over rows and steps        */
    double  prefill_ms;       /* device time of the prompt forward (HIP events on the call's stream)         */
    double  decode_ms;        /* device time of all decode forwards                                          */
    int32_t polls;            /* ss_generate_microbatch: host reads of the device's unfinished-row count     */
    int32_t idle_steps;       /* ss_generate_microbatch: forwards run after the last row had finished        */
} ss_stats;

/*
 * Generate one micro-batch greedily (Sec. 4.1): the prompts are processed, then one token per row per
 * step until every row has emitted min(target_len, max_new) tokens; the token that the prompt forward
 * yields counts as the first generated one, so steps = min(max_new, max target_len).
 * End of sequence is simulated: row i is finished exactly when it has emitted target_lens[i] tokens.
 *   w               weights handle; one call at a time per handle (SS_ESTATE otherwise)
 *   prompt_tokens   host, int32[prompt_offsets[B]], ragged concatenation of the prompts, ids in [0, vocab)
 *   prompt_offsets  host, int32[B+1], strictly increasing from 0 (no empty prompt)
 *   max_new         cap on generated tokens per row, >= 1
 *   target_lens     host, int32[B], >= 1
 *   flags           0 or SS_COMPACT.  Without it a finished row keeps being computed on its own last
 *                   token until the micro-batch ends (the padding that vanilla batching pays for);
 *                   with it the live batch shrinks.  Lengths and flags are identical either way; tokens
 *                   are too, except where a row's two largest logits lie within the rounding difference
 *                   between two launch shapes (about 1e-3 of the largest logit) once the live batch has
 *                   shrunk past a multiple of 16 rows.
 *   out_tokens      host, int32[B*max_new] row-major; -1 after the emitted length
 *   out_lens        host, int32[B]   = min(target, max_new)
 *   out_failed      host, uint8[B]   = target > max_new  (an FCR failure: to be recomputed later)
 *   stats           host, nullable
 *   hip_stream      a hipStream_t to run on, or NULL for the handle's own stream
 * Errors: SS_EINVAL (B <= 0, NULL, bad offsets/ids/lengths, prompt + max_new > 4096 positions),
 *         SS_ENOMEM, SS_EDEVICE, SS_ESTATE.
 */
int ss_decode_microbatch(ss_weights* w, const int32_t* prompt_tokens, const int32_t* prompt_offsets, int32_t B,
                         int32_t max_new, const int32_t* target_lens, uint32_t flags, int32_t* out_tokens,
                         int32_t* out_lens, uint8_t* out_failed, ss_stats* stats, void* hip_stream);

/*
 * ss_decode_microbatch for callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): same arguments, same results, but the whole device workspace
 * (activations, partial sums, the micro-batch's key/value cache, bookkeeping tables) is laid out inside one
 * static device array of SS_STATIC_SCRATCH_BYTES that the library holds on every GPU it is loaded on until
 * the process ends.  The call allocates and frees no device memory and creates no stream or event.
 *   - A call whose workspace does not fit returns SS_EINVAL with a message that gives the bytes needed and the
 *     bytes available; nothing has run then.  Roughly: activations and partial sums for sum(prompt lengths)
 *     token-rows plus n_layers * 2 * d_model * 2 bytes per key/value slot, sum(prompt length + max_new) slots.
 *   - The array keeps the previous call's bytes; the call clears what must read as zero itself.
 *   - Every static call on one GPU uses that GPU's one array: a second static call on the same GPU while one is
 *     running (another handle, another thread) is refused with SS_ESTATE; calls that bypass that check race.
 *   - ss_decode_microbatch and every other entry point are unaffected and may follow or precede it freely.
 */
#define SS_STATIC_SCRATCH_BYTES (64u << 20)
int ss_decode_microbatch_static(ss_weights* w, const int32_t* prompt_tokens, const int32_t* prompt_offsets, int32_t B,
                                int32_t max_new, const int32_t* target_lens, uint32_t flags, int32_t* out_tokens,
                                int32_t* out_lens, uint8_t* out_failed, ss_stats* stats, void* hip_stream);

/*
 * Teacher-forced logits (test / measurement entry point).  Each of the B rows is a token sequence
 * tokens[offsets[i] .. offsets[i+1]); the first n_prompt[i] tokens are processed in one prompt forward,
 * the remaining ones are fed one per decode step (all rows advance together, exactly as in
 * ss_decode_microbatch, but the next input is the given token instead of the argmax).
 *   logits_out  host, float32, one [vocab] row per position >= n_prompt[i]-1 of every row, ordered by
 *               row then position: sum_i (len_i - n_prompt[i] + 1) rows.
 *   n_prompt    host, int32[B], 1 <= n_prompt[i] <= len_i.  n_prompt[i] == len_i makes row i a pure
 *               prompt forward.
 *   all_prompt_logits  nonzero: n_prompt[i] must equal len_i and logits are returned for every position
 *               (len_i rows per sequence) - checks the prompt path position by position.
 */
int ss_forward_logits(ss_weights* w, const int32_t* tokens, const int32_t* offsets, int32_t B,
                      const int32_t* n_prompt, int32_t all_prompt_logits, float* logits_out, void* hip_stream);

typedef struct {
    int32_t n_mb_first, n_mb_failure; /* micro-batches in the first pass and in the recomputation pass */
    int32_t n_failed;                 /* queries that overran their cap in the first pass              */
    int64_t steps;                    /* forwards over both passes                                     */
    int64_t padded_row_steps;         /* sum over micro-batches of B*steps                             */
    int64_t computed_row_steps;       /* rows actually computed (== padded without SS_COMPACT)         */
    int64_t useful_tokens;            /* sum of target_lens: every query's tokens counted once         */
    int64_t prompt_tokens;            /* prompt tokens processed, recomputation included               */
    double  wall_ms;                  /* host wall time of the whole group, plan building excluded     */
    double  plan_ms;                  /* host time spent building the two plans                        */
    double  prefill_ms, decode_ms;    /* device time (HIP events) summed over micro-batches            */
    int64_t polls, idle_steps;        /* ss_run_group_generate: summed over micro-batches (see ss_stats) */
} ss_group_stats;

/*
 * Whole group (Sec. 4.1 pipeline without the length predictor): plan -> generate every micro-batch ->
 * collect failures, discard their partial output and key/value state -> recomputation pass.
 *   pred_lens   host, int32[n] or NULL (vanilla)
 *   out_tokens  host, int32[n*base_len] row-major, -1 after each query's length
 *   out_lens    host, int32[n] = target_lens on success
 * policy->flags & SS_COMPACT selects the compacting engine for every micro-batch.
 */
int ss_run_group(ss_weights* w, const int32_t* prompt_tokens, const int32_t* prompt_offsets, int32_t n,
                 const int32_t* target_lens, const int32_t* pred_lens, int32_t bin, const ss_policy* policy,
                 int32_t* out_tokens, int32_t* out_lens, ss_group_stats* stats, void* hip_stream);

/* ------------------------------------------------------------------ generation that ends by itself */

/*
 * How rows end and how tokens are chosen when the host does not know the response lengths in advance
 * (Sec. 4.2, Experimental Setting: responses are sampled at a temperature and end at the model's end-of-sequence token or at
 * the limit on new tokens).
 */
typedef struct {
    int32_t eos_id;             /* id that ends a row; it is emitted and counted.  -1 = no such id            */
    float   temperature;        /* 0 = greedy (largest logit, lowest index on ties); > 0 = draw from
                                   softmax(logits / temperature) by inverse CDF in vocabulary order:
                                   the smallest v whose cumulative probability exceeds the draw               */
    const float* draws;         /* host, float32, draws[i*draws_stride + s] in [0,1) is the draw for token
                                   number s of row (query) i.  NULL with temperature > 0: the draws come from
                                   the library's counter-based generator instead (seed, draw_ids below)        */
    int32_t draws_stride;       /* with draws: >= max_new (ss_generate_microbatch) / >= base_len
                                   (ss_run_group_generate)                                                    */
    uint64_t seed;              /* generator key.  The draw for token number s of the row with id q is
                                   (x0 >> 8) * 2^-24, x0 = first output word of Philox4x32-10 (Salmon et al.,
                                   "Parallel random numbers: as easy as 1, 2, 3", SC 2011) on the counter
                                   (s, q, 0, 0) under the key (seed mod 2^32, seed >> 32)                       */
    const int32_t* draw_ids;    /* host, int32 per row (query), >= 0, nullable: the id q of each row; NULL = the
                                   row's (query's) index.  A row keeps its draws wherever it is scheduled        */
    const int32_t* target_lens; /* host, int32 per row, nullable: a simulated end of sequence after that many
                                   tokens, whichever of it and eos_id comes first.  The host loop never looks
                                   at it: the device applies it, the host learns of it by polling             */
    int32_t sync_every;         /* decode forwards between two host reads of the device's count of unfinished
                                   rows, >= 1.  Rows that finish between reads leave the live batch at once
                                   on the device (SS_COMPACT) but keep their place in the launch grids until
                                   the next read; up to sync_every-1 forwards may run after the last row ended */
} ss_gen_opts;

/*
 * ss_decode_microbatch for rows that end by themselves: token choice per `opts`, a row ends when it emits
 * opts->eos_id, reaches its optional target length, or has emitted max_new tokens.  End detection, the
 * shrinking of the live batch and the sampling all run on the device; the host only polls a counter.
 * Given the same weights, prompts and draws the output of a row does not depend on flags, on sync_every or on
 * what the other rows hold; across batch compositions that change the launch shapes (the total prompt length,
 * the number of 16-row strips) logits agree to about 1e-3 of the largest, and a sampled token can differ where its
 * draw lies within that of an interval edge.
 *   out_lens    host, int32[B]: tokens emitted (the end-of-sequence token included)
 *   out_failed  host, uint8[B]: the row was still unfinished after max_new tokens (Sec. 4.1 failure)
 * Other arguments, ownership and errors as ss_decode_microbatch; additionally SS_EINVAL for a NULL opts,
 * eos_id outside [-1, vocab), temperature < 0 or not finite, sync_every < 1, draws given with
 * draws_stride < max_new or a draw outside [0,1), draw_ids[i] < 0, target_lens[i] < 1.
 */
int ss_generate_microbatch(ss_weights* w, const int32_t* prompt_tokens, const int32_t* prompt_offsets, int32_t B,
                           int32_t max_new, const ss_gen_opts* opts, uint32_t flags, int32_t* out_tokens,
                           int32_t* out_lens, uint8_t* out_failed, ss_stats* stats, void* hip_stream);

/*
 * ss_run_group for rows that end by themselves.  opts->draws, opts->draw_ids and opts->target_lens are indexed
 * by query (n rows, stride draws_stride >= policy->base_len), so a recomputed query sees the same draws and
 * repeats its first attempt before going on, except where a draw lies so close to an edge of its token's
 * probability interval that the rounding differences between two batch compositions (logits agree to about 1e-3 of
 * the largest) decide it the other way.  A query that is unfinished at a cap below
 * policy->base_len is collected and recomputed with cap = base_len; one that is unfinished at base_len is
 * complete (truncated there).  stats->useful_tokens = sum of out_lens.
 */
int ss_run_group_generate(ss_weights* w, const int32_t* prompt_tokens, const int32_t* prompt_offsets, int32_t n,
                          const int32_t* pred_lens, int32_t bin, const ss_policy* policy, const ss_gen_opts* opts,
                          int32_t* out_tokens, int32_t* out_lens, ss_group_stats* stats, void* hip_stream);

/*
 * Measurement entry point: time `iters` decode forwards of B rows whose key/value history holds `ctx`
 * tokens each (synthetic state: every row is first prefilled with a ctx-token prompt taken from
 * `prompt_tokens`, host int32[B*ctx]).  The same kernels and launch configuration as a decode step of
 * ss_decode_microbatch, replayed on the same positions so that every iteration moves the same bytes.
 *   ms_out  host, double[iters]: device time of each forward (HIP events on the stream used).
 */
int ss_bench_decode_step(ss_weights* w, const int32_t* prompt_tokens, int32_t B, int32_t ctx, int32_t iters,
                         double* ms_out, void* hip_stream);

/*
 * Measurement entry point: ss_bench_decode_step on `lanes` lanes at once (1 .. SS_IN_FLIGHT_MAX), as a group pass
 * with SS_OPT_IN_FLIGHT = lanes runs that many micro-batches: each of `lanes` host threads prefills its own B rows of
 * ctx tokens on its own stream, all wait for each other, then each times `iters` decode forwards.
 *   ms_out  host, double[lanes*iters]: lane 0's forwards, then lane 1's, ... (device time of each, HIP events on
 *           that lane's stream).  Every lane streams the whole model once per forward.
 */
int ss_bench_decode_steps_in_flight(ss_weights* w, const int32_t* prompt_tokens, int32_t B, int32_t ctx, int32_t iters,
                                    int32_t lanes, double* ms_out);

/*
 * Measurement entry point: the projection kernels of one decode step alone.  Launches, back to back on
 * one stream, exactly the matrix kernels a B-row decode forward launches (per layer q|k|v, o, gate|up
 * with the SwiGLU epilogue, down; then the LM head) with the same launch configuration, on whatever the
 * activation buffers currently hold, `iters` times.  Every weight byte of the model is streamed once per
 * iteration, so bytes/iteration = the model's weight bytes.  ms_out: host, double[iters], device time of
 * each iteration (HIP events).  launches_out: host, nullable, number of kernel launches per iteration.
 */
int ss_bench_weight_stream(ss_weights* w, int32_t B, int32_t iters, double* ms_out, int32_t* launches_out,
                           void* hip_stream);

/*
 * Measurement entry point: the ceiling ss_bench_weight_stream is compared with.  Launches, back to back on one
 * stream, one plain read kernel per weight matrix in the order a decode forward uses them (per layer q|k|v, o,
 * gate|up, down; then the LM head): the same bytes in the same launch sizes, nothing computed, `iters` times.
 *   ms_out     host, double[iters], device time of each iteration (HIP events)
 *   bytes_out  host, nullable: bytes read per iteration (each matrix rounded down to whole 64 KiB chunks)
 */
int ss_bench_read_stream(ss_weights* w, int32_t iters, double* ms_out, int64_t* bytes_out, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* SS_H */
