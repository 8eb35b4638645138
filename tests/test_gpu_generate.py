"""GPU parity of generation that ends by itself (temperature sampling, a real end-of-sequence id, host
polling), through the C ABI, against the sampling oracle on the same seeded prompts and draws.

A sampled token is a function of (logits, draw).  The logits are held to the bar of test_gpu_parity.py;
the function is held to the oracle's rule, and the two checks are made on every emitted position:

  (a) the choice given the logits: the oracle's rule (fp64 softmax, CDF in vocabulary order) applied to the
      GPU's own teacher-forced logits on the GPU's own prefix must give the emitted token whenever the
      draw is further from the edges of the chosen CDF interval than rounding can move them.  Where the
      test can rebuild the micro-batch the tokens came from, those logits are computed with the same launches
      (the same prompts in one prompt forward, decode forwards of at most 16 rows, whose per-row arithmetic
      does not depend on how many rows are fed): the very numbers the tokens were chosen from, delta =
      SAME_PATH_DELTA.  Otherwise they come from the same kernels run on a different batch composition (other
      k-splits, other summation order), measured below to differ by less than GPU_PATH_DELTA; logits that differ by at most delta
      move every probability by a factor within exp(+-2*delta/T) and hence any CDF value by at most
      (exp(2*delta/T) - 1)/4; SUM_SLACK covers the kernel's fp32 summation.  For T = 0 the top-2 margin
      must exceed 2*delta.
  (b) end to end: the same with the oracle's logits and delta = the measured max |gpu - oracle| logit
      difference of that row (which must itself meet the logit bar).  On random-init models this decides
      few positions; they must match, and their number is reported.

Lengths, failure flags, -1 padding and counters are bit-exact against what the row's own tokens imply,
and against the oracle's whole result for rows decided at every position.
"""
import math

import numpy as np
import pytest

from paper_2305_13144_amd import binding as ss
from paper_2305_13144_amd import synth
from oracle import sampling_oracle as sm
from oracle import sched_oracle as so
from oracle.model_oracle import OracleModel

from test_gpu_parity import LOGIT_TOL, MARGIN, _say

pytestmark = pytest.mark.gpu

SUM_SLACK = 1e-5        # fp32 summation of the CDF in the kernel against fp64 in the oracle
# Logits of one prefix computed in two batch compositions, per unit of max |logit| (asserted below): other kernels sum
# in another order, which can move an activation to the neighbouring half-precision value (2^-11 relative).
GPU_PATH_DELTA = 1e-3
SAME_PATH_DELTA = 1e-6  # the same launches and per-row arithmetic as the run that chose the tokens


@pytest.fixture(scope="module")
def tiny(oracle_built):
    W = synth.make_weights(synth.TINY, seed=1, norm_jitter=0.1, threads=1)
    gw = ss.Weights(synth.TINY, W)
    yield W, OracleModel(synth.TINY, W, "f64"), gw
    gw.close()


def undecided_band(delta, T):
    """Margin below which two evaluations whose logits differ by at most delta may choose differently."""
    return 2 * delta if T == 0 else (math.exp(2 * delta / T) - 1) / 4 + SUM_SLACK


def microbatch_logits(gw, prompts, rows_tokens):
    """GPU logits of every row of one micro-batch (at most 16 rows, in their scheduled order) on its own emitted
    prefix, from ONE teacher-forced call: list of [len(tokens_i), vocab] arrays."""
    assert len(prompts) <= 16
    seqs = [np.concatenate([p, t[:len(t) - 1]]).astype(np.int32) for p, t in zip(prompts, rows_tokens)]
    offs = np.concatenate([[0], np.cumsum([len(q) for q in seqs])]).astype(np.int32)
    got = ss.ss_forward_logits(gw, np.concatenate(seqs), offs, np.array([len(p) for p in prompts], np.int32))
    cuts = np.cumsum([len(t) for t in rows_tokens])
    assert got.shape[0] == cuts[-1]
    return [g.astype(np.float64) for g in np.split(got, cuts[:-1])]


def group_logits(gw, w, tokens, lens, plan, failure_plan, wanted):
    """microbatch_logits for the queries in `wanted` of a scheduled group: each query with the micro-batch that
    produced its final tokens (first pass, or the recomputation pass if it overran its cap).  A co-scheduled row
    that failed in the first pass is fed its final tokens up to the cap: what it is fed only decides how long it
    stays in the forwards, never another row's logits."""
    out = {}
    done_first = set()
    for mbs, final_pass in ((plan, False), (failure_plan, True)):
        for mb in mbs:
            mine = [q for q in mb.idx if q in wanted and q not in out and (final_pass or int(lens[q]) <= mb.cap)]
            if not mine:
                continue
            rows = [tokens[q, :min(int(lens[q]), mb.cap)] for q in mb.idx]
            got = microbatch_logits(gw, [w.prompt(q) for q in mb.idx], rows)
            for q in mine:
                out[q] = got[mb.idx.index(q)]
    assert set(out) == set(wanted)
    return out


def check_row_on_own_prefix(om, gw, prompt, toks, T, draws, what, got=None):
    """Checks (a) and (b) of the header on every emitted token of one row.  got: the row's GPU logits from the
    launches that chose its tokens (microbatch_logits); None: they are computed here, the row alone.
    Returns (decided given the GPU's logits, decided end to end, positions)."""
    L = len(toks)
    seq = np.concatenate([prompt, toks[:L - 1]]).astype(np.int32) if L > 1 else np.asarray(prompt, np.int32)
    ref = om.teacher_forced(seq, first=len(prompt) - 1)
    assert ref.shape[0] == L
    path_delta = GPU_PATH_DELTA if got is None else SAME_PATH_DELTA
    if got is None:
        got = ss.ss_forward_logits(gw, seq, [0, len(seq)], [len(prompt)]).astype(np.float64)
    assert got.shape == ref.shape
    delta = float(np.abs(got - ref).max())
    assert delta <= LOGIT_TOL * np.abs(ref).max(), what
    given = end2end = 0
    for s in range(L):
        u = float(draws[s]) if T > 0 else 0.0
        tok, mg = sm.sample_token(got[s], T, u)
        if mg > undecided_band(path_delta * max(1.0, float(np.abs(got).max())), T):
            given += 1
            assert tok == toks[s], (what, "given the logits", s, tok, int(toks[s]), mg)
        tok, mg = sm.sample_token(ref[s], T, u)
        if mg > undecided_band(delta, T):
            end2end += 1
            assert tok == toks[s], (what, "end to end", s, tok, int(toks[s]), mg, delta)
    return given, end2end, L


def implied_end(toks_row, eos, cap, target=None):
    """(length, failed) that a row's own emitted tokens imply."""
    hits = np.flatnonzero(toks_row[:cap] == eos) if eos >= 0 else np.zeros(0, int)
    length = cap
    ended = False
    if len(hits):
        length, ended = int(hits[0]) + 1, True
    if target is not None and target <= length:
        length, ended = int(target), True
    return length, not ended


def polling_protocol(lens, cap, sync):
    """(forwards, polls) of a host that reads the unfinished-row count after the prompt forward and then after
    every `sync`-th decode forward (never after the last possible one), and stops on reading zero."""
    seen = int((np.asarray(lens) > 1).sum())
    forwards = polls = 1
    g = 1
    while g < cap and seen > 0:
        forwards += 1
        if g % sync == 0 and g + 1 < cap:
            polls += 1
            seen = int((np.asarray(lens) > g + 1).sum())
        g += 1
    return forwards, polls


# ------------------------------------------------------------------ sampling
@pytest.mark.parametrize("T", [1.0, 0.5, 0.1])
def test_tiny_sampled_microbatch_own_prefix(tiny, T):
    """16 ragged rows, 24 sampled tokens each, no end id: every decided position matches the oracle."""
    W, om, gw = tiny
    w = synth.make_workload(1)
    cap = 24
    draws = synth.make_draws(w.n, cap, seed=500 + int(T * 10))
    _say(f"tiny sampled micro-batch T={T}")
    r = ss.ss_generate_microbatch(gw, w.prompt_tokens, w.prompt_offsets, cap, eos_id=-1, temperature=T, draws=draws,
                                  sync_every=5)
    assert (r["lens"] == cap).all() and r["failed"].all()
    assert r["stats"]["steps"] == cap and r["stats"]["idle_steps"] == 0
    giv = e2e = tot = 0
    got = microbatch_logits(gw, [w.prompt(i) for i in range(w.n)], [r["tokens"][i] for i in range(w.n)])
    for i in range(w.n):
        g, e, L = check_row_on_own_prefix(om, gw, w.prompt(i), r["tokens"][i], T, draws[i], f"T={T} row {i}", got[i])
        giv, e2e, tot = giv + g, e2e + e, tot + L
    _say(f"  positions decided and equal: {giv}/{tot} given the logits, {e2e}/{tot} end to end")
    assert giv >= 0.8 * tot
    # the batch-composition difference that GPU_PATH_DELTA stands for: all rows together against one row alone
    seqs = [np.concatenate([w.prompt(i), r["tokens"][i, :cap - 1]]).astype(np.int32) for i in range(w.n)]
    offs = np.concatenate([[0], np.cumsum([len(q) for q in seqs])]).astype(np.int32)
    together = ss.ss_forward_logits(gw, np.concatenate(seqs), offs, w.prompt_lens)
    alone = ss.ss_forward_logits(gw, seqs[5], [0, len(seqs[5])], [int(w.prompt_lens[5])])
    path_delta = float(np.abs(together[5 * cap:6 * cap] - alone).max())
    _say(f"  same prefix in a batch of 16 and alone: max logit difference {path_delta:.2e}")
    assert path_delta <= GPU_PATH_DELTA * max(1.0, float(np.abs(alone).max()))
    # the choice is a function of (weights, prompt, draws) only: compaction flag, poll period and batch
    # composition change nothing
    r2 = ss.ss_generate_microbatch(gw, w.prompt_tokens, w.prompt_offsets, cap, eos_id=-1, temperature=T, draws=draws,
                                   sync_every=1, flags=ss.SS_COMPACT)
    assert np.array_equal(r2["tokens"], r["tokens"])
    sub = [3, 11]
    toks, offs = synth.gather_prompts(w, sub)
    r3 = ss.ss_generate_microbatch(gw, toks, offs, cap, eos_id=-1, temperature=T, draws=draws[sub], sync_every=24)
    agree = [(r3["tokens"][k] == r["tokens"][i]).all() for k, i in enumerate(sub)]
    _say(f"  rows re-run in a batch of 2: identical = {agree}")   # other kernels, other rounding: reported only


def test_sampler_distribution_peaked_and_flat_draws(tiny):
    """Draws at the extremes (0 and just below 1) and a low temperature: first and last tokens of the CDF."""
    W, om, gw = tiny
    w = synth.make_workload(1)
    cap = 6
    draws = np.zeros((w.n, cap), np.float32)
    draws[::2] = np.float32(1.0) - np.float32(2.0 ** -24)
    r = ss.ss_generate_microbatch(gw, w.prompt_tokens, w.prompt_offsets, cap, temperature=0.7, draws=draws)
    for i in range(w.n):
        check_row_on_own_prefix(om, gw, w.prompt(i), r["tokens"][i], 0.7, draws[i], f"extreme draws row {i}")
    # u = 0 always picks token 0 (its mass is positive); u -> 1 picks the last token with non-negligible mass
    assert (r["tokens"][1::2] == 0).all()
    assert (r["tokens"][::2] >= synth.TINY.vocab - 4).all()


def test_draws_on_the_edges_of_the_cdf_with_bit_equal_logits(tiny):
    """Every LM-head row identical -> all logits of a position are bit-equal -> every token has mass exactly 1/V, and
    with V a power of two the edges k/V of the CDF are exact in both precisions.  A draw equal to an edge must pick the
    token above it, the largest float below the edge the token under it (token v owns [c_{v-1}, c_v)); every token is
    compared with the oracle's rule on the same (all-equal) logits, with no undecided band."""
    W, om, gw = tiny
    V = synth.TINY.vocab
    assert V & (V - 1) == 0
    W2 = [t.copy() for t in W]
    W2[-1][:] = W2[-1][5]
    gw2 = ss.Weights(synth.TINY, W2)
    try:
        w = synth.make_workload(1)
        cap = 8
        rng = np.random.default_rng(77)
        ks = rng.integers(1, V, size=(w.n, cap))
        ks[0, :4] = [1, V - 1, V // 2, 3]
        draws = (ks / V).astype(np.float32)
        draws[:, 1::2] = np.nextafter(draws[:, 1::2], np.float32(0))       # odd token numbers: just under the edge
        draws[1, 0], draws[1, 2] = 0.0, np.nextafter(np.float32(1), np.float32(0))
        r = ss.ss_generate_microbatch(gw2, w.prompt_tokens, w.prompt_offsets, cap, temperature=0.5, draws=draws)
        want = np.array([[sm.sample_token(np.zeros(V), 0.5, float(draws[i, s]))[0] for s in range(cap)]
                         for i in range(w.n)], np.int32)
        assert want[0, :4].tolist() == [1, V - 2, V // 2, 2] and want[1, 0] == 0 and want[1, 2] == V - 1
        assert np.array_equal(r["lens"], np.full(w.n, cap)) and np.array_equal(r["tokens"], want)
    finally:
        gw2.close()


def test_generated_draws_equal_the_oracles_table(tiny):
    """Draws generated on the device from (seed, row id, token number) give exactly the tokens that the same call
    gives when it is handed the oracle's table of those draws: the two generators agree bit for bit."""
    W, om, gw = tiny
    w = synth.make_workload(1)
    cap, seed = 20, (0x1234ABCD << 32) | 0x9E3779B9
    for ids in (None, np.arange(w.n, dtype=np.int32)[::-1] * 1000 + 7):
        table = sm.generated_draws(seed, range(w.n) if ids is None else ids, cap)
        a = ss.ss_generate_microbatch(gw, w.prompt_tokens, w.prompt_offsets, cap, temperature=0.8, seed=seed,
                                      draw_ids=ids, target_lens=w.target_lens, flags=ss.SS_COMPACT, sync_every=2)
        b = ss.ss_generate_microbatch(gw, w.prompt_tokens, w.prompt_offsets, cap, temperature=0.8, draws=table,
                                      target_lens=w.target_lens, flags=ss.SS_COMPACT, sync_every=2)
        assert np.array_equal(a["tokens"], b["tokens"]) and np.array_equal(a["lens"], b["lens"])
        g, e, L = check_row_on_own_prefix(om, gw, w.prompt(2), a["tokens"][2, :int(a["lens"][2])], 0.8, table[2],
                                          "generated draws row 2")
        _say(f"  generated draws, ids {'default' if ids is None else 'given'}: row 2 decided {g}/{L}")
    other = ss.ss_generate_microbatch(gw, w.prompt_tokens, w.prompt_offsets, cap, temperature=0.8, seed=seed + 1,
                                      target_lens=w.target_lens, flags=ss.SS_COMPACT, sync_every=2)
    assert not np.array_equal(other["tokens"], a["tokens"])
    # in a scheduled group the id of a row is its query index, wherever the plan puts it, also when it is recomputed
    wg = synth.make_group(synth.TINY, 40, 555, ("uniform", 4, 20), ("lognormal", 10.0, 0.7, 1, 32), 0.3, 32, 8,
                          ("SORT", "BIN", "FCR", "VBS", "COMPACT"), base_batch=4, max_batch=16)
    pol = ss.make_policy(wg.flags, wg.base_batch, wg.l_max, wg.max_batch)
    table = sm.generated_draws(seed, range(wg.n), wg.l_max)
    a = ss.ss_run_group_generate(gw, wg.prompt_tokens, wg.prompt_offsets, wg.pred_lens, wg.bin_width, pol,
                                 temperature=0.8, seed=seed, target_lens=wg.target_lens, sync_every=1)
    b = ss.ss_run_group_generate(gw, wg.prompt_tokens, wg.prompt_offsets, wg.pred_lens, wg.bin_width, pol,
                                 temperature=0.8, draws=table, target_lens=wg.target_lens, sync_every=1)
    assert a["stats"]["n_failed"] >= 1 and np.array_equal(a["lens"], wg.target_lens)
    assert np.array_equal(a["tokens"], b["tokens"])


# ------------------------------------------------------------------ end-of-sequence id
@pytest.mark.parametrize("T,flags,sync", [(0.0, 0, 4), (0.0, ss.SS_COMPACT, 1), (0.1, ss.SS_COMPACT, 3), (0.1, 0, 8)])
def test_tiny_eos_ends_rows_at_different_steps(tiny, T, flags, sync):
    """The end id is the token the oracle's unbounded runs emit most often, so rows end at different, data
    dependent steps that the host does not know; some never end and fail at the cap."""
    W, om, gw = tiny
    w = synth.make_workload(1)
    cap = 28
    draws = synth.make_draws(w.n, cap, seed=600)
    free = [sm.generate_query(om, w.prompt(i), cap, -1, T, draws[i]) for i in range(w.n)]
    ids, counts = np.unique(np.concatenate([np.unique(f["tokens"]) for f in free]), return_counts=True)
    eos = int(ids[np.argmax(counts)])
    ends = [int(np.flatnonzero(f["tokens"] == eos)[0]) + 1 if (f["tokens"] == eos).any() else None for f in free]
    _say(f"tiny eos={eos} T={T} flags={flags} sync_every={sync}: oracle ends {ends}")
    assert sum(e is not None for e in ends) >= 3
    r = ss.ss_generate_microbatch(gw, w.prompt_tokens, w.prompt_offsets, cap, eos_id=eos, temperature=T, draws=draws,
                                  sync_every=sync, flags=flags)
    exact = giv = tot = 0
    got = microbatch_logits(gw, [w.prompt(i) for i in range(w.n)], [r["tokens"][i, :int(r["lens"][i])] for i in range(w.n)])
    for i in range(w.n):
        L = int(r["lens"][i])
        row = r["tokens"][i]
        # what the row's own tokens imply: bit-exact
        assert (row[:L] >= 0).all() and (row[L:] == -1).all()
        assert (L, bool(r["failed"][i])) == implied_end(row[:L], eos, cap), i
        assert (row[:L - 1] != eos).all()
        g, e, _ = check_row_on_own_prefix(om, gw, w.prompt(i), row[:L], T, draws[i], f"eos row {i}", got[i])
        giv, tot = giv + g, tot + L
        # a row decided end to end at every position: the oracle's whole result, bit-exact
        if e == L:
            ref = sm.generate_query(om, w.prompt(i), cap, eos, T, draws[i])
            exact += 1
            assert L == ref["length"] and bool(r["failed"][i]) == ref["failed"], i
            assert np.array_equal(row[:L], ref["tokens"]), i
    _say(f"  {giv}/{tot} positions decided given the logits and equal; {exact}/{w.n} rows decided end to end at every "
         f"position and bit-exact; lens {r['lens'].tolist()}")
    assert giv >= 0.8 * tot
    assert len(set(r["lens"].tolist())) >= 3
    st = r["stats"]
    longest = int(r["lens"].max())
    assert st["steps"] - longest == st["idle_steps"] and 0 <= st["idle_steps"] < sync
    assert (st["steps"], st["polls"]) == polling_protocol(r["lens"], cap, sync)
    if not flags:
        assert st["row_steps"] == w.n * st["steps"]
    else:
        assert st["row_steps"] <= w.n * st["steps"]
        if sync == 1:   # polled after every forward: exactly the rows that still owed a token were computed
            assert st["row_steps"] == sum(int(l) for l in r["lens"])


def test_tiny_all_rows_end_on_first_token(tiny):
    """Every row's first token is its end id's position 0 (target length 1): one forward, nothing to decode."""
    W, om, gw = tiny
    w = synth.make_workload(1)
    r = ss.ss_generate_microbatch(gw, w.prompt_tokens, w.prompt_offsets, 9, target_lens=np.ones(w.n, np.int32),
                                  flags=ss.SS_COMPACT)
    assert (r["lens"] == 1).all() and not r["failed"].any() and r["stats"]["steps"] == 1
    assert (r["tokens"][:, 1:] == -1).all()
    g = ss.ss_decode_microbatch(gw, w.prompt_tokens, w.prompt_offsets, 9, np.ones(w.n, np.int32))
    assert np.array_equal(g["tokens"], r["tokens"])


@pytest.mark.parametrize("flags", [0, ss.SS_COMPACT])
@pytest.mark.parametrize("sync", [1, 7])
def test_tiny_polled_target_lengths_equal_known_lengths(tiny, flags, sync):
    """Simulated ends applied by the device and discovered by polling give the tokens, lengths and failure
    flags of the entry point whose host knows the lengths (same kernels on the same rows: bit-exact)."""
    W, om, gw = tiny
    w = synth.make_workload(1)
    cap = 20
    known = ss.ss_decode_microbatch(gw, w.prompt_tokens, w.prompt_offsets, cap, w.target_lens, flags)
    r = ss.ss_generate_microbatch(gw, w.prompt_tokens, w.prompt_offsets, cap, target_lens=w.target_lens,
                                  sync_every=sync, flags=flags)
    assert np.array_equal(r["lens"], known["lens"]) and np.array_equal(r["failed"], known["failed"])
    assert np.array_equal(r["lens"], np.minimum(w.target_lens, cap))
    assert np.array_equal(r["failed"].astype(bool), w.target_lens > cap)
    if sync == 1 or not flags:
        assert np.array_equal(r["tokens"], known["tokens"])
    else:   # rows between polls ride in larger launches: other kernel variants, tokens may differ at near-ties
        same = (r["tokens"] == known["tokens"]).all(axis=1)
        _say(f"  rows identical to the known-length run: {int(same.sum())}/{w.n}")
    st = r["stats"]
    assert st["steps"] == known["stats"]["steps"] + st["idle_steps"] and st["idle_steps"] < sync
    assert (st["steps"], st["polls"]) == polling_protocol(r["lens"], cap, sync)


# ------------------------------------------------------------------ whole group
def test_tiny_group_generate_with_failures_and_recomputation(tiny):
    """A scheduled group whose rows end by sampled end ids or simulated ends: queries that overrun their
    bin's cap are collected and recomputed with the same draws."""
    W, om, gw = tiny
    w = synth.make_group(synth.TINY, 64, 4242, ("uniform", 4, 30), ("lognormal", 20.0, 0.7, 1, 64), 0.3, 64, 8,
                         ("SORT", "BIN", "FCR", "VBS", "COMPACT"), base_batch=4, max_batch=16)
    T = 0.1
    draws = synth.make_draws(w.n, w.l_max, seed=700)
    pol = ss.make_policy(w.flags, w.base_batch, w.l_max, w.max_batch)
    # the end id: the id that the oracle's forced-length runs of the first queries emit most often
    probe = [sm.generate_query(om, w.prompt(i), int(w.target_lens[i]), -1, T, draws[i],
                               target_len=int(w.target_lens[i])) for i in range(12)]
    ids, counts = np.unique(np.concatenate([p["tokens"] for p in probe]), return_counts=True)
    eos = int(ids[np.argmax(counts)])
    _say(f"tiny group of {w.n}, T={T}, eos={eos}")
    r = ss.ss_run_group_generate(gw, w.prompt_tokens, w.prompt_offsets, w.pred_lens, w.bin_width, pol, eos_id=eos,
                                 temperature=T, draws=draws, target_lens=w.target_lens, sync_every=4)
    gs = r["stats"]
    plan = so.schedule(w.pred_lens, w.n, w.bin_width,
                       so.Policy(flags=tuple(w.flags), base_batch=w.base_batch, l_max=w.l_max, max_batch=w.max_batch))
    cap_of = np.zeros(w.n, np.int64)
    for mb in plan:
        cap_of[np.asarray(mb.idx)] = mb.cap
    n_failed = 0
    decided = total = 0
    opol = so.Policy(flags=tuple(w.flags), base_batch=w.base_batch, l_max=w.l_max, max_batch=w.max_batch)
    overran = [i for i in range(w.n) if int(r["lens"][i]) > cap_of[i]]
    got = group_logits(gw, w, r["tokens"], r["lens"], plan, so.schedule_failures(w.pred_lens, overran, w.bin_width, opol),
                       set(range(0, w.n, 4)))
    for i in range(w.n):
        L = int(r["lens"][i])
        row = r["tokens"][i]
        assert (row[:L] >= 0).all() and (row[L:] == -1).all()
        length, failed = implied_end(row[:L], eos, w.l_max, int(w.target_lens[i]))
        assert L == length and not failed
        n_failed += L > cap_of[i]
        if i % 4 == 0:
            d, _, t = check_row_on_own_prefix(om, gw, w.prompt(i), row[:L], T, draws[i], f"group query {i}", got[i])
            decided += d
            total += t
    _say(f"  {decided}/{total} sampled positions decided given the logits and equal; failures {gs['n_failed']}, "
         f"polls {gs['polls']}, idle forwards {gs['idle_steps']}")
    assert gs["n_failed"] == n_failed and n_failed >= 1
    assert gs["useful_tokens"] == int(r["lens"].sum())
    assert gs["n_mb_first"] == len(plan)
    assert decided >= 0.8 * total
    # polled after every forward, the run is step for step the one the scheduler oracle accounts for when it is
    # given the lengths the rows turned out to have: forwards, padded and computed row-steps, failures, all exact
    r1 = ss.ss_run_group_generate(gw, w.prompt_tokens, w.prompt_offsets, w.pred_lens, w.bin_width, pol, eos_id=eos,
                                  temperature=T, draws=draws, target_lens=w.target_lens, sync_every=1)
    assert np.array_equal(r1["lens"], r["lens"])
    ref = so.run_group(w.pred_lens, r1["lens"], w.bin_width,
                       so.Policy(flags=tuple(w.flags), base_batch=w.base_batch, l_max=w.l_max, max_batch=w.max_batch))
    g1 = r1["stats"]
    assert g1["idle_steps"] == 0
    assert g1["steps"] == ref["steps"] and g1["padded_row_steps"] == ref["padded_row_steps"]
    assert g1["computed_row_steps"] == ref["live_row_steps"]
    assert g1["n_failed"] == ref["n_failed"] and g1["useful_tokens"] == ref["useful_tokens"]
    assert g1["n_mb_first"] == ref["first"].n_mb and g1["n_mb_failure"] == ref["second"].n_mb


def test_tiny_group_rows_without_any_end_are_truncated_at_the_global_limit(tiny):
    """No simulated lengths and an end id that almost never comes up (T = 1 over 1024 near-equal logits): a row
    that is unfinished at a cap below the global limit fails and is recomputed; unfinished at the global limit it
    is complete.  Every count equals the scheduler oracle's for the lengths the rows turned out to have."""
    W, om, gw = tiny
    w = synth.make_group(synth.TINY, 48, 909, ("uniform", 4, 16), ("uniform", 1, 24), 0.3, 24, 8,
                         ("SORT", "BIN", "FCR", "VBS", "COMPACT"), base_batch=4, max_batch=16)
    pol = ss.make_policy(w.flags, w.base_batch, w.l_max, w.max_batch)
    eos, seed = 77, 4242
    ids = np.arange(w.n, dtype=np.int32) * 3 + 11            # explicit draw ids, indexed by query
    r = ss.ss_run_group_generate(gw, w.prompt_tokens, w.prompt_offsets, w.pred_lens, w.bin_width, pol, eos_id=eos,
                                 temperature=1.0, seed=seed, draw_ids=ids, sync_every=1)
    table = sm.generated_draws(seed, ids, w.l_max)
    ended = 0
    for i in range(w.n):
        L = int(r["lens"][i])
        row = r["tokens"][i]
        assert (row[:L] >= 0).all() and (row[L:] == -1).all()
        length, unfinished = implied_end(row[:L], eos, w.l_max)
        assert L == length
        ended += not unfinished
    _say(f"  {ended}/{w.n} rows met the end id; the others ran to the global limit of {w.l_max}")
    assert (r["lens"] == w.l_max).sum() >= w.n // 2
    ref = so.run_group(w.pred_lens, r["lens"], w.bin_width,
                       so.Policy(flags=tuple(w.flags), base_batch=w.base_batch, l_max=w.l_max, max_batch=w.max_batch))
    got = group_logits(gw, w, r["tokens"], r["lens"], ref["plan"], ref["failure_plan"], {5})
    d, _, t = check_row_on_own_prefix(om, gw, w.prompt(5), r["tokens"][5, :int(r["lens"][5])], 1.0, table[5], "query 5",
                                      got[5])
    assert d >= 0.7 * t
    g = r["stats"]
    assert g["n_failed"] == ref["n_failed"] >= 1 and g["steps"] == ref["steps"]
    assert g["padded_row_steps"] == ref["padded_row_steps"] and g["computed_row_steps"] == ref["live_row_steps"]
    assert g["useful_tokens"] == int(r["lens"].sum()) == ref["useful_tokens"]


def test_caller_supplied_stream(tiny):
    """The entry points run on a stream the caller created (here through the HIP runtime the library links
    against) and return the same results as on the library's own stream."""
    import ctypes
    W, om, gw = tiny
    w = synth.make_workload(1)
    hip = ctypes.CDLL("libamdhip64.so")
    stream = ctypes.c_void_p()
    assert hip.hipStreamCreate(ctypes.byref(stream)) == 0
    try:
        a = ss.ss_decode_microbatch(gw, w.prompt_tokens, w.prompt_offsets, 12, w.target_lens, ss.SS_COMPACT)
        b = ss.ss_decode_microbatch(gw, w.prompt_tokens, w.prompt_offsets, 12, w.target_lens, ss.SS_COMPACT,
                                    stream=stream.value)
        assert np.array_equal(a["tokens"], b["tokens"]) and np.array_equal(a["lens"], b["lens"])
        c = ss.ss_generate_microbatch(gw, w.prompt_tokens, w.prompt_offsets, 12, temperature=0.6, seed=5,
                                      target_lens=w.target_lens, sync_every=2)
        d = ss.ss_generate_microbatch(gw, w.prompt_tokens, w.prompt_offsets, 12, temperature=0.6, seed=5,
                                      target_lens=w.target_lens, sync_every=2, stream=stream.value)
        assert np.array_equal(c["tokens"], d["tokens"])
        la = ss.ss_forward_logits(gw, w.prompt(0), [0, len(w.prompt(0))], [len(w.prompt(0))])
        lb = ss.ss_forward_logits(gw, w.prompt(0), [0, len(w.prompt(0))], [len(w.prompt(0))], stream=stream.value)
        assert np.array_equal(la, lb)
    finally:
        assert hip.hipStreamSynchronize(stream) == 0
        assert hip.hipStreamDestroy(stream) == 0


# ------------------------------------------------------------------ full-width vocabulary
def test_wide_sampled_tokens_vocab_32000(oracle_built):
    """7B widths at 2 layers: the sampler's chunking at vocab 32000 (1000 busy threads, 24 idle)."""
    shape = synth.LLAMA7B.with_layers(2)
    W = synth.make_weights(shape, seed=2, norm_jitter=0.05)
    gw = ss.Weights(shape, W)
    try:
        om = OracleModel(shape, W, "f64")
        w = synth.make_group(shape, 5, 99, ("uniform", 5, 12), ("uniform", 1, 4), None, 4, 0, ())
        cap = 4
        for T in (0.3, 0.05):
            draws = synth.make_draws(w.n, cap, seed=800)
            _say(f"wide sampled micro-batch, T={T}")
            r = ss.ss_generate_microbatch(gw, w.prompt_tokens, w.prompt_offsets, cap, temperature=T, draws=draws)
            dec = e2e = tot = 0
            got = microbatch_logits(gw, [w.prompt(i) for i in range(w.n)], [r["tokens"][i] for i in range(w.n)])
            for i in range(w.n):
                d, e, L = check_row_on_own_prefix(om, gw, w.prompt(i), r["tokens"][i], T, draws[i], f"wide T={T} row {i}",
                                                  got[i])
                dec, e2e, tot = dec + d, e2e + e, tot + L
            _say(f"  positions decided and equal: {dec}/{tot} given the logits, {e2e}/{tot} end to end")
            assert dec >= 0.6 * tot
    finally:
        gw.close()


# ------------------------------------------------------------------ argument checking
def test_generate_rejects_bad_options(tiny):
    W, om, gw = tiny
    w = synth.make_workload(1)
    ok = dict(eos_id=-1, temperature=0.5, draws=synth.make_draws(w.n, 8, seed=1), sync_every=2)

    def call(**kw):
        a = dict(ok)
        a.update(kw)
        return ss.ss_generate_microbatch(gw, w.prompt_tokens, w.prompt_offsets, 8, **a)

    call()
    for bad in (dict(eos_id=-2), dict(eos_id=synth.TINY.vocab), dict(temperature=-0.1), dict(temperature=float("nan")),
                dict(sync_every=0), dict(draws=synth.make_draws(w.n, 7, seed=1)),
                dict(target_lens=np.zeros(w.n, np.int32)), dict(draws=None, draw_ids=np.full(w.n, -1, np.int32))):
        with pytest.raises(ss.SsError) as e:
            call(**bad)
        assert e.value.code == ss.SS_EINVAL, bad
    d = synth.make_draws(w.n, 8, seed=1)
    d[3, 2] = 1.0
    with pytest.raises(ss.SsError):
        call(draws=d)
    # the handle is usable after every rejection
    assert call()["lens"].shape == (w.n,)
