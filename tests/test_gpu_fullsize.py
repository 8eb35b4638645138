"""GPU parity at the configured sizes: full-depth LLaMA-7B shape (configs 2-4), 13B widths (config 5),
the variable-batch-size row counts (up to 256 rows), and the whole scheduled group in the launch
configuration bench.py times.  The oracle cannot run a whole 7B group in reasonable time, so whole-group
results are checked by exact integer properties plus sampled outputs the oracle computes one by one
(teacher-forced on the GPU's own prefix; see test_gpu_parity.py for the bars)."""
import numpy as np
import pytest

from paper_2305_13144_amd import binding as ss
from paper_2305_13144_amd import synth
from oracle import sched_oracle as so
from oracle.model_oracle import OracleModel

from test_gpu_parity import (check_logits, check_tokens_teacher_forced, forced_batch, oracle_forced_logits, _say)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def full7b(oracle_built):
    shape = synth.LLAMA7B
    _say("generating full-depth 7B weights (seed 2)")
    W = synth.make_weights(shape, seed=2, threads=16)
    gw = ss.Weights(shape, W)
    yield shape, W, OracleModel(shape, W, "f64"), gw
    gw.close()


@pytest.fixture(scope="module")
def wide13(oracle_built):
    shape = synth.LLAMA13B.with_layers(2)
    W = synth.make_weights(shape, seed=5, norm_jitter=0.05, threads=16)
    gw = ss.Weights(shape, W)
    yield shape, W, OracleModel(shape, W, "f64"), gw
    gw.close()


def test_7b_full_depth_logits_teacher_forced(full7b):
    """32 layers: the logit error bar at the depth the benchmark runs at, prompt forward and decode steps."""
    shape, W, om, gw = full7b
    w = synth.make_workload(3)
    rng = np.random.default_rng(21)
    rows, extra = [3, 10, 17], [4, 0, 6]
    toks, offs, npr = forced_batch(w, rows, extra, rng)
    _say(f"7B x32 teacher-forced: prompts {npr.tolist()} + forced {extra}")
    got = ss.ss_forward_logits(gw, toks, offs, npr)
    ref = oracle_forced_logits(om, toks, offs, npr)
    check_logits(got, ref, "7B full depth")


def test_7b_config3_first_microbatches(full7b):
    """The first and a later micro-batch of config 3's plan, generated on the GPU; sampled rows re-derived by
    the oracle token by token."""
    shape, W, om, gw = full7b
    w = synth.make_workload(3)
    pol = ss.make_policy(w.flags, w.base_batch, w.l_max, w.max_batch)
    plan = ss.ss_schedule(w.pred_lens, w.n, w.bin_width, pol)
    for k in (0, 5):
        idx, cap = plan[k]
        toks, offs = synth.gather_prompts(w, idx)
        t = w.target_lens[idx]
        _say(f"config 3 micro-batch {k}: {len(idx)} rows, cap {cap}")
        r = ss.ss_decode_microbatch(gw, toks, offs, cap, t, 0)
        assert np.array_equal(r["lens"], np.minimum(t, cap))
        assert np.array_equal(r["failed"].astype(bool), t > cap)
        assert r["stats"]["steps"] == min(cap, int(t.max()))
        for j in (0, len(idx) - 1):
            L = int(r["lens"][j])
            assert (r["tokens"][j, :L] >= 0).all() and (r["tokens"][j, L:] == -1).all()
            dcd, tot = check_tokens_teacher_forced(om, w.prompt(idx[j]), r["tokens"][j, :L], upto=16, what=f"mb {k} row {j}")
            _say(f"  row {j}: {dcd}/{tot} decided positions match")


def test_7b_whole_group_config3_as_benchmarked(full7b):
    """ss_run_group on the full config-3 group, exactly what bench.py times."""
    shape, W, om, gw = full7b
    w = synth.make_workload(3)
    pol = ss.make_policy(w.flags, w.base_batch, w.l_max, w.max_batch)
    _say("7B whole group, config 3 (about half a minute on the GPU)")
    r = ss.ss_run_group(gw, w.prompt_tokens, w.prompt_offsets, w.target_lens, w.pred_lens, w.bin_width, pol)
    ref = so.run_group(w.pred_lens, w.target_lens, w.bin_width,
                       so.Policy(flags=w.flags, base_batch=w.base_batch, l_max=w.l_max, max_batch=w.max_batch))
    s = r["stats"]
    assert np.array_equal(r["lens"], w.target_lens)                       # every query emitted once, in full
    assert s["steps"] == ref["steps"] and s["padded_row_steps"] == ref["padded_row_steps"]
    assert s["n_failed"] == ref["n_failed"] and s["useful_tokens"] == ref["useful_tokens"] == int(w.target_lens.sum())
    assert (s["n_mb_first"], s["n_mb_failure"]) == (ref["first"].n_mb, ref["second"].n_mb)
    for i in range(w.n):
        t = int(w.target_lens[i])
        assert (r["tokens"][i, :t] >= 0).all() and (r["tokens"][i, :t] < shape.vocab).all()
        assert (r["tokens"][i, t:] == -1).all()
    failed = set(ref["first"].failed)
    ok = next(i for i in range(w.n) if i not in failed and w.target_lens[i] >= 4)
    redo = sorted(failed)[0]                                               # a query that went through recomputation
    for i in (ok, redo):
        dcd, tot = check_tokens_teacher_forced(om, w.prompt(i), r["tokens"][i, :int(w.target_lens[i])], upto=16,
                                               what=f"query {i}")
        _say(f"  query {i}: {dcd}/{tot} decided positions match")


def _check_group_against_scheduler_oracle(w, r, ref, vocab, compact):
    """Every counter of ss_group_stats against the scheduler oracle; every query emitted once, in full, -1 after."""
    s = r["stats"]
    assert np.array_equal(r["lens"], w.target_lens)
    assert s["steps"] == ref["steps"] and s["padded_row_steps"] == ref["padded_row_steps"]
    assert s["computed_row_steps"] == (ref["live_row_steps"] if compact else ref["padded_row_steps"])
    assert s["n_failed"] == ref["n_failed"] and s["useful_tokens"] == ref["useful_tokens"] == int(w.target_lens.sum())
    assert (s["n_mb_first"], s["n_mb_failure"]) == (ref["first"].n_mb, ref["second"].n_mb)
    prompts_run = int(w.prompt_lens.sum()) + sum(int(w.prompt_lens[i]) for i in ref["first"].failed)
    assert s["prompt_tokens"] == prompts_run                                 # recomputed queries pay their prompt twice
    for i in range(w.n):
        t = int(w.target_lens[i])
        assert (r["tokens"][i, :t] >= 0).all() and (r["tokens"][i, :t] < vocab).all()
        assert (r["tokens"][i, t:] == -1).all()


def test_7b_whole_group_config2_vanilla_as_benchmarked(full7b):
    """Config 2: the same 256 queries in arrival order, fixed batches of 16, every batch run to its longest
    response.  This is the denominator of the scheduled-over-vanilla ratio that bench.py reports."""
    shape, W, om, gw = full7b
    w = synth.make_workload(2)
    assert w.pred_lens is None and w.flags == ()
    pol = ss.make_policy((), w.base_batch, w.l_max, w.max_batch)
    _say("7B whole group, config 2 (vanilla batching; about 20 s on the GPU)")
    r = ss.ss_run_group(gw, w.prompt_tokens, w.prompt_offsets, w.target_lens, None, 0, pol)
    ref = so.run_group(None, w.target_lens, 0, so.Policy(flags=(), base_batch=w.base_batch, l_max=w.l_max,
                                                          max_batch=w.max_batch))
    _check_group_against_scheduler_oracle(w, r, ref, shape.vocab, compact=False)
    # the definition itself: 16 chunks of 16 in arrival order, each as long as its longest response
    t = w.target_lens
    assert r["stats"]["steps"] == sum(int(t[c:c + 16].max()) for c in range(0, w.n, 16))
    assert r["stats"]["n_failed"] == 0 and r["stats"]["n_mb_failure"] == 0
    short = sorted(range(w.n), key=lambda i: (int(w.prompt_lens[i]), i))
    picks = [next(i for i in short if t[i] >= 16), next(i for i in short if t[i] >= 16 and i >= 128)]
    for i in picks:
        dcd, tot = check_tokens_teacher_forced(om, w.prompt(i), r["tokens"][i, :int(t[i])], upto=16, what=f"query {i}")
        _say(f"  query {i}: {dcd}/{tot} decided positions match")


def test_7b_whole_group_config4_as_benchmarked(full7b):
    """ss_run_group on the full config-4 group (1024 queries, variable batch size up to 128 rows, compaction, prompt
    forwards of several thousand token-rows), exactly what `bench.py --cfg 4` times: every count against the
    scheduler oracle, every query emitted once and in full, sampled queries re-derived by the oracle."""
    shape, W, om, gw = full7b
    w = synth.make_workload(4)
    pol = ss.make_policy(w.flags, w.base_batch, w.l_max, w.max_batch)
    _say("7B whole group, config 4 (about 40 s on the GPU)")
    r = ss.ss_run_group(gw, w.prompt_tokens, w.prompt_offsets, w.target_lens, w.pred_lens, w.bin_width, pol)
    ref = so.run_group(w.pred_lens, w.target_lens, w.bin_width,
                       so.Policy(flags=w.flags, base_batch=w.base_batch, l_max=w.l_max, max_batch=w.max_batch))
    s = r["stats"]
    assert np.array_equal(r["lens"], w.target_lens)
    assert s["steps"] == ref["steps"] and s["padded_row_steps"] == ref["padded_row_steps"]
    assert s["computed_row_steps"] == ref["live_row_steps"]                # compaction: only rows that still owe tokens
    assert s["n_failed"] == ref["n_failed"] and s["useful_tokens"] == ref["useful_tokens"] == int(w.target_lens.sum())
    assert (s["n_mb_first"], s["n_mb_failure"]) == (ref["first"].n_mb, ref["second"].n_mb)
    for i in range(w.n):
        t = int(w.target_lens[i])
        assert (r["tokens"][i, :t] >= 0).all() and (r["tokens"][i, :t] < shape.vocab).all()
        assert (r["tokens"][i, t:] == -1).all()
    failed = set(ref["first"].failed)
    plan = so.schedule(w.pred_lens, w.n, w.bin_width,
                       so.Policy(flags=w.flags, base_batch=w.base_batch, l_max=w.l_max, max_batch=w.max_batch))
    big = max(plan, key=lambda mb: len(mb.idx))
    _say(f"  largest micro-batch: {len(big.idx)} rows, cap {big.cap}")
    in_big = next(i for i in big.idx if i not in failed and w.target_lens[i] >= 3)   # ran in the widest micro-batch
    redo = sorted(failed)[0]
    for i in (in_big, redo):
        dcd, tot = check_tokens_teacher_forced(om, w.prompt(i), r["tokens"][i, :int(w.target_lens[i])], upto=16,
                                               what=f"query {i}")
        _say(f"  query {i}: {dcd}/{tot} decided positions match")


def test_13b_widths_logits_and_vbs_batch(wide13):
    """Config 5's widths (d 5120, 40 heads, ffn 13824) at 2 layers: logits, then a 256-row micro-batch
    (its largest variable batch size) with compaction, sampled rows against the oracle."""
    shape, W, om, gw = wide13
    w = synth.make_workload(5, n=256, shape=shape)
    rng = np.random.default_rng(22)
    toks, offs, npr = forced_batch(w, [0, 1, 2], [2, 5, 0], rng)
    got = ss.ss_forward_logits(gw, toks, offs, npr)
    check_logits(got, oracle_forced_logits(om, toks, offs, npr), "13B widths")
    cap = 6
    t = np.minimum(w.target_lens, 9)
    _say("13B widths: 256-row micro-batch, cap 6, compaction on")
    r = ss.ss_decode_microbatch(gw, w.prompt_tokens, w.prompt_offsets, cap, t, ss.SS_COMPACT)
    assert np.array_equal(r["lens"], np.minimum(t, cap)) and np.array_equal(r["failed"].astype(bool), t > cap)
    assert r["stats"]["row_steps"] == int(np.minimum(t, cap).sum())
    for j in (0, 100, 255):
        check_tokens_teacher_forced(om, w.prompt(j), r["tokens"][j, :int(r["lens"][j])], what=f"row {j}")


@pytest.fixture(scope="module")
def full13b(oracle_built):
    shape = synth.LLAMA13B
    _say("generating full-depth 13B weights (seed 5)")
    W = synth.make_weights(shape, seed=5, threads=16)
    gw = ss.Weights(shape, W)
    yield shape, W, OracleModel(shape, W, "f64"), gw
    gw.close()


def test_13b_full_depth_config5_microbatch(full13b):
    """Config 5 at its real size: LLaMA-13B shape, 40 layers.  Teacher-forced logits, then the first
    micro-batch of its plan (the largest variable batch) generated with compaction; sampled rows re-derived
    by the oracle over their first 16 tokens."""
    shape, W, om, gw = full13b
    w = synth.make_workload(5)
    rng = np.random.default_rng(23)
    toks, offs, npr = forced_batch(w, [2, 9], [3, 0], rng)
    _say(f"13B x40 teacher-forced: prompts {npr.tolist()}")
    got = ss.ss_forward_logits(gw, toks, offs, npr)
    check_logits(got, oracle_forced_logits(om, toks, offs, npr), "13B full depth")
    pol = ss.make_policy(w.flags, w.base_batch, w.l_max, w.max_batch)
    plan = ss.ss_schedule(w.pred_lens, w.n, w.bin_width, pol)
    idx, cap = plan[0]
    ptoks, poffs = synth.gather_prompts(w, idx)
    t = w.target_lens[idx]
    _say(f"config 5 micro-batch 0: {len(idx)} rows, cap {cap}")
    r = ss.ss_decode_microbatch(gw, ptoks, poffs, cap, t, ss.SS_COMPACT)
    assert np.array_equal(r["lens"], np.minimum(t, cap))
    assert np.array_equal(r["failed"].astype(bool), t > cap)
    assert r["stats"]["row_steps"] == int(np.minimum(t, cap).sum())
    plen = poffs[1:] - poffs[:-1]
    long_rows = [j for j in np.argsort(plen, kind="stable") if r["lens"][j] >= 16][:4]   # shortest prompts: cheapest for the oracle
    assert len(long_rows) == 4
    for j in long_rows:
        L = int(r["lens"][j])
        dcd, tot = check_tokens_teacher_forced(om, w.prompt(idx[j]), r["tokens"][j, :L], upto=16, what=f"row {j}")
        _say(f"  row {j} (prompt {plen[j]}): {dcd}/{tot} decided positions match")


def test_13b_whole_group_config5_as_benchmarked(full13b):
    """ss_run_group on the full config-5 group (LLaMA-13B shape, 1024 queries, bins of 64, variable batch size up
    to 256 rows, compaction, recomputation pass), exactly what `bench.py --cfg 5` times."""
    shape, W, om, gw = full13b
    w = synth.make_workload(5)
    pol = ss.make_policy(w.flags, w.base_batch, w.l_max, w.max_batch)
    opol = so.Policy(flags=w.flags, base_batch=w.base_batch, l_max=w.l_max, max_batch=w.max_batch)
    _say("13B whole group, config 5 (about 100 s on the GPU)")
    ss.ss_set_verbose(1)
    try:
        r = ss.ss_run_group(gw, w.prompt_tokens, w.prompt_offsets, w.target_lens, w.pred_lens, w.bin_width, pol)
    finally:
        ss.ss_set_verbose(0)
    ref = so.run_group(w.pred_lens, w.target_lens, w.bin_width, opol)
    _check_group_against_scheduler_oracle(w, r, ref, shape.vocab, compact=True)
    failed = set(ref["first"].failed)
    big = max(ref["plan"], key=lambda mb: len(mb.idx))
    _say(f"  largest micro-batch: {len(big.idx)} rows, cap {big.cap}; {len(failed)} queries recomputed")
    by_prompt = lambda ids: sorted(ids, key=lambda i: (int(w.prompt_lens[i]), i))
    in_big = next(i for i in by_prompt(big.idx) if i not in failed and w.target_lens[i] >= 8)
    redo = next(i for i in by_prompt(failed) if w.target_lens[i] >= 16)
    for i in (in_big, redo):
        dcd, tot = check_tokens_teacher_forced(om, w.prompt(i), r["tokens"][i, :int(w.target_lens[i])], upto=16,
                                               what=f"query {i}")
        _say(f"  query {i}: {dcd}/{tot} decided positions match")


@pytest.mark.parametrize("rows", [163, 81, 54])
def test_7b_widths_variable_batch_sizes(rows, oracle_built):
    """Config 4's batch sizes for the 50/100/150-token bins at 7B widths (2 layers), compaction on and off."""
    shape = synth.LLAMA7B.with_layers(2)
    W = synth.make_weights(shape, seed=2, norm_jitter=0.05, threads=16)
    gw = ss.Weights(shape, W)
    om = OracleModel(shape, W, "f64")
    try:
        w = synth.make_workload(4, n=rows, shape=shape)
        t = np.minimum(w.target_lens, 7)
        for flags in (0, ss.SS_COMPACT):
            _say(f"7B widths: {rows}-row micro-batch flags={flags}")
            r = ss.ss_decode_microbatch(gw, w.prompt_tokens, w.prompt_offsets, 5, t, flags)
            assert np.array_equal(r["lens"], np.minimum(t, 5))
            for j in (0, rows // 2, rows - 1):
                check_tokens_teacher_forced(om, w.prompt(j), r["tokens"][j, :int(r["lens"][j])], what=f"row {j}")
    finally:
        gw.close()


def test_7b_full_depth_sampled_rows_that_end_by_themselves(full7b):
    """Full depth, vocabulary 32000, the launch configuration the benchmark's sampled leg runs: 16 rows sampled at
    T = 0.5 with device-side ends; every emitted token is the oracle's inverse-CDF choice on the GPU's own logits
    and prefix, lengths and flags are exact, and the logits themselves meet the bar."""
    from test_gpu_generate import check_row_on_own_prefix, microbatch_logits
    shape, W, om, gw = full7b
    w = synth.make_workload(3)
    idx = list(range(16))
    toks, offs = synth.gather_prompts(w, idx)
    cap = 6
    t = np.array([1, 2, 3, 4, 5, 6, 7, 8, 6, 6, 6, 6, 3, 3, 9, 1], np.int32)
    draws = synth.make_draws(16, cap, seed=31)
    _say("7B x32 sampled micro-batch with device-side ends")
    for T in (0.5, 0.05):
        r = ss.ss_generate_microbatch(gw, toks, offs, cap, temperature=T, draws=draws, target_lens=t, sync_every=2,
                                      flags=ss.SS_COMPACT)
        assert np.array_equal(r["lens"], np.minimum(t, cap))
        assert np.array_equal(r["failed"].astype(bool), t > cap)
        assert r["stats"]["steps"] == cap + 0 and r["stats"]["idle_steps"] == 0
        dec = tot = 0
        got = microbatch_logits(gw, [w.prompt(i) for i in idx], [r["tokens"][j, :int(r["lens"][j])] for j in range(16)])
        for j in (5, 14):
            L = int(r["lens"][j])
            assert (r["tokens"][j, :L] >= 0).all() and (r["tokens"][j, L:] == -1).all()
            g, e, L = check_row_on_own_prefix(om, gw, w.prompt(idx[j]), r["tokens"][j, :L], T, draws[j], f"7B T={T} row {j}",
                                              got[j])
            dec, tot = dec + g, tot + L
        _say(f"  T={T}: {dec}/{tot} positions decided given the logits and equal")
        if T < 0.1:
            assert dec >= 0.5 * tot
