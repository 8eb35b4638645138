"""Pins of the scheduler/accounting oracle: the values the paper prints, closed forms,
hand-enumerated small groups, invariants, and reductions to the vanilla schedule."""
import os

import numpy as np
import pytest

from paper_2305_13144_amd import synth
from oracle import sched_oracle as so


def _golden():
    out = {}
    path = os.path.join(os.path.dirname(__file__), "golden", "paper_values.txt")
    for line in open(path):
        line = line.strip()
        if line and not line.startswith("#"):
            k, v = [s.strip() for s in line.split("=")]
            out[k] = int(v)
    return out


G = _golden()


# ------------------------------------------------------------------ values printed in the paper
def test_paper_bin_cell_and_rounding():
    w = G["bin_cell"]
    assert [so.bin_upper(p, w, 512) for p in (1, 49, 50, 51, 100, 101, 499, 500)] == [50, 50, 50, 100, 100, 150, 500, 500]
    # predictions beyond the global limit land in the bin that holds the limit
    assert so.bin_upper(501, w, 512) == 550 and so.bin_upper(9999, w, 512) == 550
    assert so.bin_upper(2000, 64, 1024) == 1024


def test_paper_vbs_pow2_rule():
    thr = G["vbs_pow2_threshold"]
    assert so.vbs_paper_pow2(thr) == G["vbs_pow2_at_or_above_threshold"]
    assert so.vbs_paper_pow2(thr + 200) == G["vbs_pow2_at_or_above_threshold"]
    assert so.vbs_paper_pow2(50) == G["vbs_pow2_L50"]
    assert so.vbs_paper_pow2(100) == G["vbs_pow2_L100"]
    assert so.vbs_paper_pow2(200) == G["vbs_pow2_L200"]
    assert so.vbs_paper_pow2(150) == 64          # 85.3 lies nearer 64 than 128
    assert so.vbs_paper_pow2(250) == 64          # 51.2 lies nearer 64 than 32
    outs = [so.vbs_paper_pow2(L) for L in range(50, 300, 50)]
    assert all(a >= b for a, b in zip(outs, outs[1:]))     # larger batches for shorter responses


def test_paper_vbs_pow2_rule_is_the_nearest_power_of_two_by_brute_force():
    """Sec. 4.2: below 300 the batch size is 256*50/L rounded to the nearest power of two.  For every L the result
    must be the power of two closest to 12800/L among all of them, found here by trying each one in exact rational
    arithmetic (no L makes two of them equally close: 12800/L = 1.5 * 2^k has no integer solution)."""
    from fractions import Fraction
    powers = [2 ** k for k in range(0, 15)]
    for L in range(1, 300):
        x = Fraction(256 * 50, L)
        dist = sorted((abs(x - b), b) for b in powers)
        assert dist[0][0] != dist[1][0]
        assert so.vbs_paper_pow2(L) == dist[0][1], L
    # the places where the constant shows: 12800/260 = 49.2 is nearer 64 (a numerator of 12288 would say 32)
    assert so.vbs_paper_pow2(260) == 64 and so.vbs_paper_pow2(270) == 32
    assert so.vbs_paper_pow2(130) == 128 and so.vbs_paper_pow2(134) == 64


# ------------------------------------------------------------------ closed forms of the configured rule
def test_vbs_clamp_floor_tables():
    got = [so.vbs_clamp_floor(ub, 16, 512, 256) for ub in range(50, 600, 50)]
    assert got == [163, 81, 54, 40, 32, 27, 23, 20, 18, 16, 16]
    got = [so.vbs_clamp_floor(ub, 16, 1024, 256) for ub in range(64, 64 * 9, 64)]
    assert got == [256, 128, 85, 64, 51, 42, 36, 32]
    assert so.vbs_clamp_floor(1024, 16, 1024, 256) == 16 and so.vbs_clamp_floor(10, 16, 512, 256) == 256
    # constant tokens per batch: B*L never exceeds B0*L_max unless the lower clamp is active
    for ub in range(50, 600, 50):
        b = so.vbs_clamp_floor(ub, 16, 512, 256)
        assert b * ub <= 16 * 512 or b == 16


# ------------------------------------------------------------------ a group enumerated by hand
PRED = [30, 120, 55, 49, 260, 51, 100, 7]
TRUE = [40, 130, 101, 50, 250, 60, 99, 3]


def test_hand_enumerated_binned_fcr_group():
    pol = so.Policy(flags=("SORT", "BIN", "FCR"), base_batch=2, l_max=512, max_batch=256)
    plan = so.schedule(PRED, 8, 50, pol)
    # bins: 50 -> {0,3,7}, 100 -> {2,5,6}, 150 -> {1}, 300 -> {4}; chunks of 2 inside each bin
    assert [(m.idx, m.cap) for m in plan] == [([0, 3], 50), ([7], 50), ([2, 5], 100), ([6], 100), ([1], 150), ([4], 300)]
    r = so.run_group(PRED, TRUE, 50, pol)
    assert [m["steps"] for m in r["first"].per_mb] == [50, 3, 100, 99, 130, 250]
    assert r["first"].failed == [2]                       # 101 > 100
    assert r["first"].padded_row_steps == 782 and r["first"].live_row_steps == 732
    assert [(m.idx, m.cap) for m in r["failure_plan"]] == [([2], 512)]
    assert r["second"].steps == 101 and r["second"].padded_row_steps == 101
    assert r["steps"] == 733 and r["useful_tokens"] == 733 and r["n_failed"] == 1
    assert r["padded_row_steps"] == 883
    assert r["avg_len_weighted"] == pytest.approx(883 / 9)


def test_hand_enumerated_vanilla_group():
    pol = so.Policy(flags=(), base_batch=2, l_max=512)
    r = so.run_group(None, TRUE, 0, pol)
    assert [(m.idx, m.cap) for m in r["plan"]] == [([0, 1], 512), ([2, 3], 512), ([4, 5], 512), ([6, 7], 512)]
    assert [m["steps"] for m in r["first"].per_mb] == [130, 101, 250, 99]
    assert r["padded_row_steps"] == 1160 and r["n_failed"] == 0
    assert r["redundancy"] == pytest.approx(1 - 733 / 1160)


def test_predictions_without_the_sort_flag_are_ignored():
    """The vanilla baseline of Sec. 4.2 batches in arrival order even when predictions are at hand."""
    pol = so.Policy(flags=(), base_batch=3, l_max=64)
    plan = so.schedule(PRED, len(PRED), 50, pol)
    assert [(m.idx, m.cap) for m in plan] == [([0, 1, 2], 64), ([3, 4, 5], 64), ([6, 7], 64)]


def test_hand_enumerated_sorted_fcr_without_bins():
    pol = so.Policy(flags=("SORT", "FCR"), base_batch=3, l_max=512)
    plan = so.schedule(PRED, 8, 0, pol)
    # sorted by prediction: 7(7) 0(30) 3(49) | 5(51) 2(55) 6(100) | 1(120) 4(260); cap = largest prediction in the chunk
    assert [(m.idx, m.cap) for m in plan] == [([7, 0, 3], 49), ([5, 2, 6], 100), ([1, 4], 260)]
    a = so.account(plan, TRUE)
    assert a.failed == [3, 2]                             # 50 > 49 and 101 > 100; 130 and 250 fit under 260


def test_hand_enumerated_vbs_bins():
    pol = so.Policy(flags=("SORT", "BIN", "FCR", "VBS"), base_batch=2, l_max=100, max_batch=4)
    pred = [10, 20, 30, 40, 50, 60, 70, 80, 90, 100, 45, 5]
    plan = so.schedule(pred, len(pred), 50, pol)
    # bin 50 holds {0,1,2,3,4,10,11}: batch = clamp(floor(2*100/50), 2, 4) = 4 -> chunks of 4 and 3
    # bin 100 holds {5,6,7,8,9}:      batch = clamp(floor(2*100/100), 2, 4) = 2 -> 2, 2, 1
    assert [(m.idx, m.cap) for m in plan] == [([0, 1, 2, 3], 50), ([4, 10, 11], 50), ([5, 6], 100), ([7, 8], 100), ([9], 100)]


# ------------------------------------------------------------------ the recomputation pass, enumerated by hand
# Several failures whose (scheduled length, index) order is not their index order: Sec. 4.1 collects the failures
# and recomputes them after the group; they are re-batched in the order of their scheduled length.
PRED_F = [260, 30, 120, 55, 49, 110, 20, 210]
TRUE_F = [400, 60, 100, 180, 50, 300, 10, 205]


def test_hand_enumerated_failure_pass_order_with_bins():
    pol = so.Policy(flags=("SORT", "BIN", "FCR"), base_batch=2, l_max=512, max_batch=256)
    r = so.run_group(PRED_F, TRUE_F, 50, pol)
    # bins: 50 -> {1,4,6}, 100 -> {3}, 150 -> {2,5}, 250 -> {7}, 300 -> {0}
    assert [(m.idx, m.cap) for m in r["plan"]] == [([1, 4], 50), ([6], 50), ([3], 100), ([2, 5], 150), ([7], 250), ([0], 300)]
    assert [m["steps"] for m in r["first"].per_mb] == [50, 10, 100, 150, 205, 300]
    assert r["first"].steps == 815 and r["first"].padded_row_steps == 1015 and r["first"].live_row_steps == 965
    # 60 > 50, 180 > 100, 300 > 150, 400 > 300 fail; 50 <= 50 does not
    assert sorted(r["first"].failed) == [0, 1, 3, 5]
    # by (bin edge, index): 1 (50), 3 (100), 5 (150), 0 (300); batches of 2; the short rows share a batch
    assert [(m.idx, m.cap) for m in r["failure_plan"]] == [([1, 3], 512), ([5, 0], 512)]
    assert [m["steps"] for m in r["second"].per_mb] == [180, 400]
    assert r["second"].steps == 580 and r["second"].padded_row_steps == 1160      # index order would cost 400 + 300
    assert r["steps"] == 1395 and r["useful_tokens"] == 1305 and r["n_failed"] == 4
    # Sec. 4.2's metrics, by hand: 4 of the 8 queries failed; every row-step of both passes is paid for
    # (1015 + 1160 = 2175), of which 1305 produced a token that is kept (the failed rows' first attempts, 50 + 100 +
    # 150 + 300 row-steps, are thrown away, so they count as waste although they were "live")
    assert r["failure_ratio"] == 4 / 8
    assert r["padded_row_steps"] == 2175 and r["live_row_steps"] == 965 + 940
    assert r["redundancy"] == 1.0 - 1305 / 2175
    assert r["avg_len_weighted"] == 2175 / 12 and r["avg_len_unweighted"] == 1395 / 8
    # the order does not depend on the order the failures are handed over in
    for given in ([0, 1, 3, 5], [5, 3, 1, 0], [3, 0, 5, 1]):
        assert [m.idx for m in so.schedule_failures(PRED_F, given, 50, pol)] == [[1, 3], [5, 0]]


def test_hand_enumerated_failure_pass_order_without_bins_and_ties():
    pol = so.Policy(flags=("SORT", "FCR"), base_batch=2, l_max=512)
    r = so.run_group(PRED_F, TRUE_F, 0, pol)
    # sorted by prediction: 6(20) 1(30) | 4(49) 3(55) | 5(110) 2(120) | 7(210) 0(260)
    assert [(m.idx, m.cap) for m in r["plan"]] == [([6, 1], 30), ([4, 3], 55), ([5, 2], 120), ([7, 0], 260)]
    assert sorted(r["first"].failed) == [0, 1, 3, 5]
    assert [(m.idx, m.cap) for m in r["failure_plan"]] == [([1, 3], 512), ([5, 0], 512)]
    assert r["second"].steps == 180 + 400
    # equal scheduled lengths: the arrival index decides (stable), whatever order the list comes in
    pred = [80, 70, 80, 70, 60]
    plan = so.schedule_failures(pred, [4, 2, 0, 3, 1], 50, so.Policy(flags=("SORT", "BIN", "FCR"), base_batch=2, l_max=512))
    assert [(m.idx, m.cap) for m in plan] == [([0, 1], 512), ([2, 3], 512), ([4], 512)]   # one bin (100): index order
    plan = so.schedule_failures(pred, [4, 2, 0, 3, 1], 0, so.Policy(flags=("SORT", "FCR"), base_batch=2, l_max=512))
    assert [m.idx for m in plan] == [[4, 1], [3, 0], [2]]                                   # 60 | 70 70 | 80 80


# ------------------------------------------------------------------ VBS without bins, enumerated by hand
def test_hand_enumerated_vbs_without_bins():
    """Sec. 4.1 VBS keeps the tokens per batch constant; without bins a chunk of the sorted list is the longest
    one whose size does not exceed the batch size allowed for its largest prediction."""
    pol = so.Policy(flags=("SORT", "FCR", "VBS"), base_batch=2, l_max=100, max_batch=8)
    # allowed batch = clamp(floor(2*100/L), 2, 8): 10, 12, 20, 25 -> 8; 30 -> 6; 40 -> 5; 50 -> 4; 55 -> 3; 70, 100 -> 2
    assert [pol.batch_for(L) for L in (10, 12, 20, 25, 30, 40, 50, 55, 70, 100)] == [8, 8, 8, 8, 6, 5, 4, 3, 2, 2]
    pred = [55, 10, 100, 25, 40, 12, 70, 30, 100, 20, 50, 25]
    # sorted: 1(10) 5(12) 9(20) 3(25) 11(25) 7(30) 4(40) 10(50) 0(55) 6(70) 2(100) 8(100)
    # chunk 1 takes 6 rows (the 6th has L = 30, which allows 6; a 7th would have L = 40, which allows 5);
    # chunk 2 takes 3 (the 3rd has L = 55 -> 3; a 4th would have L = 70 -> 2); chunk 3 takes 2 (L = 100 -> 2).
    plan = so.schedule(pred, len(pred), 0, pol)
    assert [(m.idx, m.cap) for m in plan] == [([1, 5, 9, 3, 11, 7], 30), ([4, 10, 0], 55), ([6, 2], 100), ([8], 100)]
    # without FCR the same chunks run to the global limit
    plan = so.schedule(pred, len(pred), 0, so.Policy(flags=("SORT", "VBS"), base_batch=2, l_max=100, max_batch=8))
    assert [(m.idx, m.cap) for m in plan] == [([1, 5, 9, 3, 11, 7], 100), ([4, 10, 0], 100), ([6, 2], 100), ([8], 100)]


# ------------------------------------------------------------------ invariants on the five configured groups
def _policy(w):
    return so.Policy(flags=w.flags, base_batch=w.base_batch, l_max=w.l_max, max_batch=w.max_batch)


@pytest.mark.parametrize("cfg", [2, 3, 4, 5])
def test_plan_invariants(cfg):
    w = synth.make_workload(cfg)
    pol = _policy(w)
    r = so.run_group(w.pred_lens, w.target_lens, w.bin_width, pol)
    plan = r["plan"]
    flat = [i for m in plan for i in m.idx]
    assert sorted(flat) == list(range(w.n))                                    # a permutation: every query once
    t = w.target_lens
    if w.pred_lens is not None:
        key = [so.bin_upper(int(p), w.bin_width, w.l_max) for p in w.pred_lens]
        seen = {}
        for k, m in enumerate(plan):
            ub = {key[i] for i in m.idx}
            assert len(ub) == 1                                                # one bin per micro-batch
            ub = ub.pop()
            assert m.cap == min(ub, w.l_max)
            assert len(m.idx) <= pol.batch_for(ub)
            seen.setdefault(ub, []).append(len(m.idx))
        for ub, sizes in seen.items():
            assert all(s == pol.batch_for(ub) for s in sizes[:-1])             # only a bin's last chunk is short
        assert list(seen) == sorted(seen)                                      # ascending bins
    # failures are exactly the rows whose true length exceeds their cap, and each is recomputed exactly once
    failed = sorted(i for m in plan for i in m.idx if t[i] > m.cap)
    assert sorted(r["first"].failed) == failed
    assert sorted(i for m in r["failure_plan"] for i in m.idx) == failed
    assert all(m.cap == w.l_max and len(m.idx) <= w.base_batch for m in r["failure_plan"])
    # token accounting: every query's useful tokens are emitted once; steps are the per-micro-batch maxima
    emitted = sum(min(int(t[i]), m.cap) for m in plan for i in m.idx if t[i] <= m.cap)
    emitted += sum(int(t[i]) for m in r["failure_plan"] for i in m.idx)
    assert emitted == int(t.sum()) == r["useful_tokens"]
    assert r["steps"] == sum(min(m.cap, max(int(t[i]) for i in m.idx)) for m in plan + r["failure_plan"])
    assert r["live_row_steps"] <= r["padded_row_steps"]


def test_reductions_to_vanilla():
    w = synth.make_workload(3)
    n, t = w.n, w.target_lens
    vanilla = so.schedule(None, n, 0, so.Policy(flags=(), base_batch=16, l_max=512))
    assert [m.idx for m in vanilla] == [list(range(s, s + 16)) for s in range(0, n, 16)]
    # all predictions equal -> one bin, arrival order -> the vanilla chunks (cap aside)
    same = so.schedule([100] * n, n, 50, so.Policy(flags=("SORT", "BIN"), base_batch=16, l_max=512))
    assert [(m.idx, m.cap) for m in same] == [(m.idx, 512) for m in vanilla]
    # a bin as wide as the limit, no VBS -> vanilla chunks
    wide = so.schedule(w.pred_lens, n, 512, so.Policy(flags=("SORT", "BIN", "FCR"), base_batch=16, l_max=512))
    assert [m.idx for m in wide] == [m.idx for m in vanilla]
    # FCR off -> cap is the global limit and nothing fails
    r = so.run_group(w.pred_lens, t, 50, so.Policy(flags=("SORT", "BIN"), base_batch=16, l_max=512))
    assert r["n_failed"] == 0 and all(m.cap == 512 for m in r["plan"])
    # a perfect predictor never fails (the paper's upper-bound row uses the true length as the prediction)
    r = so.run_group(t, t, 50, so.Policy(flags=("SORT", "BIN", "FCR"), base_batch=16, l_max=512))
    assert r["n_failed"] == 0
    rv = so.run_group(None, t, 0, so.Policy(flags=(), base_batch=16, l_max=512))
    assert r["padded_row_steps"] < rv["padded_row_steps"]


def test_vbs_without_bins_keeps_tokens_per_batch():
    w = synth.make_workload(4)
    pol = so.Policy(flags=("SORT", "FCR", "VBS"), base_batch=16, l_max=512, max_batch=256)
    plan = so.schedule(w.pred_lens, w.n, 0, pol)
    assert sorted(i for m in plan for i in m.idx) == list(range(w.n))
    for m in plan:
        longest = max(int(w.pred_lens[i]) for i in m.idx)
        assert len(m.idx) <= pol.batch_for(longest)
        assert m.cap == min(longest, 512)


def test_synthetic_groups_look_like_the_papers():
    """Plausibility only (different data): vanilla wastes most row-steps, scheduling removes a large part."""
    w2, w3 = synth.make_workload(2), synth.make_workload(3)
    assert np.array_equal(w2.target_lens, w3.target_lens) and np.array_equal(w2.prompt_tokens, w3.prompt_tokens)
    v = so.run_group(None, w2.target_lens, 0, _policy(w2))
    s = so.run_group(w3.pred_lens, w3.target_lens, w3.bin_width, _policy(w3))
    assert 0.45 < v["redundancy"] < 0.80
    assert s["padded_row_steps"] < 0.8 * v["padded_row_steps"]
    assert 0.05 < s["failure_ratio"] < 0.45
