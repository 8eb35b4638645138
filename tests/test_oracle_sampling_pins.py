"""Pins of the sampling / end-of-sequence oracle against things other than itself: closed forms
(two-token sigmoid, equal logits), a library softmax through stratified draws, invariances of the
softmax, the greedy limit, an independent library model (torch fp64) for the free-running loop, and
the truncation property of an end-of-sequence token (Sec. 4.2, Experimental Setting: temperature sampling, rows end at their
end-of-sequence token or at the limit on new tokens; Sec. 4.1: unfinished at the limit = failed)."""
import math

import numpy as np
import pytest
import scipy.special
import torch

from paper_2305_13144_amd import synth
from oracle import sampling_oracle as sm
from oracle.model_oracle import OracleModel


# ------------------------------------------------------------------ one draw
def test_two_tokens_closed_form():
    """P(token 0) = sigmoid((l0 - l1) / T): token 0 exactly when u is below it."""
    rng = np.random.default_rng(0)
    for _ in range(300):
        l0, l1 = rng.normal(size=2) * 3
        T = float(rng.uniform(0.2, 2.0))
        u = float(rng.random())
        p0 = 1.0 / (1.0 + math.exp(-(l0 - l1) / T))
        if abs(u - p0) < 1e-9:
            continue
        tok, mg = sm.sample_token([l0, l1], T, u)
        assert tok == (0 if u < p0 else 1)
        want = min(u, p0 - u) if tok == 0 else min(u - p0, 1 - u)   # distance to the chosen interval's nearer edge
        assert math.isclose(mg, want, rel_tol=1e-9, abs_tol=1e-12), (mg, want)


def test_equal_logits_pick_floor_u_times_v():
    rng = np.random.default_rng(1)
    for V in (2, 7, 64, 1000):
        for _ in range(50):
            u = float(rng.random())
            if abs(u * V - round(u * V)) < 1e-6:
                continue
            tok, _ = sm.sample_token(np.full(V, 1.2345), 0.7, u)
            assert tok == int(math.floor(u * V))


def test_stratified_draws_reproduce_library_softmax():
    """N evenly spaced draws hit token v  N*p_v times (to within one), p from scipy's softmax."""
    rng = np.random.default_rng(2)
    l = rng.normal(size=40) * 2.0
    T = 0.5
    N = 20000
    counts = np.zeros(40, np.int64)
    for k in range(N):
        tok, _ = sm.sample_token(l, T, (k + 0.5) / N)
        counts[tok] += 1
    p = scipy.special.softmax(l / T)
    assert counts.sum() == N
    assert np.abs(counts - N * p).max() <= 1.0 + 1e-6
    assert np.allclose(sm.token_probabilities(l, T), p, rtol=1e-12, atol=0)


def test_vocabulary_order_of_the_cdf():
    """u just above the mass of tokens 0..k-1 picks token k: the CDF runs in index order, not sorted by mass."""
    l = np.array([0.3, 2.0, -1.0, 0.9, 0.0])
    T = 0.8
    p = scipy.special.softmax(l / T)
    edges = np.concatenate([[0.0], np.cumsum(p)])
    for k in range(5):
        assert sm.sample_token(l, T, float(edges[k] + 1e-7))[0] == k
        assert sm.sample_token(l, T, float(edges[k + 1] - 1e-7))[0] == k
    assert sm.sample_token(l, T, 0.0)[0] == 0


def test_a_draw_on_an_interval_edge_belongs_to_the_next_token():
    """Token v owns the half-open interval [c_{v-1}, c_v) of the CDF, so that a uniform u in [0,1) picks it with
    probability p_v exactly: u equal to an edge picks the token above it.  Equal logits with a power-of-two count make
    every edge exact in binary."""
    for V in (2, 4, 8):
        l = np.full(V, -0.75)
        for k in range(1, V):
            assert sm.sample_token(l, 0.5, k / V)[0] == k
            assert sm.sample_token(l, 0.5, float(np.nextafter(k / V, 0.0)))[0] == k - 1
        assert sm.sample_token(l, 0.5, 0.0)[0] == 0


def test_a_cdf_that_rounding_leaves_below_the_draw_ends_on_the_last_token():
    """Ten equal masses of 0.1 add up to 1 - 2^-53 in double precision; the largest draw below 1 is not exceeded by any
    partial sum, and the definition's answer (the last interval reaches up to 1) is the last token."""
    acc = 0.0
    for _ in range(10):
        acc += 0.1
    u = float(np.nextafter(1.0, 0.0))
    assert acc == u                                   # the premise: no partial sum is > u
    tok, mg = sm.sample_token(np.zeros(10), 1.0, u)
    assert tok == 9 and mg == 0.0


def test_softmax_invariances():
    rng = np.random.default_rng(3)
    l = rng.normal(size=100)
    for _ in range(100):
        u = float(rng.random())
        T = float(rng.uniform(0.3, 1.5))
        a, mg = sm.sample_token(l, T, u)
        if mg < 1e-9:
            continue
        assert sm.sample_token(l + 17.25, T, u)[0] == a          # shift of every logit
        assert sm.sample_token(l * 3.0, T * 3.0, u)[0] == a      # common scale of logits and temperature


def test_low_temperature_tends_to_greedy_and_t0_is_argmax_lowest_index():
    rng = np.random.default_rng(4)
    for _ in range(50):
        l = rng.normal(size=200)
        srt = np.sort(l)
        if srt[-1] - srt[-2] < 0.05:
            continue
        assert sm.sample_token(l, 1e-3, float(rng.uniform(0.01, 0.99)))[0] == int(np.argmax(l))
        tok, mg = sm.sample_token(l, 0.0, 0.123)
        assert tok == int(np.argmax(l)) and math.isclose(mg, srt[-1] - srt[-2], rel_tol=1e-12)
    assert sm.sample_token([1.0, 5.0, 5.0, 2.0], 0.0, 0.9) == (1, 0.0)


def test_high_temperature_tends_to_uniform():
    l = np.random.default_rng(5).normal(size=50)
    for u in (0.011, 0.505, 0.987):
        assert sm.sample_token(l, 1e6, u)[0] == int(math.floor(u * 50))


# ------------------------------------------------------------------ the generation loop
@pytest.fixture(scope="module")
def tiny(oracle_built):
    from tests.test_oracle_model_pins import _hf_model
    W = synth.make_weights(synth.TINY, seed=11, norm_jitter=0.1, threads=1)
    return W, OracleModel(synth.TINY, W, "f64"), _hf_model(synth.TINY, W)


def _library_generate(hf, prompt, cap, T, draws):
    """The same definition on an independent library model: torch fp64 softmax + cumsum + searchsorted."""
    seq = list(int(t) for t in prompt)
    out = []
    for s in range(cap):
        with torch.no_grad():
            lg = hf(torch.tensor(seq, dtype=torch.int64)[None]).logits[0, -1]
        if T == 0:
            t = int(torch.argmax(lg))
        else:
            cdf = torch.cumsum(torch.softmax(lg / T, dim=-1), dim=-1)
            t = min(int(torch.searchsorted(cdf, torch.tensor(float(draws[s]), dtype=torch.float64), right=True)),
                    lg.numel() - 1)
        out.append(t)
        seq.append(t)
    return out


@pytest.mark.parametrize("T", [0.5, 1.0])
def test_free_running_sampling_matches_library_model(tiny, T):
    W, om, hf = tiny
    w = synth.make_workload(1)
    draws = synth.make_draws(w.n, 24, seed=77)
    for i in (0, 4, 9):
        r = sm.generate_query(om, w.prompt(i), 24, -1, T, draws[i])
        assert r["length"] == 24 and r["failed"]
        ref = _library_generate(hf, w.prompt(i), 24, T, draws[i])
        # the two evaluations differ near 1e-7 in the logits: they may part ways only at a draw that close
        # to an edge of the CDF (after which the prefixes differ and nothing more can be compared)
        agree = 0
        for s in range(24):
            if int(r["tokens"][s]) != ref[s]:
                assert r["margins"][s] < 1e-6, (i, s, r["margins"][s])
                break
            agree += 1
        assert agree >= 20


def test_eos_truncates_the_unbounded_run(tiny):
    """With an end-of-sequence id the output is the run without one, cut after its first occurrence."""
    W, om, _ = tiny
    w = synth.make_workload(1)
    draws = synth.make_draws(w.n, 40, seed=78)
    i, cap, T = 2, 40, 1.0
    free = sm.generate_query(om, w.prompt(i), cap, -1, T, draws[i])
    assert free["failed"] and free["length"] == cap
    for k in (0, 1, 7, cap - 1):
        eos = int(free["tokens"][k])
        first = int(np.flatnonzero(free["tokens"] == eos)[0])
        r = sm.generate_query(om, w.prompt(i), cap, eos, T, draws[i])
        assert r["length"] == first + 1 and not r["failed"]
        assert np.array_equal(r["tokens"], free["tokens"][:first + 1])
        assert r["tokens"][-1] == eos and (r["tokens"][:-1] != eos).all()
    # a smaller cap only cuts the sequence; the row fails iff its end lies beyond the cap
    eos = int(free["tokens"][7])
    first = int(np.flatnonzero(free["tokens"] == eos)[0])
    for c in (first, first + 1, first + 2):
        r = sm.generate_query(om, w.prompt(i), c, eos, T, draws[i])
        assert r["length"] == min(c, first + 1)
        assert r["failed"] == (first + 1 > c)
        assert np.array_equal(r["tokens"], free["tokens"][:r["length"]])


def test_forced_length_combines_with_eos_and_greedy_equals_the_greedy_oracle(tiny):
    W, om, _ = tiny
    w = synth.make_workload(1)
    i = 6
    greedy, _ = om.greedy_query(w.prompt(i), 12)
    r = sm.generate_query(om, w.prompt(i), 30, -1, 0.0, None, target_len=12)
    assert r["length"] == 12 and not r["failed"] and np.array_equal(r["tokens"], greedy[:12])
    r = sm.generate_query(om, w.prompt(i), 8, -1, 0.0, None, target_len=12)
    assert r["length"] == 8 and r["failed"] and np.array_equal(r["tokens"], greedy[:8])
    r = sm.generate_query(om, w.prompt(i), 12, -1, 0.0, None, target_len=12)
    assert r["length"] == 12 and not r["failed"]
    eos = int(greedy[4])
    first = int(np.flatnonzero(greedy == eos)[0])
    r = sm.generate_query(om, w.prompt(i), 30, eos, 0.0, None, target_len=12)
    assert r["length"] == first + 1 and not r["failed"]
    r = sm.generate_query(om, w.prompt(i), 30, eos, 0.0, None, target_len=first)
    assert r["length"] == max(first, 1)


def test_next_token_on_prefix_is_the_loop_step(tiny):
    W, om, _ = tiny
    w = synth.make_workload(1)
    draws = synth.make_draws(w.n, 10, seed=79)
    r = sm.generate_query(om, w.prompt(3), 10, -1, 0.7, draws[3])
    for s in (0, 4, 9):
        tok, mg = sm.next_token_on_prefix(om, w.prompt(3), r["tokens"][:s], 0.7, float(draws[3, s]))
        if r["margins"][s] > 1e-9:
            assert tok == r["tokens"][s]
            assert math.isclose(mg, r["margins"][s], rel_tol=1e-6, abs_tol=1e-12)


def test_draws_are_seeded_and_in_range():
    a = synth.make_draws(5, 9, seed=3)
    b = synth.make_draws(5, 9, seed=3)
    assert a.dtype == np.float32 and a.shape == (5, 9) and np.array_equal(a, b)
    assert (a >= 0).all() and (a < 1).all() and not np.array_equal(a, synth.make_draws(5, 9, seed=4))


# ------------------------------------------------------------------ counter-based draws
def test_philox_known_answer_vectors():
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")
    n = 0
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        ctr, key, out = [[int(x, 16) for x in part.split()] for part in line.split("|")]
        assert sm.philox4x32_10(ctr, key) == tuple(out)
        n += 1
    assert n == 3


_TRITON_CHILD = r"""
import os, sys
os.environ["TRITON_INTERPRET"] = "1"          # the library's CPU interpreter: no GPU, no compilation
import numpy as np, torch, triton, triton.language as tl

@triton.jit
def k(seed_ptr, c_ptr, out_ptr, N: tl.constexpr):
    i = tl.arange(0, N)
    o0, o1, o2, o3 = tl.philox(tl.load(seed_ptr + i), tl.load(c_ptr + i), tl.load(c_ptr + N + i),
                               tl.load(c_ptr + 2 * N + i), tl.load(c_ptr + 3 * N + i))
    tl.store(out_ptr + i, o0)
    tl.store(out_ptr + N + i, o1)
    tl.store(out_ptr + 2 * N + i, o2)
    tl.store(out_ptr + 3 * N + i, o3)

N = 256
rng = np.random.default_rng(int(sys.argv[1]))
seed = rng.integers(-2**63, 2**63, size=N, dtype=np.int64)
ctr = rng.integers(0, 2**32, size=(4, N), dtype=np.uint64).astype(np.uint32)
ctr[0, :8] = [0, 1, 2, 3, 0xffffffff, 0, 7, 511]          # the sampler's counters: (token number, row id, 0, 0)
ctr[1, :8] = [0, 5, 1, 77, 3, 0xffffffff, 2, 9]
ctr[2:, :8] = 0
kat = [l.split("|") for l in open(sys.argv[2]) if l.strip() and not l.startswith("#")]     # inputs of the published vectors
for j, (c, key, _) in enumerate(kat):
    ctr[:, 8 + j] = [int(x, 16) for x in c.split()]
    k0, k1 = [int(x, 16) for x in key.split()]
    seed[8 + j] = np.array([(k1 << 32) | k0], np.uint64).astype(np.int64)[0]
out = torch.zeros(4, N, dtype=torch.uint32)
k[(1,)](torch.from_numpy(seed), torch.from_numpy(ctr.copy()), out, N=N)
o = out.numpy()
for j in range(N):
    print(int(seed[j]) & (2**64 - 1), *[int(x) for x in ctr[:, j]], *[int(x) for x in o[:, j]])
"""


def test_philox_matches_an_independent_library_implementation():
    """The oracle's Philox4x32-10 against the one a tensor-compiler library ships for its random numbers, run in
    that library's CPU interpreter on 256 seeded (counter, key) pairs (the library takes the key as one 64-bit seed:
    low word first).  This pins the round function, its constants, the key schedule and the word order to code that
    shares nothing with this repository; the three published vectors above pin the same things to the paper's table."""
    import subprocess
    import sys
    pytest.importorskip("triton")
    import os
    kat_path = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")
    r = subprocess.run([sys.executable, "-c", _TRITON_CHILD, "2024", kat_path], capture_output=True, text=True, timeout=600)
    if r.returncode != 0 and "philox" not in r.stderr:
        pytest.skip("the library's CPU interpreter does not run here: " + r.stderr.strip().splitlines()[-1][:200])
    assert r.returncode == 0, r.stderr[-2000:]
    rows = [[int(x) for x in line.split()] for line in r.stdout.strip().splitlines()]
    assert len(rows) == 256
    for seed, c0, c1, c2, c3, *out in rows:
        assert sm.philox4x32_10((c0, c1, c2, c3), (seed & 0xFFFFFFFF, seed >> 32)) == tuple(out)
    # rows 8-10 are the inputs of the stored known-answer vectors: the library gives the stored outputs
    stored = [[int(x, 16) for x in l.split("|")[2].split()] for l in open(kat_path) if l.strip() and not l.startswith("#")]
    assert [row[5:] for row in rows[8:8 + len(stored)]] == stored and len(stored) == 3
    # the draw the sampler uses: counter (token number, row id, 0, 0), top 24 bits of the first word
    for seed, c0, c1, c2, c3, *out in rows[:8]:
        assert c2 == 0 and c3 == 0
        assert sm.generated_draw(seed, c1, c0) == np.float32((out[0] >> 8) * 2.0 ** -24)


def test_generated_draw_is_top_24_bits_of_the_first_word():
    # counter (0,0,0,0), key 0: first word 0x6627e8d5 -> 0x6627e8 * 2^-24
    assert sm.generated_draw(0, 0, 0) == np.float32(0x6627E8 / 2.0 ** 24)
    # the 64-bit seed supplies the key words: low half first
    x0 = sm.philox4x32_10((5, 9, 0, 0), (0xA4093822, 0x299F31D0))[0]
    assert sm.generated_draw((0x299F31D0 << 32) | 0xA4093822, 9, 5) == np.float32((x0 >> 8) / 2.0 ** 24)
    t = sm.generated_draws(12345, [0, 1, 7], 50)
    assert t.dtype == np.float32 and t.shape == (3, 50) and (t >= 0).all() and (t < 1).all()
    assert len(np.unique(t)) == 150                                   # a bijection on distinct counters: no repeats here
    assert np.array_equal(t[2], sm.generated_draws(12345, [7], 50)[0])  # a row's draws depend on its id only
    assert not np.array_equal(t, sm.generated_draws(12346, [0, 1, 7], 50))


def test_generated_draws_are_uniform():
    """Kolmogorov-Smirnov distance of 20000 draws to U[0,1) (scipy), and the lag-1 correlation along a row."""
    import scipy.stats
    t = sm.generated_draws(2023, range(40), 500).astype(np.float64)
    assert scipy.stats.kstest(t.ravel(), "uniform").statistic < 0.012
    x = t - 0.5
    assert abs((x[:, 1:] * x[:, :-1]).mean() / x.var()) < 0.03
