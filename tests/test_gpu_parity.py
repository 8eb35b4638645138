"""GPU parity: the HIP path (through the C ABI) against the CPU oracle on the same seeded inputs.

Bars (written here, used everywhere below):
  * integers (plans, lengths, failure flags, counters, -1 padding): bit-exact;
  * teacher-forced logits: max |gpu - oracle| <= 3e-2 * max |oracle logit| at every position;
  * greedy tokens: the token the GPU emitted after a prefix must be the oracle's argmax on that same
    prefix whenever the oracle's top-1/top-2 margin there exceeds 0.1 (random-init models have many
    near-ties, so free-running sequences may legitimately part ways at a near-tie; every position is
    therefore checked teacher-forced on the GPU's own prefix).
"""
import numpy as np
import pytest

from paper_2305_13144_amd import binding as ss
from paper_2305_13144_amd import synth
from oracle import sched_oracle as so
from oracle.model_oracle import OracleModel

pytestmark = pytest.mark.gpu

LOGIT_TOL = 3e-2
MARGIN = 0.1


def _say(msg):
    print(msg, flush=True)


# ------------------------------------------------------------------ helpers
def check_logits(gpu, ref, what):
    scale = np.abs(ref).max()
    err = np.abs(gpu.astype(np.float64) - ref).max(axis=-1)
    worst = float(err.max())
    _say(f"  {what}: max|err| = {worst:.3e}  (= {worst / scale:.2e} of max|logit| {scale:.3f})")
    assert worst <= LOGIT_TOL * scale, what
    big = np.partition(ref, -2, axis=-1)
    margin = big[:, -1] - big[:, -2]
    decided = margin > MARGIN
    assert (gpu.argmax(-1)[decided] == ref.argmax(-1)[decided]).all(), what
    return worst / scale


def check_tokens_teacher_forced(om, prompt, toks, upto=None, what=""):
    """Every emitted token must be the oracle's greedy choice on the GPU's own prefix (where decided)."""
    L = len(toks) if upto is None else min(upto, len(toks))
    seq = np.concatenate([prompt, toks[:L - 1]]).astype(np.int32) if L > 1 else np.asarray(prompt, np.int32)
    lg = om.teacher_forced(seq, first=len(prompt) - 1)
    assert lg.shape[0] == L
    big = np.partition(lg, -2, axis=-1)
    margin = big[:, -1] - big[:, -2]
    ref = lg.argmax(-1)
    decided = margin > MARGIN
    bad = [g for g in range(L) if decided[g] and ref[g] != toks[g]]
    assert not bad, (what, bad[:5])
    return int(decided.sum()), L


def forced_batch(w, rows, extra, rng):
    """Ragged prompts of the given rows followed by `extra[i]` random forced tokens."""
    toks, offs, npr = [], [0], []
    for i, e in zip(rows, extra):
        p = w.prompt(i)
        t = np.concatenate([p, rng.integers(0, w.shape.vocab, size=e).astype(np.int32)])
        toks.append(t)
        offs.append(offs[-1] + len(t))
        npr.append(len(p))
    return np.concatenate(toks).astype(np.int32), np.array(offs, np.int32), np.array(npr, np.int32)


def oracle_forced_logits(om, toks, offs, npr):
    out = []
    for i in range(len(npr)):
        out.append(om.teacher_forced(toks[offs[i]:offs[i + 1]], first=int(npr[i]) - 1))
    return np.concatenate(out, axis=0)


# ------------------------------------------------------------------ fixtures
@pytest.fixture(scope="module")
def tiny(oracle_built):
    W = synth.make_weights(synth.TINY, seed=1, norm_jitter=0.1, threads=1)
    gw = ss.Weights(synth.TINY, W)
    yield W, OracleModel(synth.TINY, W, "f64"), gw
    gw.close()


@pytest.fixture(scope="module")
def wide2(oracle_built):
    """7B widths (d 4096, 32 heads of 128, ffn 11008, vocab 32000) at 2 layers: every kernel at its real shape."""
    shape = synth.LLAMA7B.with_layers(2)
    W = synth.make_weights(shape, seed=2, norm_jitter=0.05)
    gw = ss.Weights(shape, W)
    yield shape, W, OracleModel(shape, W, "f64"), gw
    gw.close()


# ------------------------------------------------------------------ teacher-forced logits
def test_tiny_prompt_logits_every_position(tiny):
    """Prompt (prefill) path position by position: ragged rows, spans several 16-row strips and a ragged tail."""
    W, om, gw = tiny
    w = synth.make_workload(1)
    _say("tiny prompt logits, all positions, 16 ragged rows")
    got = ss.ss_forward_logits(gw, w.prompt_tokens, w.prompt_offsets, w.prompt_lens, all_prompt_logits=True)
    ref = np.concatenate([om.teacher_forced(w.prompt(i), first=0) for i in range(w.n)], axis=0)
    assert got.shape == ref.shape
    check_logits(got, ref, "tiny prefill")


def test_tiny_prompt_logits_across_attention_tiles(tiny):
    """Prompt attention works in tiles of 64 queries and 32 keys: prompt lengths on and around every tile edge
    (1 .. 200 tokens, head_dim 64), logits at every position against the oracle."""
    W, om, gw = tiny
    rng = np.random.default_rng(64)
    lens = [1, 2, 31, 32, 33, 63, 64, 65, 96, 127, 128, 129, 200]
    prompts = [rng.integers(0, synth.TINY.vocab, size=n).astype(np.int32) for n in lens]
    toks = np.concatenate(prompts)
    offs = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    _say(f"tiny prompt logits, all positions, prompt lengths {lens}")
    got = ss.ss_forward_logits(gw, toks, offs, np.array(lens, np.int32), all_prompt_logits=True)
    ref = np.concatenate([om.teacher_forced(p, first=0) for p in prompts], axis=0)
    assert got.shape == ref.shape
    check_logits(got, ref, "tiny prefill across tiles")


def test_wide_prompt_logits_across_attention_tiles(wide2):
    """The same at head_dim 128 (7B widths): a 150-token and a 70-token prompt next to short ones, logits at every
    position of the two long rows."""
    shape, W, om, gw = wide2
    rng = np.random.default_rng(65)
    lens = [150, 5, 70, 33]
    prompts = [rng.integers(0, shape.vocab, size=n).astype(np.int32) for n in lens]
    toks = np.concatenate(prompts)
    offs = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    _say(f"7B-width prompt logits, all positions, prompt lengths {lens}")
    got = ss.ss_forward_logits(gw, toks, offs, np.array(lens, np.int32), all_prompt_logits=True)
    for i in (0, 2):
        ref = om.teacher_forced(prompts[i], first=0)
        check_logits(got[offs[i]:offs[i + 1]], ref, f"wide2 prefill row {i} ({lens[i]} tokens)")


@pytest.mark.parametrize("rows", [1, 5, 16, 23, 40, 64, 100])
def test_tiny_decode_logits_teacher_forced(tiny, rows):
    """Prompt forward then decode steps on forced tokens; row counts cover 1..4 strips of the skinny
    kernel, its ragged tails, and the tiled kernel (100 rows); rows drop out at different steps."""
    W, om, gw = tiny
    rng = np.random.default_rng(100 + rows)
    w = synth.make_group(synth.TINY, rows, 777 + rows, ("uniform", 3, 40), ("uniform", 1, 8), None, 8, 0, ())
    extra = rng.integers(0, 7, size=rows)
    toks, offs, npr = forced_batch(w, range(rows), extra, rng)
    _say(f"tiny teacher-forced decode, {rows} rows")
    got = ss.ss_forward_logits(gw, toks, offs, npr)
    ref = oracle_forced_logits(om, toks, offs, npr)
    assert got.shape == ref.shape
    check_logits(got, ref, f"tiny decode B={rows}")


@pytest.mark.parametrize("mode", [1, 2])
@pytest.mark.parametrize("rows", [1, 16, 23, 40, 64, 70, 100, 128])
def test_tiny_decode_logits_each_small_batch_projection_kernel(tiny, rows, mode):
    """Both kernels for small-batch projections, forced for every projection: the k-splitting one (mode 1; the
    tiled kernel above 64 rows) and the one that stages activations once per workgroup (mode 2, up to 128
    rows), here with fewer strips than compute units, idle waves, 1-8 row strips with ragged tails and a k
    range (ffn 688 -> 22 k-blocks) that ends inside a chunk."""
    W, om, gw = tiny
    rng = np.random.default_rng(300 + rows)
    w = synth.make_group(synth.TINY, rows, 555 + rows, ("uniform", 3, 40), ("uniform", 1, 8), None, 8, 0, ())
    toks, offs, npr = forced_batch(w, range(rows), rng.integers(0, 5, size=rows), rng)
    ref = oracle_forced_logits(om, toks, offs, npr)
    _say(f"tiny teacher-forced decode, {rows} rows, projection kernel mode {mode}")
    ss.ss_set_gemm_mode(mode)
    try:
        got = ss.ss_forward_logits(gw, toks, offs, npr)
    finally:
        ss.ss_set_gemm_mode(0)
    check_logits(got, ref, f"tiny decode B={rows} mode={mode}")


@pytest.mark.parametrize("rows", [16, 40, 100])
def test_odd_shape_many_strips_per_workgroup(oracle_built, rows):
    """A one-layer shape with a very wide MLP (ffn 16448 -> 1028 gate/up strip pairs, 514 k-blocks in the down
    projection) and a large vocabulary (40000 -> 2500 strips): the activation-staging kernel with 8 waves per
    workgroup and the SwiGLU epilogue, and with more workgroups than compute units, which none of the LLaMA
    shapes reaches."""
    shape = synth.ModelShape("wide-ffn", 1, 256, 4, 64, 16448, 40000)
    W = synth.make_weights(shape, seed=11, norm_jitter=0.1, threads=4)
    gw = ss.Weights(shape, W)
    om = OracleModel(shape, W, "f64")
    try:
        rng = np.random.default_rng(400 + rows)
        w = synth.make_group(shape, rows, 901 + rows, ("uniform", 3, 20), ("uniform", 1, 8), None, 8, 0, ())
        toks, offs, npr = forced_batch(w, range(rows), rng.integers(0, 4, size=rows), rng)
        ref = oracle_forced_logits(om, toks, offs, npr)
        for mode in (0, 2):
            _say(f"wide-ffn shape, {rows} rows, projection kernel mode {mode}")
            ss.ss_set_gemm_mode(mode)
            try:
                got = ss.ss_forward_logits(gw, toks, offs, npr)
            finally:
                ss.ss_set_gemm_mode(0)
            check_logits(got, ref, f"wide-ffn B={rows} mode={mode}")
    finally:
        gw.close()


def test_tiny_long_contexts_decode_logits(tiny):
    """Contexts of several hundred to 1500 slots: the decode attention takes 256 slots per round trip, so
    these rows need 2 to 6 of them, with ragged last passes; rows of very different lengths share the batch."""
    W, om, gw = tiny
    rng = np.random.default_rng(77)
    w = synth.make_group(synth.TINY, 5, 4242, ("uniform", 250, 1500), ("uniform", 1, 8), None, 8, 0, ())
    toks, offs, npr = forced_batch(w, range(5), [6, 3, 5, 4, 6], rng)
    _say(f"tiny teacher-forced decode at long contexts: prompts {npr.tolist()}")
    got = ss.ss_forward_logits(gw, toks, offs, npr)
    ref = oracle_forced_logits(om, toks, offs, npr)
    assert got.shape == ref.shape
    check_logits(got, ref, "tiny long contexts")


def test_tiny_large_batch_with_compaction_matches_oracle_rows(tiny):
    """600 rows in one micro-batch (tiled kernels for the prompt and the first steps, then the small-batch
    kernels as rows finish and compaction shrinks the batch): lengths exact, sampled rows re-derived by the oracle."""
    W, om, gw = tiny
    w = synth.make_group(synth.TINY, 600, 31337, ("uniform", 4, 24), ("uniform", 1, 12), None, 12, 0, ())
    cap = 9
    _say("tiny 600-row micro-batch, cap 9, compaction on")
    r = ss.ss_decode_microbatch(gw, w.prompt_tokens, w.prompt_offsets, cap, w.target_lens, ss.SS_COMPACT)
    assert np.array_equal(r["lens"], np.minimum(w.target_lens, cap))
    assert np.array_equal(r["failed"].astype(bool), w.target_lens > cap)
    assert r["stats"]["row_steps"] == int(np.minimum(w.target_lens, cap).sum())
    for j in (0, 1, 77, 300, 511, 599):
        L = int(r["lens"][j])
        assert (r["tokens"][j, :L] >= 0).all() and (r["tokens"][j, L:] == -1).all()
        check_tokens_teacher_forced(om, w.prompt(j), r["tokens"][j, :L], what=f"row {j}")


def test_f32_source_weights_are_rounded_like_the_generator(tiny):
    """Config 1 ships fp32 weights: the library rounds them to bf16 (nearest even) at load."""
    W, om, gw = tiny
    rng = np.random.default_rng(5)
    specs = synth.TINY.tensor_specs()
    children = np.random.SeedSequence(99).spawn(len(specs))
    f32 = []
    for (name, shp), c in zip(specs, children):
        g = np.random.Generator(np.random.PCG64(c))
        f32.append((np.ones(shp) + 0.1 * g.standard_normal(shp) if len(shp) == 1
                    else 0.02 * g.standard_normal(shp)).astype(np.float32))
    bits = [synth.f32_to_bf16_bits(t) for t in f32]
    om2 = OracleModel(synth.TINY, bits, "f64")
    gw2 = ss.Weights(synth.TINY, f32, ss.SS_F32)
    gw3 = ss.Weights(synth.TINY, bits, ss.SS_BF16)
    try:
        w = synth.make_workload(1)
        a = ss.ss_forward_logits(gw2, w.prompt_tokens, w.prompt_offsets, w.prompt_lens)
        b = ss.ss_forward_logits(gw3, w.prompt_tokens, w.prompt_offsets, w.prompt_lens)
        assert np.array_equal(a, b)               # same bf16 weights either way -> same bits out
        ref = np.stack([om2.teacher_forced(w.prompt(i), first=len(w.prompt(i)) - 1)[0] for i in range(w.n)])
        check_logits(a, ref, "fp32-source weights")
    finally:
        gw2.close()
        gw3.close()


def test_wide_logits_teacher_forced(wide2):
    shape, W, om, gw = wide2
    rng = np.random.default_rng(8)
    w = synth.make_workload(2, n=6, shape=shape)
    rows = [0, 1, 2, 3]
    extra = [3, 0, 5, 2]
    toks, offs, npr = forced_batch(w, rows, extra, rng)
    _say(f"7B-width x2 layers teacher-forced: prompts {npr.tolist()} extra {extra}")
    got = ss.ss_forward_logits(gw, toks, offs, npr)
    ref = oracle_forced_logits(om, toks, offs, npr)
    check_logits(got, ref, "wide2 prompt+decode")


@pytest.mark.parametrize("mode", [1, 2])
def test_wide_decode_logits_each_small_batch_projection_kernel(wide2, mode):
    """7B widths, 20 rows (two row strips, the second ragged): every projection through one kernel, then the other."""
    shape, W, om, gw = wide2
    rng = np.random.default_rng(18)
    w = synth.make_workload(2, n=20, shape=shape)
    toks, offs, npr = forced_batch(w, range(20), [2] * 20, rng)
    ref = oracle_forced_logits(om, toks, offs, npr)
    _say(f"7B-width x2 layers, 20 rows, projection kernel mode {mode}")
    ss.ss_set_gemm_mode(mode)
    try:
        got = ss.ss_forward_logits(gw, toks, offs, npr)
    finally:
        ss.ss_set_gemm_mode(0)
    check_logits(got, ref, f"wide2 B=20 mode={mode}")


@pytest.mark.parametrize("rows", [17, 33, 48, 49, 64, 100, 128, 129, 176, 200, 256])
def test_wide_decode_logits_across_row_strips(wide2, rows):
    """7B widths, 2-16 row strips, the kernel choice of the library itself (mode 0) and the same with the
    two-waves-per-unit split of the sweep kernel switched off (mode 4; the split is used above 96 rows),
    ragged last strips.  Three rows against the oracle in each mode; the two modes differ only in the order of fp32
    sums, which can move an activation by one unit of its half-precision rounding (2^-11) and a logit by that order."""
    shape, W, om, gw = wide2
    rng = np.random.default_rng(500 + rows)
    w = synth.make_group(shape, rows, 900 + rows, ("uniform", 3, 12), ("uniform", 1, 8), None, 8, 0, ())
    toks, offs, npr = forced_batch(w, range(rows), rng.integers(1, 3, size=rows), rng)
    out_off = np.concatenate([[0], np.cumsum(np.diff(offs) - npr + 1)])
    got = {}
    for mode in (0, 4):
        ss.ss_set_gemm_mode(mode)
        try:
            _say(f"7B-width x2 layers, {rows} rows, mode {mode}")
            got[mode] = ss.ss_forward_logits(gw, toks, offs, npr)
        finally:
            ss.ss_set_gemm_mode(0)
    for i in (0, rows // 2, rows - 1):
        ref = om.teacher_forced(toks[offs[i]:offs[i + 1]], first=int(npr[i]) - 1)
        for mode in (0, 4):
            check_logits(got[mode][out_off[i]:out_off[i + 1]], ref, f"B={rows} row {i} mode {mode}")
    scale = np.abs(got[0]).max()
    assert np.abs(got[0] - got[4]).max() <= 2e-3 * scale


def test_wide_prompt_forward_through_tiled_kernel(wide2):
    """> 64 prompt token-rows at real widths: tiled MFMA kernel incl. its ragged row and column tails."""
    shape, W, om, gw = wide2
    w = synth.make_workload(2, n=4, shape=shape)
    _say(f"7B-width x2 layers prompt logits, {int(w.prompt_offsets[-1])} token-rows")
    got = ss.ss_forward_logits(gw, w.prompt_tokens, w.prompt_offsets, w.prompt_lens)
    ref = np.stack([om.teacher_forced(w.prompt(i), first=len(w.prompt(i)) - 1)[0] for i in range(w.n)])
    check_logits(got, ref, "wide2 prefill")


# ------------------------------------------------------------------ micro-batch generation
@pytest.mark.parametrize("flags", [0, ss.SS_COMPACT])
@pytest.mark.parametrize("cap", [48, 20, 1])
def test_tiny_microbatch_config1(tiny, flags, cap):
    """Config 1: 16 queries, one padded batch (and the same with a cap, and with compaction)."""
    W, om, gw = tiny
    w = synth.make_workload(1)
    _say(f"tiny micro-batch cap={cap} flags={flags}")
    r = ss.ss_decode_microbatch(gw, w.prompt_tokens, w.prompt_offsets, cap, w.target_lens, flags)
    t = w.target_lens
    assert np.array_equal(r["lens"], np.minimum(t, cap))
    assert np.array_equal(r["failed"].astype(bool), t > cap)
    steps = min(cap, int(t.max()))
    assert r["stats"]["steps"] == steps and r["stats"]["rows"] == w.n
    want_rows = int(np.minimum(t, cap).sum()) if flags else w.n * steps
    assert r["stats"]["row_steps"] == want_rows
    assert r["stats"]["prompt_tokens"] == int(w.prompt_offsets[-1])
    decided = total = 0
    for i in range(w.n):
        L = int(r["lens"][i])
        assert (r["tokens"][i, :L] >= 0).all() and (r["tokens"][i, L:] == -1).all()
        dcd, tot = check_tokens_teacher_forced(om, w.prompt(i), r["tokens"][i, :L], what=f"row {i}")
        decided += dcd
        total += tot
    _say(f"  {decided}/{total} positions had a decided oracle argmax; all matched")


def test_compaction_does_not_change_outputs(tiny):
    """Same micro-batch padded and compacted: identical lengths/flags; tokens equal to the oracle's greedy
    sequence prefix up to the first undecided position in both."""
    W, om, gw = tiny
    w = synth.make_group(synth.TINY, 37, 4242, ("uniform", 4, 30), ("uniform", 1, 30), None, 30, 0, ())
    a = ss.ss_decode_microbatch(gw, w.prompt_tokens, w.prompt_offsets, 24, w.target_lens, 0)
    b = ss.ss_decode_microbatch(gw, w.prompt_tokens, w.prompt_offsets, 24, w.target_lens, ss.SS_COMPACT)
    assert np.array_equal(a["lens"], b["lens"]) and np.array_equal(a["failed"], b["failed"])
    ref = om.greedy_microbatch(w.prompt_tokens, w.prompt_offsets, 24, w.target_lens)
    assert np.array_equal(ref["lens"], a["lens"]) and np.array_equal(ref["failed"], a["failed"])
    for i in range(w.n):
        L = int(ref["lens"][i])
        und = np.nonzero(ref["margins"][i, :L] <= MARGIN)[0]
        k = int(und[0]) if len(und) else L
        assert np.array_equal(a["tokens"][i, :k], ref["tokens"][i, :k])
        assert np.array_equal(b["tokens"][i, :k], ref["tokens"][i, :k])


def test_wide_microbatch(wide2):
    shape, W, om, gw = wide2
    w = synth.make_workload(3, n=16, shape=shape)
    cap = 6
    _say("7B-width x2 layers micro-batch of 16, cap 6")
    r = ss.ss_decode_microbatch(gw, w.prompt_tokens, w.prompt_offsets, cap, w.target_lens, 0)
    assert np.array_equal(r["lens"], np.minimum(w.target_lens, cap))
    assert np.array_equal(r["failed"].astype(bool), w.target_lens > cap)
    for i in (0, 7, 15):
        check_tokens_teacher_forced(om, w.prompt(i), r["tokens"][i, :int(r["lens"][i])], what=f"row {i}")


def test_exact_ties_pick_the_lowest_token_id(tiny):
    """Every LM-head row identical -> all logits of a position are bit-equal -> greedy must emit id 0 (the
    oracle's rule: lowest index on exact ties), on the prompt forward and on every decode step."""
    W, om, gw = tiny
    W2 = [t.copy() for t in W]
    W2[-1][:] = W2[-1][17]
    gw2 = ss.Weights(synth.TINY, W2)
    try:
        w = synth.make_workload(1)
        r = ss.ss_decode_microbatch(gw2, w.prompt_tokens, w.prompt_offsets, 12, w.target_lens, 0)
        ref = OracleModel(synth.TINY, W2, "f64").greedy_microbatch(w.prompt_tokens, w.prompt_offsets, 12, w.target_lens)
        assert (ref["tokens"][ref["tokens"] >= 0] == 0).all()
        assert np.array_equal(r["tokens"], ref["tokens"])
    finally:
        gw2.close()


def test_non_finite_logits_and_huge_keys_still_give_ids_inside_the_vocabulary(tiny):
    """The token id feeds the next step's embedding lookup, so it must be a valid id whatever the arithmetic does:
    a row whose logits are all NaN yields id 0 greedily (no logit compares greater than the start value) and
    vocab-1 when sampled (no chunk of the CDF exceeds the draw); keys beyond the half range are stored saturated,
    so the softmax stays finite."""
    W, om, gw = tiny
    w = synth.make_workload(1)
    nan_head = [t.copy() for t in W]
    nan_head[-1][:] = 0x7FC0                                   # bf16 quiet NaN in every LM-head weight
    g1 = ss.Weights(synth.TINY, nan_head)
    try:
        r = ss.ss_decode_microbatch(g1, w.prompt_tokens, w.prompt_offsets, 6, w.target_lens, 0)
        emitted = r["tokens"][r["tokens"] >= 0]
        assert np.array_equal(r["lens"], np.minimum(w.target_lens, 6)) and (emitted == 0).all()
        draws = synth.make_draws(w.n, 6, seed=3)
        g = ss.ss_generate_microbatch(g1, w.prompt_tokens, w.prompt_offsets, 6, temperature=0.7, draws=draws,
                                      target_lens=w.target_lens, sync_every=1)
        emitted = g["tokens"][g["tokens"] >= 0]
        assert (emitted == synth.TINY.vocab - 1).all()
    finally:
        g1.close()
    big_k = [t.copy() for t in W]
    for l in range(synth.TINY.n_layers):                       # wk of every layer scaled by 2^20: |k| far above 65504
        wk = big_k[1 + 9 * l + 2]
        big_k[1 + 9 * l + 2] = synth.f32_to_bf16_bits(synth.bf16_bits_to_f32(wk) * float(2 ** 20))
    g2 = ss.Weights(synth.TINY, big_k)
    try:
        r = ss.ss_decode_microbatch(g2, w.prompt_tokens, w.prompt_offsets, 6, w.target_lens, 0)
        emitted = r["tokens"][r["tokens"] >= 0]
        assert np.array_equal(r["lens"], np.minimum(w.target_lens, 6))
        assert ((emitted >= 0) & (emitted < synth.TINY.vocab)).all()
        lg = ss.ss_forward_logits(g2, w.prompt_tokens[:w.prompt_offsets[2]], w.prompt_offsets[:3], w.prompt_lens[:2])
        assert np.isfinite(lg).all()
    finally:
        g2.close()


# ------------------------------------------------------------------ whole group
@pytest.mark.parametrize("flags", [(), ("SORT", "BIN", "FCR"), ("SORT", "BIN", "FCR", "VBS", "COMPACT"),
                                   ("SORT", "FCR", "VBS")])
def test_tiny_group_every_policy_same_answers(tiny, flags):
    """The schedule must not change any query's output (the paper's 'without compromising' claim):
    lengths exact, counters equal to the accounting oracle, tokens checked against the model oracle."""
    W, om, gw = tiny
    w = synth.make_group(synth.TINY, 96, 31337, ("uniform", 4, 24), ("lognormal", 12.0, 0.7, 1, 40), 0.3, 40, 8,
                         flags, base_batch=4, max_batch=32)
    pol = ss.make_policy(flags, 4, 40, 32)
    pred = w.pred_lens if "SORT" in flags else None
    _say(f"tiny group of 96, flags={flags}")
    r = ss.ss_run_group(gw, w.prompt_tokens, w.prompt_offsets, w.target_lens, pred, 8 if "BIN" in flags else 0, pol)
    assert np.array_equal(r["lens"], w.target_lens)
    ref = so.run_group(pred, w.target_lens, 8 if "BIN" in flags else 0,
                       so.Policy(flags=flags, base_batch=4, l_max=40, max_batch=32))
    s = r["stats"]
    assert s["steps"] == ref["steps"] and s["padded_row_steps"] == ref["padded_row_steps"]
    assert s["n_failed"] == ref["n_failed"] and s["useful_tokens"] == ref["useful_tokens"]
    assert s["n_mb_first"] == ref["first"].n_mb and s["n_mb_failure"] == ref["second"].n_mb
    want_rows = ref["live_row_steps"] if "COMPACT" in flags else ref["padded_row_steps"]
    assert s["computed_row_steps"] == want_rows
    for i in range(0, w.n, 5):
        t = int(w.target_lens[i])
        assert (r["tokens"][i, t:] == -1).all()
        check_tokens_teacher_forced(om, w.prompt(i), r["tokens"][i, :t], what=f"query {i}")


def test_group_results_do_not_depend_on_microbatches_in_flight(tiny):
    """Two to four micro-batches in flight (as many host threads, streams and workspaces) against one at a time: every
    query's tokens and every counter of the group are the same, for known lengths and for sampled rows that end
    by themselves, with failures and a recomputation pass in both."""
    W, om, gw = tiny
    flags = ("SORT", "BIN", "FCR", "VBS", "COMPACT")
    w = synth.make_group(synth.TINY, 128, 777, ("uniform", 4, 30), ("lognormal", 14.0, 0.7, 1, 48), 0.3, 48, 8,
                         flags, base_batch=4, max_batch=32)
    pol = ss.make_policy(flags, 4, 48, 32)
    draws = synth.make_draws(w.n, w.l_max, seed=11)
    counters = ("steps", "padded_row_steps", "computed_row_steps", "n_failed", "useful_tokens", "n_mb_first",
                "n_mb_failure", "prompt_tokens", "polls", "idle_steps")
    got = {}
    try:
        for lanes in (1, 2, 4, 3):
            gw.set_option(ss.SS_OPT_IN_FLIGHT, lanes)
            _say(f"tiny group of {w.n}, {lanes} in flight")
            a = ss.ss_run_group(gw, w.prompt_tokens, w.prompt_offsets, w.target_lens, w.pred_lens, 8, pol)
            b = ss.ss_run_group_generate(gw, w.prompt_tokens, w.prompt_offsets, w.pred_lens, 8, pol, eos_id=-1,
                                         temperature=0.7, draws=draws, target_lens=w.target_lens, sync_every=1)
            c = ss.ss_run_group(gw, w.prompt_tokens, w.prompt_offsets, w.target_lens, None, 0,
                                ss.make_policy((), 4, 48, 32))
            if not got:
                got = dict(a=a, b=b, c=c)
                assert a["stats"]["n_failed"] >= 1 and a["stats"]["n_mb_first"] >= 8
                continue
            for k, r in (("a", a), ("b", b), ("c", c)):
                assert np.array_equal(r["tokens"], got[k]["tokens"]), k
                assert np.array_equal(r["lens"], got[k]["lens"]), k
                for name in counters:
                    assert r["stats"][name] == got[k]["stats"][name], (k, name)
    finally:
        gw.set_option(ss.SS_OPT_IN_FLIGHT, ss.SS_IN_FLIGHT_DEFAULT)
    with pytest.raises(ss.SsError):
        gw.set_option(ss.SS_OPT_IN_FLIGHT, ss.SS_IN_FLIGHT_MAX + 1)
    with pytest.raises(ss.SsError):
        gw.set_option(ss.SS_OPT_IN_FLIGHT, 0)


def test_an_error_in_one_microbatch_ends_the_group_call_cleanly(tiny):
    """One query's prompt leaves no room for its cap (prompt + cap > 4096 positions): whichever lane meets its
    micro-batch reports the error, the other lane stops after the micro-batch it is on, the call returns the error
    with its message, and the handle works afterwards - with one, two and four micro-batches in flight."""
    W, om, gw = tiny
    w = synth.make_group(synth.TINY, 40, 4321, ("uniform", 4, 20), ("uniform", 1, 12), 0.3, 12, 4, ("SORT", "BIN", "FCR"),
                         base_batch=4, max_batch=4)
    pol = ss.make_policy(("SORT", "BIN", "FCR"), 4, 12, 4)
    good = ss.ss_run_group(gw, w.prompt_tokens, w.prompt_offsets, w.target_lens, w.pred_lens, 4, pol)
    rng = np.random.default_rng(1)
    prompts = [w.prompt(i) for i in range(w.n)]
    prompts[17] = rng.integers(0, synth.TINY.vocab, size=4095).astype(np.int32)      # 4095 + any cap >= 4 > 4096
    toks = np.concatenate(prompts).astype(np.int32)
    offs = np.concatenate([[0], np.cumsum([len(p) for p in prompts])]).astype(np.int32)
    try:
        for lanes in (4, 2, 1):
            gw.set_option(ss.SS_OPT_IN_FLIGHT, lanes)
            _say(f"group with one impossible query, {lanes} in flight")
            with pytest.raises(ss.SsError) as e:
                ss.ss_run_group(gw, toks, offs, w.target_lens, w.pred_lens, 4, pol)
            assert e.value.code == ss.SS_EINVAL and "positions" in str(e.value)
            again = ss.ss_run_group(gw, w.prompt_tokens, w.prompt_offsets, w.target_lens, w.pred_lens, 4, pol)
            assert np.array_equal(again["tokens"], good["tokens"]) and again["stats"]["steps"] == good["stats"]["steps"]
    finally:
        gw.set_option(ss.SS_OPT_IN_FLIGHT, ss.SS_IN_FLIGHT_DEFAULT)


def test_runs_are_bit_repeatable(tiny, wide2):
    """Race canary: every reduction is ordered (no float atomics), so two runs of the same call must agree
    bit for bit - logits and tokens, skinny and tiled kernels, padded and compacted."""
    W, om, gw = tiny
    w = synth.make_group(synth.TINY, 90, 99, ("uniform", 4, 30), ("uniform", 1, 20), None, 20, 0, ())
    a = ss.ss_forward_logits(gw, w.prompt_tokens, w.prompt_offsets, w.prompt_lens)
    b = ss.ss_forward_logits(gw, w.prompt_tokens, w.prompt_offsets, w.prompt_lens)
    assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
    for flags in (0, ss.SS_COMPACT):
        r1 = ss.ss_decode_microbatch(gw, w.prompt_tokens, w.prompt_offsets, 16, w.target_lens, flags)
        r2 = ss.ss_decode_microbatch(gw, w.prompt_tokens, w.prompt_offsets, 16, w.target_lens, flags)
        assert np.array_equal(r1["tokens"], r2["tokens"])
    shape, W2, om2, gw2 = wide2
    w2 = synth.make_workload(3, n=16, shape=shape)
    r1 = ss.ss_decode_microbatch(gw2, w2.prompt_tokens, w2.prompt_offsets, 8, w2.target_lens, 0)
    r2 = ss.ss_decode_microbatch(gw2, w2.prompt_tokens, w2.prompt_offsets, 8, w2.target_lens, 0)
    assert np.array_equal(r1["tokens"], r2["tokens"])


# ------------------------------------------------------------------ error paths that need a handle
def test_limits_longest_row_and_largest_batch(tiny):
    """The documented maxima: a row that fills all 4096 positions (prompt 4090 + 6 generated; the last decode
    attention reads 4095 slots in 16 passes), one position more is rejected; a micro-batch of 1024 rows (the
    bookkeeping kernel's limit, one thread per row), 1025 are rejected; and the smallest call (1 row, 1 token)."""
    W, om, gw = tiny
    rng = np.random.default_rng(4096)
    long_prompt = rng.integers(0, synth.TINY.vocab, size=4090).astype(np.int32)
    forced = rng.integers(0, synth.TINY.vocab, size=6).astype(np.int32)
    seq = np.concatenate([long_prompt, forced])
    _say("tiny row of 4096 positions, teacher-forced")
    got = ss.ss_forward_logits(gw, seq, [0, 4096], [4090])
    ref = om.teacher_forced(seq, first=4089)
    assert got.shape == ref.shape == (7, synth.TINY.vocab)
    check_logits(got, ref, "4096 positions")
    r = ss.ss_decode_microbatch(gw, long_prompt, [0, 4090], 6, [6])
    assert r["lens"].tolist() == [6] and (r["tokens"][0] >= 0).all()
    check_tokens_teacher_forced(om, long_prompt, r["tokens"][0], what="4096 positions, generated")
    with pytest.raises(ss.SsError) as e:
        ss.ss_decode_microbatch(gw, long_prompt, [0, 4090], 7, [7])
    assert e.value.code == ss.SS_EINVAL

    _say("tiny 1024-row micro-batch")
    w = synth.make_group(synth.TINY, 1025, 2024, ("uniform", 3, 9), ("uniform", 1, 5), None, 5, 0, ())
    toks, offs = synth.gather_prompts(w, range(1024))
    t = w.target_lens[:1024]
    for flags in (0, ss.SS_COMPACT):
        r = ss.ss_decode_microbatch(gw, toks, offs, 4, t, flags)
        assert np.array_equal(r["lens"], np.minimum(t, 4)) and np.array_equal(r["failed"].astype(bool), t > 4)
        assert r["stats"]["row_steps"] == (int(np.minimum(t, 4).sum()) if flags else 1024 * int(min(4, t.max())))
        for j in (0, 63, 64, 1000, 1023):
            L = int(r["lens"][j])
            assert (r["tokens"][j, :L] >= 0).all() and (r["tokens"][j, L:] == -1).all()
            check_tokens_teacher_forced(om, w.prompt(j), r["tokens"][j, :L], what=f"1024 rows, row {j}")
    with pytest.raises(ss.SsError) as e:
        ss.ss_decode_microbatch(gw, w.prompt_tokens, w.prompt_offsets, 4, w.target_lens, 0)
    assert e.value.code == ss.SS_EINVAL

    r = ss.ss_decode_microbatch(gw, [5], [0, 1], 1, [1])
    assert r["lens"].tolist() == [1] and r["stats"]["steps"] == 1
    check_tokens_teacher_forced(om, np.array([5], np.int32), r["tokens"][0], what="1 row, 1 token")


def test_invalid_generation_arguments(tiny):
    W, om, gw = tiny
    good = dict(prompt_tokens=[1, 2, 3, 4], prompt_offsets=[0, 2, 4], max_new=4, target_lens=[2, 3])
    for bad in (dict(prompt_offsets=[0, 2, 2]), dict(prompt_offsets=[1, 2, 4]), dict(prompt_tokens=[1, 2, 3, 1024]),
                dict(prompt_tokens=[1, -2, 3, 4]), dict(max_new=0), dict(target_lens=[2, 0]), dict(max_new=5000),
                dict(flags=ss.SS_SORT)):
        args = {**good, **bad}
        with pytest.raises(ss.SsError) as e:
            ss.ss_decode_microbatch(gw, **args)
        assert e.value.code == ss.SS_EINVAL
    r = ss.ss_decode_microbatch(gw, **good)       # the handle still works after rejected calls
    assert r["lens"].tolist() == [2, 3]


def test_small_weights_keep_their_value_on_the_device(tiny):
    """Weights live on the device as IEEE half.  A projection whose bf16 weights are all of magnitude ~1e-5 (half's
    subnormal range starts at 6.1e-5; bf16 values down to 2^-17 = 7.6e-6 are exact in it, smaller ones are off by
    less than 3e-8) must still give the oracle's logits: nothing is flushed to zero on the way through the matrix
    cores.  The LM head is scaled by 2^-11, so every logit comes from such weights; a down projection scaled the
    same way checks a matrix in the middle of the network."""
    W, om, gw = tiny
    specs = synth.TINY.tensor_specs()
    names = [n for n, _ in specs]
    w = synth.make_workload(1)
    for which in ([len(W) - 1], [i for i, n in enumerate(names) if n.endswith("wd")][:1]):
        W2 = list(W)
        for i in which:
            f = (W[i].astype(np.uint32) << 16).view(np.float32) * np.float32(2.0 ** -11)
            W2[i] = synth.f32_to_bf16_bits(f)       # a power of two: exact
            mag = np.abs((W2[i].astype(np.uint32) << 16).view(np.float32))
            assert np.median(mag) < 2e-5 and (mag < 6.1e-5).mean() > 0.95
        om2 = OracleModel(synth.TINY, W2, "f64")
        gw2 = ss.Weights(synth.TINY, W2)
        try:
            _say(f"tiny, tensor {names[which[0]]} scaled into half's subnormal range")
            got = ss.ss_forward_logits(gw2, w.prompt_tokens, w.prompt_offsets, w.prompt_lens)
            ref = np.stack([om2.teacher_forced(w.prompt(i), first=len(w.prompt(i)) - 1)[0] for i in range(w.n)])
            assert np.abs(ref).max() > 0
            check_logits(got, ref, f"{names[which[0]]} x 2^-11")
        finally:
            gw2.close()


def test_unknown_option_is_refused(tiny):
    W, om, gw = tiny
    for opt, val in ((1, 0), (99, 0), (ss.SS_OPT_IN_FLIGHT, -1)):
        with pytest.raises(ss.SsError) as e:
            gw.set_option(opt, val)
        assert e.value.code == ss.SS_EINVAL


def test_second_call_on_a_busy_handle_is_refused(tiny):
    """One call at a time per handle: while a long call runs on one thread, a call on the same handle from
    another thread returns SS_ESTATE at once, disturbs nothing, and the handle works afterwards."""
    import threading
    W, om, gw = tiny
    w = synth.make_group(synth.TINY, 512, 4242, ("uniform", 8, 32), ("uniform", 24, 48), None, 48, 0, ())
    pol = ss.make_policy((), 16, 48, 256)
    import time
    started, result, refused = threading.Event(), {}, []

    def long_call():
        started.set()
        while "r" not in result:          # the short call may hold the handle at the instant this one starts
            try:
                result["r"] = ss.ss_run_group(gw, w.prompt_tokens, w.prompt_offsets, w.target_lens, None, 0, pol)
            except ss.SsError as e:
                assert e.code == ss.SS_ESTATE and "in flight" in str(e)
                refused.append("long")

    a = threading.Thread(target=long_call)
    a.start()
    started.wait()
    while a.is_alive():
        time.sleep(0.002)
        try:
            ss.ss_decode_microbatch(gw, [1, 2, 3], [0, 3], 2, [2])
        except ss.SsError as e:
            assert e.code == ss.SS_ESTATE and "in flight" in str(e)
            refused.append("short")
    a.join()
    assert "short" in refused, "the long call never overlapped a second one"
    assert np.array_equal(result["r"]["lens"], w.target_lens)               # the long call was not disturbed
    r = ss.ss_decode_microbatch(gw, [1, 2, 3], [0, 3], 2, [2])               # and the handle is free again
    assert r["lens"].tolist() == [2]
    for i in (0, 511):
        check_tokens_teacher_forced(om, w.prompt(i), result["r"]["tokens"][i, :int(w.target_lens[i])], upto=8,
                                    what=f"query {i} of the overlapped call")
