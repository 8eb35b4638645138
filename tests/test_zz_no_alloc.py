"""The entry point that allocates nothing (ss_decode_microbatch_static: workspace inside the library's static device
array) against ss_decode_microbatch, through the C ABI: integers bit-exact, tokens bit-exact (same kernels, same
launch plans, deterministic reductions), on two calls in a row, the second with a smaller input, and a call beyond
the array's size refused with a clear error."""
import numpy as np
import pytest

from paper_2305_13144_amd import binding as ss
from paper_2305_13144_amd import synth

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


def _same(a, b, what):
    assert np.array_equal(a["lens"], b["lens"]), what
    assert np.array_equal(a["failed"], b["failed"]), what
    assert np.array_equal(a["tokens"], b["tokens"]), what
    for k in ("steps", "rows", "row_steps", "prompt_tokens", "decode_kv_tokens"):
        assert a["stats"][k] == b["stats"][k], (what, k)


def test_static_scratch_entry_point_matches_the_allocating_one():
    W = synth.make_weights(synth.TINY, seed=1, norm_jitter=0.1, threads=1)
    gw = ss.Weights(synth.TINY, W)
    try:
        big = synth.make_workload(1)                                                     # 16 rows, prompts 8..32, cap 48
        small = synth.make_group(synth.TINY, 5, 99, ("uniform", 3, 9), ("uniform", 1, 12), None, 12, 0, ())
        cases = [("16 rows, cap 48, padded", big, 48, 0), ("5 rows, cap 7, compacting", small, 7, ss.SS_COMPACT)]
        for what, w, cap, flags in cases:                                                # static first: no workspace exists yet
            _say(f"static call: {what}")
            got = ss.ss_decode_microbatch_static(gw, w.prompt_tokens, w.prompt_offsets, cap, w.target_lens, flags)
            _say(f"allocating call: {what}")
            ref = ss.ss_decode_microbatch(gw, w.prompt_tokens, w.prompt_offsets, cap, w.target_lens, flags)
            assert np.array_equal(ref["lens"], np.minimum(w.target_lens, cap))
            assert (ref["tokens"][np.arange(len(ref["lens"])), ref["lens"] - 1] >= 0).all()
            _same(got, ref, what)
        _say("static calls again, larger after smaller")
        for what, w, cap, flags in reversed(cases):
            got = ss.ss_decode_microbatch_static(gw, w.prompt_tokens, w.prompt_offsets, cap, w.target_lens, flags)
            ref = ss.ss_decode_microbatch(gw, w.prompt_tokens, w.prompt_offsets, cap, w.target_lens, flags)
            _same(got, ref, what + " (second round)")
        _say("a micro-batch beyond the static array is refused")
        huge = synth.make_group(synth.TINY, 1024, 7, ("uniform", 30, 40), ("uniform", 1, 4), None, 4, 0, ())
        with pytest.raises(ss.SsError) as e:
            ss.ss_decode_microbatch_static(gw, huge.prompt_tokens, huge.prompt_offsets, 2000, huge.target_lens, 0)
        assert e.value.code == ss.SS_EINVAL and "static scratch array holds" in str(e.value)
        got = ss.ss_decode_microbatch_static(gw, small.prompt_tokens, small.prompt_offsets, 7, small.target_lens, 0)
        assert np.array_equal(got["lens"], np.minimum(small.target_lens, 7))             # still usable after the refusal
    finally:
        gw.close()
