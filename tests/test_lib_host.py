"""CPU tests of the C-ABI library: it loads, exports every symbol the header declares, rejects bad
arguments, and its host scheduler is bit-exact with the scheduler oracle.  No GPU is touched."""
import ctypes as C
import os
import re
import zlib

import numpy as np
import pytest

from paper_2305_13144_amd import binding as ss
from paper_2305_13144_amd import synth
from oracle import sched_oracle as so

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(ss.LIB_PATH):
        from paper_2305_13144_amd import build
        build.build()
    return ss.lib()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "ss.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = sorted(set(re.findall(r"\b(ss_[a-z_]+)\s*\(", header)))
    assert declared == sorted(ss.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def _oracle_policy(flags, b0, lmax, maxb, rule="clamp_floor"):
    return so.Policy(flags=tuple(flags), base_batch=b0, l_max=lmax, max_batch=maxb, vbs_rule=rule)


def _as_pairs(plan):
    return [(list(m.idx), m.cap) for m in plan]


FLAG_SETS = [(), ("SORT",), ("SORT", "FCR"), ("SORT", "BIN"), ("SORT", "BIN", "FCR"), ("SORT", "FCR", "VBS"),
             ("SORT", "BIN", "FCR", "VBS"), ("SORT", "BIN", "VBS"), ("SORT", "BIN", "FCR", "VBS", "COMPACT")]


@pytest.mark.parametrize("cfg", [2, 3, 4, 5])
def test_schedule_bit_exact_on_configs(lib, cfg):
    w = synth.make_workload(cfg)
    pol = ss.make_policy(w.flags, w.base_batch, w.l_max, w.max_batch)
    got = ss.ss_schedule(w.pred_lens, w.n, w.bin_width, pol)
    want = so.schedule(w.pred_lens, w.n, w.bin_width, _oracle_policy(w.flags, w.base_batch, w.l_max, w.max_batch))
    assert got == _as_pairs(want)
    if w.pred_lens is not None:
        acc = so.account(want, w.target_lens)
        gotf = ss.ss_schedule_failures(w.pred_lens, w.n, sorted(acc.failed), w.bin_width, pol)
        wantf = so.schedule_failures(w.pred_lens, acc.failed, w.bin_width,
                                     _oracle_policy(w.flags, w.base_batch, w.l_max, w.max_batch))
        assert gotf == _as_pairs(wantf)


@pytest.mark.parametrize("flags", FLAG_SETS)
@pytest.mark.parametrize("rule", ["clamp_floor", "paper_pow2"])
def test_schedule_bit_exact_random_groups(lib, flags, rule):
    rng = np.random.default_rng(zlib.crc32(repr((flags, rule)).encode()))
    for trial in range(25):
        n = int(rng.integers(1, 300))
        lmax = int(rng.choice([48, 100, 512, 1024]))
        w = int(rng.choice([1, 7, 50, 64, lmax]))      # cell 1: neighbouring lengths are neighbouring bins
        b0 = int(rng.choice([1, 2, 16]))
        maxb = int(rng.choice([b0, 64, 256]))
        pred = rng.integers(1, int(lmax * 1.3) + 2, size=n).astype(np.int32)
        binw = w if "BIN" in flags else int(rng.choice([0, w]))
        pol = ss.make_policy(flags, b0, lmax, maxb, ss.SS_VBS_PAPER_POW2 if rule == "paper_pow2" else 0)
        opol = _oracle_policy(flags, b0, lmax, maxb, rule)
        got = ss.ss_schedule(pred if "SORT" in flags else None, n, binw, pol)
        want = so.schedule(pred if "SORT" in flags else None, n, binw, opol)
        assert got == _as_pairs(want), (flags, rule, trial)
        if "SORT" in flags:
            failed = sorted(rng.choice(n, size=int(rng.integers(0, n + 1)), replace=False).tolist())
            gotf = ss.ss_schedule_failures(pred, n, failed, binw, pol)
            wantf = so.schedule_failures(pred, failed, binw, opol)
            assert gotf == _as_pairs(wantf)


def test_library_batch_size_rules_for_every_length(lib):
    """The batch size the library allows for a scheduled length L, read off a group of equal predictions (the first
    chunk is as large as allowed), against the oracle's rule for every L; and predictions without SS_SORT change nothing."""
    n = 300
    for L in range(43, 360):        # from 43 up the power-of-two rule allows at most 256 rows: the group can show it
        pred = np.full(n, L, np.int32)
        got = ss.ss_schedule(pred, n, 0, ss.make_policy(("SORT", "VBS"), 16, 512, 256, ss.SS_VBS_PAPER_POW2))
        assert len(got[0][0]) == so.vbs_paper_pow2(L), L
        got = ss.ss_schedule(pred, n, 0, ss.make_policy(("SORT", "VBS"), 16, 512, 256))
        assert len(got[0][0]) == so.vbs_clamp_floor(L, 16, 512, 256), L
    pred = np.array([30, 120, 55, 49, 260, 51, 100, 7], np.int32)
    got = ss.ss_schedule(pred, 8, 50, ss.make_policy((), 3, 64))
    assert got == [([0, 1, 2], 64), ([3, 4, 5], 64), ([6, 7], 64)]


def test_schedule_rejects_bad_arguments(lib):
    pol = ss.make_policy(("SORT", "BIN", "FCR"))
    pred = np.array([10, 20, 30], np.int32)
    cases = [
        dict(pred=pred, n=0, bin=50, pol=pol),
        dict(pred=pred, n=3, bin=-1, pol=pol),
        dict(pred=np.array([10, 0, 30], np.int32), n=3, bin=50, pol=pol),
        dict(pred=None, n=3, bin=50, pol=pol),
        dict(pred=pred, n=3, bin=0, pol=pol),                                        # SS_BIN needs a bin
        dict(pred=pred, n=3, bin=50, pol=ss.make_policy(("BIN",))),                  # SS_BIN needs SS_SORT
        dict(pred=pred, n=3, bin=50, pol=ss.make_policy(("VBS",))),
        dict(pred=pred, n=3, bin=50, pol=ss.make_policy(("SORT",), base_batch=0)),
        dict(pred=pred, n=3, bin=50, pol=ss.make_policy(("SORT",), base_batch=16, max_batch=8)),
        dict(pred=pred, n=3, bin=50, pol=ss.make_policy(("SORT",), base_len=0)),
        dict(pred=pred, n=3, bin=50, pol=ss.make_policy(("SORT",), vbs_rule=7)),
    ]
    for c in cases:
        with pytest.raises(ss.SsError) as e:
            ss.ss_schedule(c["pred"], c["n"], c["bin"], c["pol"])
        assert e.value.code == ss.SS_EINVAL and len(str(e.value)) > 20
    out = C.POINTER(ss.ss_plan)()
    assert lib.ss_schedule(None, 3, 0, None, C.byref(out)) == ss.SS_EINVAL
    assert lib.ss_schedule(None, 3, 0, C.byref(ss.make_policy(())), None) == ss.SS_EINVAL
    for bad in ([5], [3], [-1], [0, 3]):                      # indices are 0 .. n-1
        with pytest.raises(ss.SsError) as e:
            ss.ss_schedule_failures(pred, 3, bad, 50, pol)
        assert e.value.code == ss.SS_EINVAL
    assert ss.ss_schedule_failures(pred, 3, [2], 50, pol) == [([2], 512)]
    with pytest.raises(ss.SsError):                           # index n is refused as such, not for what lies behind the array
        ss.ss_schedule_failures(np.array([10, 20, 30, 40], np.int32), 3, [3], 50, pol)


def test_generation_entry_points_reject_null_without_touching_a_gpu(lib):
    assert lib.ss_decode_microbatch(None, None, None, 1, 1, None, 0, None, None, None, None, None) == ss.SS_EINVAL
    assert b"NULL" in lib.ss_last_error()
    assert lib.ss_forward_logits(None, None, None, 1, None, 0, None, None) == ss.SS_EINVAL
    assert lib.ss_run_group(None, None, None, 1, None, None, 0, None, None, None, None, None) == ss.SS_EINVAL
    assert lib.ss_bench_decode_step(None, None, 1, 1, 1, None, None) == ss.SS_EINVAL
    assert lib.ss_bench_decode_steps_in_flight(None, None, 1, 1, 1, 2, None) == ss.SS_EINVAL
    assert lib.ss_bench_weight_stream(None, 1, 1, None, None, None) == ss.SS_EINVAL
    assert lib.ss_bench_read_stream(None, 1, None, None, None) == ss.SS_EINVAL
    assert lib.ss_generate_microbatch(None, None, None, 1, 1, None, 0, None, None, None, None, None) == ss.SS_EINVAL
    assert b"NULL" in lib.ss_last_error()
    assert lib.ss_run_group_generate(None, None, None, 1, None, 0, None, None, None, None, None, None) == ss.SS_EINVAL
    cfg = ss.ss_model_cfg(2, 250, 4, 64, 688, 1024, 1e4, 1e-6)       # n_heads*head_dim != d_model
    h = C.c_void_p()
    arr = (C.c_void_p * 21)()
    assert lib.ss_weights_create(C.byref(cfg), arr, ss.SS_BF16, C.byref(h)) == ss.SS_EINVAL
    lib.ss_weights_destroy(None)
    lib.ss_plan_free(None)


_NO_MEMORY_CHILD = r"""
import ctypes as C, resource, sys
from paper_2305_13144_amd import binding as ss
L = ss.lib()
pol = ss.make_policy((), 16, 512, 256)            # vanilla batching: the predictions are not read
plan = C.POINTER(ss.ss_plan)()
assert L.ss_schedule(None, 1000, 0, C.byref(pol), C.byref(plan)) == ss.SS_OK and plan.contents.n_mb == 63
L.ss_plan_free(plan)
# cap the address space a little above what the process holds now: a plan over 2^31 - 1 queries needs three arrays
# of that many int32, which cannot be had
with open("/proc/self/statm") as f:
    held = int(f.read().split()[0]) * resource.getpagesize()
resource.setrlimit(resource.RLIMIT_AS, (held + (1 << 30), held + (1 << 30)))
plan = C.POINTER(ss.ss_plan)()
rc = L.ss_schedule(None, 2**31 - 1, 0, C.byref(pol), C.byref(plan))
print("rc", rc, "plan", bool(plan), "msg", L.ss_last_error().decode())
failed = (C.c_int32 * 1)(0)
rc2 = L.ss_schedule(None, 100, 0, C.byref(pol), C.byref(plan))    # and the library goes on working
print("rc2", rc2, "n_mb", plan.contents.n_mb)
"""


def test_a_plan_that_does_not_fit_host_memory_is_an_error_code(lib):
    """No C++ exception crosses the C ABI: the scheduler answers SS_ENOMEM when its arrays cannot be allocated, sets no
    plan, and the next call works.  Runs in a child process because it lowers the process's address-space limit."""
    import subprocess
    import sys
    out = subprocess.run([sys.executable, "-c", _NO_MEMORY_CHILD], cwd=ROOT, capture_output=True, text=True, timeout=120)
    assert out.returncode == 0, out.stderr[-2000:]
    lines = out.stdout.strip().splitlines()
    assert lines[0].startswith(f"rc {ss.SS_ENOMEM} plan False msg host allocation failed"), lines
    assert lines[1] == "rc2 0 n_mb 7", lines


def test_library_plans_have_the_properties_the_method_states(lib):
    """Properties that Sec. 4.1 states of a plan, checked on the library's output for generated groups and policies
    without going through the scheduler oracle: a plan is a partition of the group; with sorting the scheduled lengths
    never decrease along it; the cap is the largest scheduled length of the micro-batch under FCR (at most the global
    limit) and the global limit otherwise; a micro-batch never holds more rows than its longest scheduled length allows;
    with bins every micro-batch lies inside one bin."""
    from hypothesis import given, settings, strategies as st

    flag_sets = [f for f in FLAG_SETS if "COMPACT" not in f]

    @settings(max_examples=300, deadline=None)
    @given(pred=st.lists(st.integers(1, 700), min_size=1, max_size=120), flags=st.sampled_from(flag_sets),
           b0=st.sampled_from([1, 2, 3, 16]), lmax=st.sampled_from([32, 100, 512]), w=st.sampled_from([1, 7, 50, 64]),
           maxb=st.sampled_from([16, 64, 256]), pow2=st.booleans())
    def check(pred, flags, b0, lmax, w, maxb, pow2):
        n = len(pred)
        binw = w if "BIN" in flags else 0
        rule = ss.SS_VBS_PAPER_POW2 if pow2 else ss.SS_VBS_CLAMP_FLOOR
        plan = ss.ss_schedule(np.array(pred, np.int32), n, binw, ss.make_policy(flags, b0, lmax, max(maxb, b0), rule))
        order = [i for idx, _ in plan for i in idx]
        assert sorted(order) == list(range(n))
        if "SORT" not in flags:
            assert order == list(range(n)) and all(cap == lmax and len(idx) <= b0 for idx, cap in plan)
            return
        top = -(-lmax // binw) * binw if binw else None
        key = [min(-(-p // binw) * binw, top) if binw else p for p in pred]
        assert all(key[a] <= key[b] for a, b in zip(order, order[1:]))
        for idx, cap in plan:
            longest = max(key[i] for i in idx)
            assert cap == (min(longest, lmax) if "FCR" in flags else lmax)
            if "VBS" in flags:
                if pow2:
                    allowed = 16 if longest >= 300 else min((2 ** k for k in range(15)), key=lambda b: abs(b - 12800 / longest))
                else:
                    allowed = max(b0, min(max(maxb, b0), b0 * lmax // longest))
            else:
                allowed = b0
            assert len(idx) <= allowed
            if binw:
                assert len({key[i] for i in idx}) == 1

    check()
