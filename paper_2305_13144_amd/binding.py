"""ctypes binding of libss.so: argument marshalling only, same names as the C ABI.

Every step of the path runs in the library's kernels; nothing here computes.  The library
must be built (``python -m paper_2305_13144_amd.build``) - there is no fallback: a missing
library raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libss.so")

SS_OK, SS_EINVAL, SS_ENOMEM, SS_EDEVICE, SS_ESTATE = 0, -1, -2, -3, -4
SS_SORT, SS_BIN, SS_FCR, SS_VBS, SS_COMPACT = 1, 2, 4, 8, 16
SS_VBS_CLAMP_FLOOR, SS_VBS_PAPER_POW2 = 0, 1
SS_OPT_IN_FLIGHT, SS_IN_FLIGHT_MAX, SS_IN_FLIGHT_DEFAULT = 2, 4, 4
SS_BF16, SS_F32 = 0, 1
FLAG_BITS = dict(SORT=SS_SORT, BIN=SS_BIN, FCR=SS_FCR, VBS=SS_VBS, COMPACT=SS_COMPACT)

EXPORTS = ["ss_last_error", "ss_set_verbose", "ss_set_gemm_mode", "ss_schedule", "ss_schedule_failures", "ss_plan_free", "ss_weights_create",
           "ss_weights_destroy", "ss_set_option", "ss_decode_microbatch", "ss_decode_microbatch_static", "ss_forward_logits", "ss_run_group", "ss_generate_microbatch",
           "ss_run_group_generate", "ss_bench_decode_step", "ss_bench_decode_steps_in_flight", "ss_bench_weight_stream", "ss_bench_read_stream"]


class SsError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"libss error {code}: {msg}")
        self.code = code


class ss_policy(C.Structure):
    _fields_ = [("flags", C.c_uint32), ("base_batch", C.c_int32), ("base_len", C.c_int32), ("max_batch", C.c_int32),
                ("vbs_rule", C.c_int32)]


class ss_plan(C.Structure):
    _fields_ = [("n", C.c_int32), ("n_mb", C.c_int32), ("mb_offsets", C.POINTER(C.c_int32)),
                ("query_idx", C.POINTER(C.c_int32)), ("mb_cap", C.POINTER(C.c_int32))]


class ss_model_cfg(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_heads", C.c_int32), ("head_dim", C.c_int32),
                ("d_ffn", C.c_int32), ("vocab", C.c_int32), ("rope_base", C.c_float), ("rms_eps", C.c_float)]


class ss_stats(C.Structure):
    _fields_ = [("steps", C.c_int32), ("rows", C.c_int32), ("row_steps", C.c_int64), ("prompt_tokens", C.c_int64),
                ("decode_kv_tokens", C.c_int64), ("prefill_ms", C.c_double), ("decode_ms", C.c_double),
                ("polls", C.c_int32), ("idle_steps", C.c_int32)]


class ss_group_stats(C.Structure):
    _fields_ = [("n_mb_first", C.c_int32), ("n_mb_failure", C.c_int32), ("n_failed", C.c_int32),
                ("steps", C.c_int64), ("padded_row_steps", C.c_int64), ("computed_row_steps", C.c_int64),
                ("useful_tokens", C.c_int64), ("prompt_tokens", C.c_int64), ("wall_ms", C.c_double),
                ("plan_ms", C.c_double), ("prefill_ms", C.c_double), ("decode_ms", C.c_double),
                ("polls", C.c_int64), ("idle_steps", C.c_int64)]


class ss_gen_opts(C.Structure):
    _fields_ = [("eos_id", C.c_int32), ("temperature", C.c_float), ("draws", C.c_void_p),
                ("draws_stride", C.c_int32), ("seed", C.c_uint64), ("draw_ids", C.c_void_p),
                ("target_lens", C.c_void_p), ("sync_every", C.c_int32)]


def _struct_dict(s: C.Structure) -> dict:
    return {name: getattr(s, name) for name, _ in s._fields_}


_lib = None


def lib():
    """The loaded library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is missing: build it with `python -m paper_2305_13144_amd.build`")
        L = C.CDLL(LIB_PATH)
        vp, i32p = C.c_void_p, C.c_void_p
        L.ss_last_error.restype = C.c_char_p
        L.ss_set_verbose.argtypes = [C.c_int32]
        L.ss_set_verbose.restype = None
        L.ss_set_gemm_mode.argtypes = [C.c_int32]
        L.ss_set_gemm_mode.restype = None
        L.ss_schedule.argtypes = [i32p, C.c_int32, C.c_int32, C.POINTER(ss_policy), C.POINTER(C.POINTER(ss_plan))]
        L.ss_schedule_failures.argtypes = [i32p, C.c_int32, i32p, C.c_int32, C.c_int32, C.POINTER(ss_policy),
                                           C.POINTER(C.POINTER(ss_plan))]
        L.ss_plan_free.argtypes = [C.POINTER(ss_plan)]
        L.ss_plan_free.restype = None
        L.ss_weights_create.argtypes = [C.POINTER(ss_model_cfg), C.POINTER(vp), C.c_int32, C.POINTER(vp)]
        L.ss_set_option.argtypes = [vp, C.c_int32, C.c_int32]
        L.ss_weights_destroy.argtypes = [vp]
        L.ss_weights_destroy.restype = None
        L.ss_decode_microbatch.argtypes = [vp, i32p, i32p, C.c_int32, C.c_int32, i32p, C.c_uint32, i32p, i32p, vp,
                                           C.POINTER(ss_stats), vp]
        L.ss_decode_microbatch_static.argtypes = L.ss_decode_microbatch.argtypes
        L.ss_forward_logits.argtypes = [vp, i32p, i32p, C.c_int32, i32p, C.c_int32, vp, vp]
        L.ss_run_group.argtypes = [vp, i32p, i32p, C.c_int32, i32p, i32p, C.c_int32, C.POINTER(ss_policy), i32p, i32p,
                                   C.POINTER(ss_group_stats), vp]
        L.ss_generate_microbatch.argtypes = [vp, i32p, i32p, C.c_int32, C.c_int32, C.POINTER(ss_gen_opts), C.c_uint32,
                                             i32p, i32p, vp, C.POINTER(ss_stats), vp]
        L.ss_run_group_generate.argtypes = [vp, i32p, i32p, C.c_int32, i32p, C.c_int32, C.POINTER(ss_policy),
                                            C.POINTER(ss_gen_opts), i32p, i32p, C.POINTER(ss_group_stats), vp]
        L.ss_bench_decode_step.argtypes = [vp, i32p, C.c_int32, C.c_int32, C.c_int32, vp, vp]
        L.ss_bench_decode_steps_in_flight.argtypes = [vp, i32p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, vp]
        L.ss_bench_weight_stream.argtypes = [vp, C.c_int32, C.c_int32, vp, vp, vp]
        L.ss_bench_read_stream.argtypes = [vp, C.c_int32, vp, vp, vp]
        for name in EXPORTS:
            if name not in ("ss_last_error", "ss_set_verbose", "ss_set_gemm_mode", "ss_plan_free", "ss_weights_destroy"):
                getattr(L, name).restype = C.c_int
        _lib = L
    return _lib


def _check(rc: int) -> None:
    if rc != SS_OK:
        raise SsError(rc, lib().ss_last_error().decode())


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def ss_set_verbose(level: int) -> None:
    lib().ss_set_verbose(level)


def ss_set_gemm_mode(mode: int) -> None:
    lib().ss_set_gemm_mode(mode)


def make_policy(flags: Sequence[str] = (), base_batch: int = 16, base_len: int = 512, max_batch: int = 256,
                vbs_rule: int = SS_VBS_CLAMP_FLOOR) -> ss_policy:
    bits = 0
    for f in flags:
        bits |= FLAG_BITS[f]
    return ss_policy(bits, base_batch, base_len, max_batch, vbs_rule)


def _plan_to_py(pp) -> list:
    p = pp.contents
    offs = [p.mb_offsets[i] for i in range(p.n_mb + 1)]
    idx = [p.query_idx[i] for i in range(p.n)]
    out = [(idx[offs[k]:offs[k + 1]], p.mb_cap[k]) for k in range(p.n_mb)]
    lib().ss_plan_free(pp)
    return out


def ss_schedule(pred_lens, n: int, bin: int, policy: ss_policy) -> list:
    """-> [(query indices, cap), ...] in execution order."""
    pl = None if pred_lens is None else _i32(pred_lens)
    out = C.POINTER(ss_plan)()
    _check(lib().ss_schedule(_ptr(pl), n, bin, C.byref(policy), C.byref(out)))
    return _plan_to_py(out)


def ss_schedule_failures(pred_lens, n: int, failed_idx, bin: int, policy: ss_policy) -> list:
    pl = None if pred_lens is None else _i32(pred_lens)
    fi = _i32(failed_idx)
    out = C.POINTER(ss_plan)()
    _check(lib().ss_schedule_failures(_ptr(pl), n, _ptr(fi), len(fi), bin, C.byref(policy), C.byref(out)))
    return _plan_to_py(out)


class Weights:
    """Owns an ss_weights handle (device-resident packed model)."""

    def __init__(self, shape, tensors: Sequence[np.ndarray], src_dtype: int = SS_BF16):
        want = np.uint16 if src_dtype == SS_BF16 else np.float32
        self._keep = [np.ascontiguousarray(t, dtype=want) for t in tensors]
        n_expected = 3 + 9 * shape.n_layers
        if len(self._keep) != n_expected:
            raise ValueError(f"expected {n_expected} tensors, got {len(self._keep)}")
        cfg = ss_model_cfg(shape.n_layers, shape.d_model, shape.n_heads, shape.head_dim, shape.d_ffn, shape.vocab,
                           shape.rope_base, shape.rms_eps)
        arr = (C.c_void_p * len(self._keep))(*[t.ctypes.data for t in self._keep])
        h = C.c_void_p()
        _check(lib().ss_weights_create(C.byref(cfg), arr, src_dtype, C.byref(h)))
        self.h = h
        self.shape = shape
        self._keep = None   # the library copied everything

    def set_option(self, option: int, value: int) -> None:
        _check(lib().ss_set_option(self.h, option, value))

    def close(self) -> None:
        if getattr(self, "h", None):
            lib().ss_weights_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def ss_decode_microbatch(w: Weights, prompt_tokens, prompt_offsets, max_new: int, target_lens, flags: int = 0,
                         stream: Optional[int] = None, static: bool = False) -> dict:
    """static=True calls ss_decode_microbatch_static (workspace in the library's static device array)."""
    pt, po, tl = _i32(prompt_tokens), _i32(prompt_offsets), _i32(target_lens)
    B = len(tl)
    toks = np.empty((B, max_new), np.int32)
    lens = np.empty(B, np.int32)
    failed = np.empty(B, np.uint8)
    st = ss_stats()
    fn = lib().ss_decode_microbatch_static if static else lib().ss_decode_microbatch
    _check(fn(w.h, _ptr(pt), _ptr(po), B, max_new, _ptr(tl), flags, _ptr(toks), _ptr(lens), _ptr(failed), C.byref(st),
              stream))
    return dict(tokens=toks, lens=lens, failed=failed, stats=_struct_dict(st))


def ss_decode_microbatch_static(w: Weights, prompt_tokens, prompt_offsets, max_new: int, target_lens, flags: int = 0,
                                stream: Optional[int] = None) -> dict:
    return ss_decode_microbatch(w, prompt_tokens, prompt_offsets, max_new, target_lens, flags, stream, static=True)


def ss_forward_logits(w: Weights, tokens, offsets, n_prompt, all_prompt_logits: bool = False,
                      stream: Optional[int] = None) -> np.ndarray:
    tk, of, npz = _i32(tokens), _i32(offsets), _i32(n_prompt)
    B = len(npz)
    lens = np.diff(of)
    rows = int(lens.sum()) if all_prompt_logits else int((lens - npz + 1).sum())
    out = np.empty((rows, w.shape.vocab), np.float32)
    _check(lib().ss_forward_logits(w.h, _ptr(tk), _ptr(of), B, _ptr(npz), int(all_prompt_logits), _ptr(out), stream))
    return out


def ss_run_group(w: Weights, prompt_tokens, prompt_offsets, target_lens, pred_lens, bin: int, policy: ss_policy,
                 stream: Optional[int] = None) -> dict:
    pt, po, tl = _i32(prompt_tokens), _i32(prompt_offsets), _i32(target_lens)
    pl = None if pred_lens is None else _i32(pred_lens)
    n = len(tl)
    toks = np.empty((n, policy.base_len), np.int32)
    lens = np.zeros(n, np.int32)
    gs = ss_group_stats()
    _check(lib().ss_run_group(w.h, _ptr(pt), _ptr(po), n, _ptr(tl), _ptr(pl), bin, C.byref(policy), _ptr(toks),
                              _ptr(lens), C.byref(gs), stream))
    return dict(tokens=toks, lens=lens, stats=_struct_dict(gs))


def _gen_opts(eos_id: int, temperature: float, draws, target_lens, sync_every: int, seed: int = 0, draw_ids=None):
    """Marshals ss_gen_opts; returns (struct, arrays to keep alive)."""
    d = None if draws is None else np.ascontiguousarray(draws, dtype=np.float32)
    tl = None if target_lens is None else _i32(target_lens)
    ids = None if draw_ids is None else _i32(draw_ids)
    o = ss_gen_opts()
    o.seed = int(seed)
    o.draw_ids = None if ids is None else ids.ctypes.data
    o.eos_id, o.temperature, o.sync_every = int(eos_id), float(temperature), int(sync_every)
    o.draws = None if d is None else d.ctypes.data
    o.draws_stride = 0 if d is None else int(d.shape[1])
    o.target_lens = None if tl is None else tl.ctypes.data
    return o, (d, tl, ids)


def ss_generate_microbatch(w: Weights, prompt_tokens, prompt_offsets, max_new: int, eos_id: int = -1,
                           temperature: float = 0.0, draws=None, target_lens=None, sync_every: int = 8,
                           flags: int = 0, seed: int = 0, draw_ids=None, stream: Optional[int] = None) -> dict:
    pt, po = _i32(prompt_tokens), _i32(prompt_offsets)
    B = len(po) - 1
    opts, keep = _gen_opts(eos_id, temperature, draws, target_lens, sync_every, seed, draw_ids)
    toks = np.empty((B, max_new), np.int32)
    lens = np.empty(B, np.int32)
    failed = np.empty(B, np.uint8)
    st = ss_stats()
    _check(lib().ss_generate_microbatch(w.h, _ptr(pt), _ptr(po), B, max_new, C.byref(opts), flags, _ptr(toks),
                                        _ptr(lens), _ptr(failed), C.byref(st), stream))
    del keep
    return dict(tokens=toks, lens=lens, failed=failed, stats=_struct_dict(st))


def ss_run_group_generate(w: Weights, prompt_tokens, prompt_offsets, pred_lens, bin: int, policy: ss_policy,
                          eos_id: int = -1, temperature: float = 0.0, draws=None, target_lens=None,
                          sync_every: int = 8, seed: int = 0, draw_ids=None, stream: Optional[int] = None) -> dict:
    pt, po = _i32(prompt_tokens), _i32(prompt_offsets)
    pl = None if pred_lens is None else _i32(pred_lens)
    n = len(po) - 1
    opts, keep = _gen_opts(eos_id, temperature, draws, target_lens, sync_every, seed, draw_ids)
    toks = np.empty((n, policy.base_len), np.int32)
    lens = np.zeros(n, np.int32)
    gs = ss_group_stats()
    _check(lib().ss_run_group_generate(w.h, _ptr(pt), _ptr(po), n, _ptr(pl), bin, C.byref(policy), C.byref(opts),
                                       _ptr(toks), _ptr(lens), C.byref(gs), stream))
    del keep
    return dict(tokens=toks, lens=lens, stats=_struct_dict(gs))


def ss_bench_decode_step(w: Weights, prompt_tokens, B: int, ctx: int, iters: int,
                         stream: Optional[int] = None) -> np.ndarray:
    pt = _i32(prompt_tokens)
    assert pt.size == B * ctx
    ms = np.empty(iters, np.float64)
    _check(lib().ss_bench_decode_step(w.h, _ptr(pt), B, ctx, iters, _ptr(ms), stream))
    return ms


def ss_bench_decode_steps_in_flight(w: Weights, prompt_tokens, B: int, ctx: int, iters: int, lanes: int = 2) -> np.ndarray:
    """[lanes, iters] device milliseconds: the lanes' decode forwards running at the same time."""
    pt = _i32(prompt_tokens)
    assert pt.size == B * ctx
    ms = np.zeros(lanes * iters, np.float64)
    _check(lib().ss_bench_decode_steps_in_flight(w.h, _ptr(pt), B, ctx, iters, lanes, _ptr(ms)))
    return ms.reshape(lanes, iters)


def ss_bench_weight_stream(w: Weights, B: int, iters: int, stream: Optional[int] = None):
    ms = np.empty(iters, np.float64)
    launches = C.c_int32(0)
    _check(lib().ss_bench_weight_stream(w.h, B, iters, _ptr(ms), C.byref(launches), stream))
    return ms, int(launches.value)


def ss_bench_read_stream(w: Weights, iters: int, stream: Optional[int] = None):
    ms = np.empty(iters, np.float64)
    nbytes = C.c_int64(0)
    _check(lib().ss_bench_read_stream(w.h, iters, _ptr(ms), C.byref(nbytes), stream))
    return ms, int(nbytes.value)
