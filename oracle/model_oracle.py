"""ctypes front end of the C oracle in ``om_model.c`` (TEST INFRASTRUCTURE ONLY).

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this.
It takes plain numpy arrays (weights as bf16 bit patterns in uint16) and knows
nothing about the HIP library.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

import numpy as np

from . import build as _build


class _Cfg(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_heads", C.c_int32), ("head_dim", C.c_int32),
                ("d_ffn", C.c_int32), ("vocab", C.c_int32), ("rope_base", C.c_float), ("rms_eps", C.c_float)]


_LIBS = {}


def _lib(kind: str):
    if kind not in _LIBS:
        path = _build.lib_path(kind)
        if not os.path.exists(path):
            _build.build(force=False)
        L = C.CDLL(path)
        L.om_model_create.restype = C.c_void_p
        L.om_model_create.argtypes = [C.POINTER(_Cfg), C.POINTER(C.c_void_p)]
        L.om_model_free.argtypes = [C.c_void_p]
        L.om_seq_create.restype = C.c_void_p
        L.om_seq_create.argtypes = [C.c_void_p, C.c_int]
        L.om_seq_free.argtypes = [C.c_void_p]
        L.om_seq_reset.argtypes = [C.c_void_p]
        L.om_forward_rows.restype = C.c_int
        L.om_forward_rows.argtypes = [C.c_void_p, C.POINTER(C.c_void_p), C.c_int, C.c_void_p, C.c_void_p, C.c_void_p,
                                      C.c_void_p, C.c_void_p]
        L.om_greedy_microbatch.restype = C.c_int
        L.om_greedy_microbatch.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_void_p,
                                           C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.om_real_size.restype = C.c_int
        L.om_c_rmsnorm.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_float, C.c_void_p]
        L.om_c_matvec.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_void_p]
        L.om_c_rope.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_float]
        L.om_c_attention.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p]
        L.om_c_argmax.restype = C.c_int
        L.om_c_argmax.argtypes = [C.c_void_p, C.c_int, C.POINTER(C.c_double)]
        _LIBS[kind] = L
    return _LIBS[kind]


def _p(a: np.ndarray):
    return a.ctypes.data_as(C.c_void_p)


class Components:
    """The oracle's building blocks, one call each, for pinning."""

    def __init__(self, kind: str = "f64"):
        self.L = _lib(kind)
        self.real = np.float64 if self.L.om_real_size() == 8 else np.float32
        if kind == "f64":
            self.L.om_c_silu.restype = C.c_double
            self.L.om_c_silu.argtypes = [C.c_double]
        else:
            self.L.om_c_silu.restype = C.c_float
            self.L.om_c_silu.argtypes = [C.c_float]

    def rmsnorm(self, x, w_bits, eps):
        x = np.ascontiguousarray(x, self.real)
        w = np.ascontiguousarray(w_bits, np.uint16)
        out = np.empty_like(x)
        self.L.om_c_rmsnorm(_p(x), _p(w), x.size, eps, _p(out))
        return out

    def matvec(self, x, w_bits):
        x = np.ascontiguousarray(x, self.real)
        w = np.ascontiguousarray(w_bits, np.uint16)
        out = np.empty(w.shape[0], self.real)
        self.L.om_c_matvec(_p(x), _p(w), w.shape[0], w.shape[1], _p(out))
        return out

    def rope(self, v, pos, base=1.0e4):
        v = np.array(v, self.real, copy=True)
        self.L.om_c_rope(_p(v), v.size, int(pos), base)
        return v

    def attention(self, q, K, V):
        q = np.ascontiguousarray(q, self.real)
        K = np.ascontiguousarray(K, self.real)
        V = np.ascontiguousarray(V, self.real)
        out = np.empty_like(q)
        self.L.om_c_attention(_p(q), _p(K), _p(V), K.shape[0], q.size, K.shape[1], _p(out))
        return out

    def silu(self, z: float) -> float:
        return float(self.L.om_c_silu(z))

    def argmax(self, logits):
        lg = np.ascontiguousarray(logits, self.real)
        mg = C.c_double(0.0)
        i = self.L.om_c_argmax(_p(lg), lg.size, C.byref(mg))
        return int(i), float(mg.value)


class OracleModel:
    """A model over borrowed bf16 tensors (list in the generator's fixed order)."""

    def __init__(self, shape, tensors: Sequence[np.ndarray], kind: str = "f64"):
        self.L = _lib(kind)
        self.shape = shape
        self.kind = kind
        self._tensors = [np.ascontiguousarray(t, np.uint16) for t in tensors]   # keep alive
        assert len(self._tensors) == len(shape.tensor_specs())
        for t, (_, shp) in zip(self._tensors, shape.tensor_specs()):
            assert tuple(t.shape) == tuple(shp)
        cfg = _Cfg(shape.n_layers, shape.d_model, shape.n_heads, shape.head_dim, shape.d_ffn, shape.vocab,
                   shape.rope_base, shape.rms_eps)
        arr = (C.c_void_p * len(self._tensors))(*[t.ctypes.data for t in self._tensors])
        self.h = self.L.om_model_create(C.byref(cfg), arr)
        if not self.h:
            raise ValueError("om_model_create rejected the configuration")

    def __del__(self):
        try:
            if getattr(self, "h", None):
                self.L.om_model_free(self.h)
                self.h = None
        except Exception:
            pass

    # -- raw token-row forward -------------------------------------------------------
    def new_seq(self, cap: int) -> int:
        return self.L.om_seq_create(self.h, cap)

    def free_seq(self, s: int) -> None:
        self.L.om_seq_free(s)

    def forward_rows(self, seqs: List[int], seq_of, tok, pos, want=None) -> np.ndarray:
        seq_of = np.ascontiguousarray(seq_of, np.int32)
        tok = np.ascontiguousarray(tok, np.int32)
        pos = np.ascontiguousarray(pos, np.int32)
        n = len(tok)
        want_a = np.ones(n, np.uint8) if want is None else np.ascontiguousarray(want, np.uint8)
        out = np.empty((int(want_a.astype(bool).sum()), self.shape.vocab), np.float64)
        sarr = (C.c_void_p * len(seqs))(*seqs)
        rc = self.L.om_forward_rows(self.h, sarr, n, _p(seq_of), _p(tok), _p(pos), _p(want_a), _p(out))
        if rc != 0:
            raise ValueError("om_forward_rows: bad argument")
        return out

    # -- teacher-forced logits -------------------------------------------------------
    def teacher_forced(self, tokens, first: int = 0, incremental: bool = False) -> np.ndarray:
        """Logits [len(tokens)-first, V] at positions first.. of one sequence fed ``tokens``.

        incremental=False: one causal forward over all positions at once.
        incremental=True : positions < first in one forward, then one forward per position
                           (the key/value history is extended step by step).
        """
        tokens = np.ascontiguousarray(tokens, np.int32)
        T = len(tokens)
        s = self.new_seq(T)
        try:
            if not incremental:
                want = (np.arange(T) >= first).astype(np.uint8)
                return self.forward_rows([s], np.zeros(T, np.int32), tokens, np.arange(T, dtype=np.int32), want)
            outs = []
            if first > 0:
                self.forward_rows([s], np.zeros(first, np.int32), tokens[:first], np.arange(first, dtype=np.int32),
                                  np.zeros(first, np.uint8))
            for t in range(first, T):
                outs.append(self.forward_rows([s], [0], tokens[t:t + 1], [t]))
            return np.concatenate(outs, axis=0)
        finally:
            self.free_seq(s)

    # -- greedy micro-batch ----------------------------------------------------------
    def greedy_microbatch(self, prompt_tokens, prompt_offsets, max_new: int, target_lens, margins: bool = True):
        pt = np.ascontiguousarray(prompt_tokens, np.int32)
        po = np.ascontiguousarray(prompt_offsets, np.int32)
        tl = np.ascontiguousarray(target_lens, np.int32)
        B = len(tl)
        toks = np.empty((B, max_new), np.int32)
        lens = np.empty(B, np.int32)
        failed = np.empty(B, np.uint8)
        mg = np.empty((B, max_new), np.float64) if margins else None
        steps = C.c_int32(0)
        rc = self.L.om_greedy_microbatch(self.h, _p(pt), _p(po), B, int(max_new), _p(tl), _p(toks), _p(lens),
                                         _p(failed), _p(mg) if margins else None, C.byref(steps))
        if rc != 0:
            raise ValueError("om_greedy_microbatch: bad argument")
        return dict(tokens=toks, lens=lens, failed=failed, margins=mg, steps=int(steps.value))

    def greedy_query(self, prompt, t: int):
        """The plain definition of one query's output: its first t greedy tokens."""
        r = self.greedy_microbatch(prompt, [0, len(prompt)], t, [t])
        return r["tokens"][0], r["margins"][0]
