"""Seeded synthetic inputs: model shapes, weights, query groups.

This module only *draws inputs*.  It contains none of the method's arithmetic
(no scheduling, no model math) and is the single source of inputs for both the
CPU oracle and the HIP path, which otherwise share nothing.

The paper evaluates on an instruction-following prompt set and a collected
real-world prompt set with a fine-tuned 7B chat model (Sec. 4.2, Experimental
Setting); neither the prompts nor the weights are available offline, so the
groups below imitate their *shape* only: short prompts, wide long-tailed
response lengths with a hard cut (Fig. 2a), random-init weights of the same
architecture.

All draws come from ``numpy.random.Generator(PCG64)`` streams spawned from one
``SeedSequence`` per object, so every value is a pure function of the seed.
"""
from __future__ import annotations

import dataclasses
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass
from typing import Dict, List, Optional, Tuple

import numpy as np


# --------------------------------------------------------------------------- shapes
@dataclass(frozen=True)
class ModelShape:
    name: str
    n_layers: int
    d_model: int
    n_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    rope_base: float = 1.0e4
    rms_eps: float = 1.0e-6

    def with_layers(self, n_layers: int) -> "ModelShape":
        return dataclasses.replace(self, n_layers=n_layers, name=f"{self.name}-L{n_layers}")

    def tensor_specs(self) -> List[Tuple[str, Tuple[int, ...]]]:
        """Fixed tensor order shared by every consumer; matrices are [out, in] row-major."""
        d, f, v = self.d_model, self.d_ffn, self.vocab
        specs: List[Tuple[str, Tuple[int, ...]]] = [("embed", (v, d))]
        for l in range(self.n_layers):
            specs += [
                (f"l{l}.attn_norm", (d,)),
                (f"l{l}.wq", (d, d)),
                (f"l{l}.wk", (d, d)),
                (f"l{l}.wv", (d, d)),
                (f"l{l}.wo", (d, d)),
                (f"l{l}.mlp_norm", (d,)),
                (f"l{l}.wg", (f, d)),
                (f"l{l}.wu", (f, d)),
                (f"l{l}.wd", (d, f)),
            ]
        specs += [("final_norm", (d,)), ("lm_head", (v, d))]
        return specs

    def weight_bytes_per_step(self) -> int:
        """bf16 bytes of every matmul weight and norm vector (embedding table excluded)."""
        d, f, v = self.d_model, self.d_ffn, self.vocab
        per_layer = (4 * d * d + 3 * d * f + 2 * d) * 2
        return self.n_layers * per_layer + (v * d + d) * 2

    def kv_bytes_per_token(self) -> int:
        return 2 * self.n_layers * self.d_model * 2


TINY = ModelShape("tiny", 2, 256, 4, 64, 688, 1024)
LLAMA7B = ModelShape("llama7b", 32, 4096, 32, 128, 11008, 32000)
LLAMA13B = ModelShape("llama13b", 40, 5120, 40, 128, 13824, 32000)


# --------------------------------------------------------------------------- bf16
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------- weights
def make_weights(shape: ModelShape, seed: int, std: float = 0.02, norm_jitter: float = 0.0,
                 threads: int = 8) -> List[np.ndarray]:
    """bf16 (uint16 bit patterns) tensors in ``shape.tensor_specs()`` order.

    Matrices ~ N(0, std) rounded to bf16.  Norm vectors are 1, or 1 + norm_jitter*N(0,1)
    when ``norm_jitter`` > 0 (tests use that so a dropped norm weight is visible).
    """
    specs = shape.tensor_specs()
    children = np.random.SeedSequence(seed).spawn(len(specs))

    def one(i: int) -> np.ndarray:
        name, shp = specs[i]
        rng = np.random.Generator(np.random.PCG64(children[i]))
        if len(shp) == 1:
            w = np.ones(shp, dtype=np.float32)
            if norm_jitter > 0.0:
                w += np.float32(norm_jitter) * rng.standard_normal(shp, dtype=np.float32)
            return f32_to_bf16_bits(w)
        out = np.empty(shp, dtype=np.uint16)
        rows = shp[0]
        step = max(1, (1 << 24) // shp[1])          # ~16M values per slab keeps temporaries small
        for r0 in range(0, rows, step):
            r1 = min(rows, r0 + step)
            blk = rng.standard_normal((r1 - r0, shp[1]), dtype=np.float32)
            blk *= np.float32(std)
            out[r0:r1] = f32_to_bf16_bits(blk)
        return out

    if threads <= 1:
        return [one(i) for i in range(len(specs))]
    with ThreadPoolExecutor(max_workers=threads) as ex:
        return list(ex.map(one, range(len(specs))))


# --------------------------------------------------------------------------- groups
@dataclass
class Workload:
    """One group of queries.  ``pred_lens`` is None for vanilla batching."""
    name: str
    shape: ModelShape
    weight_seed: int
    n: int
    prompt_offsets: np.ndarray      # int32 [n+1]
    prompt_tokens: np.ndarray       # int32 [sum p_i]
    target_lens: np.ndarray         # int32 [n]   forced response length t_i (EOS simulated there)
    pred_lens: Optional[np.ndarray]  # int32 [n]   predicted length, or None
    l_max: int                      # global cap on generated tokens
    bin_width: int                  # 0 = no binning
    base_batch: int
    max_batch: int
    flags: Tuple[str, ...]          # subset of SORT, BIN, FCR, VBS, COMPACT

    @property
    def prompt_lens(self) -> np.ndarray:
        return np.diff(self.prompt_offsets).astype(np.int32)

    def prompt(self, i: int) -> np.ndarray:
        return self.prompt_tokens[self.prompt_offsets[i]:self.prompt_offsets[i + 1]]


def _lognormal_lens(rng: np.random.Generator, n: int, median: float, sigma: float, lo: int, hi: int) -> np.ndarray:
    z = rng.standard_normal(n)
    return np.clip(np.rint(median * np.exp(sigma * z)), lo, hi).astype(np.int32)


_CONFIGS: Dict[int, dict] = {
    1: dict(shape=TINY, weight_seed=1, group_seed=20230514, n=16, prompt=("uniform", 8, 32),
            resp=("uniform", 1, 48), noise=None, l_max=48, bin=0, flags=()),
    2: dict(shape=LLAMA7B, weight_seed=2, group_seed=20230515, n=256, prompt=("lognormal", 40.0, 0.6, 8, 256),
            resp=("lognormal", 120.0, 0.7, 1, 512), noise=None, l_max=512, bin=0, flags=()),
    3: dict(shape=LLAMA7B, weight_seed=2, group_seed=20230515, n=256, prompt=("lognormal", 40.0, 0.6, 8, 256),
            resp=("lognormal", 120.0, 0.7, 1, 512), noise=0.3, l_max=512, bin=50, flags=("SORT", "BIN", "FCR")),
    4: dict(shape=LLAMA7B, weight_seed=2, group_seed=20230517, n=1024, prompt=("lognormal", 40.0, 0.6, 8, 256),
            resp=("lognormal", 120.0, 0.7, 1, 512), noise=0.3, l_max=512, bin=50,
            flags=("SORT", "BIN", "FCR", "VBS", "COMPACT")),
    5: dict(shape=LLAMA13B, weight_seed=5, group_seed=20230518, n=1024, prompt=("lognormal", 60.0, 0.6, 8, 512),
            resp=("lognormal", 120.0, 0.9, 1, 1024), noise=0.3, l_max=1024, bin=64,
            flags=("SORT", "BIN", "FCR", "VBS", "COMPACT")),
}


def make_group(shape: ModelShape, n: int, seed: int, prompt: tuple, resp: tuple, noise: Optional[float],
               l_max: int, bin_width: int, flags: Tuple[str, ...], name: str = "custom", weight_seed: int = 0,
               base_batch: int = 16, max_batch: int = 256) -> Workload:
    """Draw one group.  Independent streams: prompt lengths, prompt ids, responses, prediction noise."""
    s_plen, s_ids, s_resp, s_noise = [np.random.Generator(np.random.PCG64(c))
                                      for c in np.random.SeedSequence(seed).spawn(4)]
    if prompt[0] == "uniform":
        plens = s_plen.integers(prompt[1], prompt[2] + 1, size=n).astype(np.int32)
    else:
        plens = _lognormal_lens(s_plen, n, *prompt[1:])
    if resp[0] == "uniform":
        tl = s_resp.integers(resp[1], resp[2] + 1, size=n).astype(np.int32)
    else:
        tl = _lognormal_lens(s_resp, n, *resp[1:])
    offs = np.zeros(n + 1, dtype=np.int32)
    np.cumsum(plens, out=offs[1:])
    toks = s_ids.integers(0, shape.vocab, size=int(offs[-1])).astype(np.int32)
    pred = None
    if noise is not None:
        z = s_noise.standard_normal(n)
        pred = np.maximum(1, np.rint(tl * np.exp(noise * z))).astype(np.int32)
    return Workload(name=name, shape=shape, weight_seed=weight_seed, n=n, prompt_offsets=offs, prompt_tokens=toks,
                    target_lens=tl, pred_lens=pred, l_max=l_max, bin_width=bin_width, base_batch=base_batch,
                    max_batch=max_batch, flags=tuple(flags))


def make_workload(cfg: int, n: Optional[int] = None, shape: Optional[ModelShape] = None) -> Workload:
    """One of the five named configurations (optionally with fewer queries or a reduced-depth shape)."""
    c = _CONFIGS[cfg]
    return make_group(shape or c["shape"], n or c["n"], c["group_seed"], c["prompt"], c["resp"], c["noise"],
                      c["l_max"], c["bin"], c["flags"], name=f"cfg{cfg}", weight_seed=c["weight_seed"])


def gather_prompts(w: Workload, idx) -> Tuple[np.ndarray, np.ndarray]:
    """Ragged concat of the prompts of the queries in ``idx`` -> (tokens, offsets[len(idx)+1])."""
    idx = np.asarray(idx, dtype=np.int64)
    lens = w.prompt_lens[idx]
    offs = np.zeros(len(idx) + 1, dtype=np.int32)
    np.cumsum(lens, out=offs[1:])
    toks = np.concatenate([w.prompt(int(i)) for i in idx]) if len(idx) else np.zeros(0, np.int32)
    return toks.astype(np.int32), offs


def make_draws(n: int, l_max: int, seed: int) -> np.ndarray:
    """Uniform draws in [0,1) for (query, token number), float32 [n, l_max]: the random numbers a
    sampled generation consumes, supplied as an input to both the library and the oracle."""
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, 0x5A17])))
    return rng.random((n, l_max), dtype=np.float32)


def make_predictions_max_of(target_lens: np.ndarray, sigma: float, k: int, seed: int) -> np.ndarray:
    """Predictions of a predictor trained on the largest of k noisy observations of each length (the paper's
    Sec. 4.2 builds its training target as the maximum over several generations, which biases predictions
    upward and trades padding for fewer failures): max(1, rint(t * exp(sigma * max_k z))), z ~ N(0,1)."""
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, 0xB1A5])))
    z = rng.standard_normal((len(target_lens), k)).max(axis=1)
    return np.maximum(1, np.rint(np.asarray(target_lens) * np.exp(sigma * z))).astype(np.int32)
