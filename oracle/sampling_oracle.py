"""Oracle of generation with a real end-of-sequence token and temperature sampling
(TEST INFRASTRUCTURE ONLY: imported by tests, the smoke check and the benchmark's cpu_baseline leg).

Sec. 4.2 (Experimental Setting) of the paper: responses are sampled at a temperature and a
row stops when the model emits its end-of-sequence token or reaches the limit on new tokens;
Sec. 4.1: a row that is still unfinished when the micro-batch's limit is reached has failed.

Everything here is the plain definition, one query at a time, in fp64:

  p_v  = exp((logit_v - max logit) / T) / sum_v' exp(...)          softmax at temperature T
  token = smallest v with  p_0 + ... + p_v  >  u                    inverse CDF in vocabulary order,
          u in [0,1) being the draw supplied for (query, token number); V-1 if rounding leaves none
  T = 0 : greedy, largest logit, lowest index on exact ties

A query's output is the sequence obtained by feeding each chosen token back, ended by the first
end-of-sequence token (which is emitted and counted), by an optional forced length, or by the cap.
The draws are inputs, so the output depends on nothing but (weights, prompt, draws): not on the
micro-batch a query ran in, on compaction, on how often the host polled, or on a recomputation.

The draws may also come from a counter-based generator, so that a caller needs no table: Philox4x32-10
(Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as 1, 2, 3", SC 2011, Sec. 3.3 and Table 2 for
the round function and its constants) on the counter (token number, row id, 0, 0) under a 64-bit key; the
draw is the top 24 bits of the first output word times 2^-24.  Written here from that definition with Python
integers; pinned to the published known-answer vectors.

Pins: tests/test_oracle_sampling_pins.py.
"""
from __future__ import annotations

from typing import Optional, Sequence

import numpy as np


def token_probabilities(logits, temperature: float) -> np.ndarray:
    """softmax(logits / T) written out (fp64, max-subtracted)."""
    l = np.asarray(logits, np.float64)
    if not temperature > 0:
        raise ValueError("temperature must be > 0 here")
    e = np.exp((l - l.max()) / float(temperature))
    return e / e.sum()


def sample_token(logits, temperature: float, u: float):
    """One draw.  Returns (token, margin).

    margin: for T > 0 the distance, in probability, from u to the nearer edge of the chosen
    token's CDF interval; for T = 0 the top-1 minus top-2 logit.  A small margin marks a decision
    that a differently rounded evaluation may legitimately take the other way.
    """
    l = np.asarray(logits, np.float64)
    V = l.shape[0]
    if temperature == 0:
        best = int(np.flatnonzero(l == l.max())[0])          # lowest index on ties
        rest = np.delete(l, best)
        return best, float(l[best] - rest.max()) if V > 1 else float("inf")
    p = token_probabilities(l, temperature)
    cdf = 0.0
    for v in range(V):                                        # vocabulary order
        lo = cdf
        cdf = cdf + p[v]
        if cdf > u:
            return v, float(min(u - lo, cdf - u))
    return V - 1, 0.0


def generate_query(model, prompt: Sequence[int], cap: int, eos_id: int, temperature: float,
                   draws: Optional[Sequence[float]], target_len: Optional[int] = None):
    """One query, batch 1, its own key/value history.

    model        an OracleModel (decoder forward in fp64)
    cap          limit on generated tokens (the token chosen from the prompt's last position is number 0)
    eos_id       end-of-sequence id, or -1 for none
    draws        draws[s] for token number s (unused when temperature == 0)
    target_len   optional forced length (simulated end of sequence), combined with eos_id: whichever comes first
    Returns dict(tokens int32[len], margins float64[len], length, failed).
    failed: the row was still unfinished after `cap` tokens.
    """
    prompt = np.asarray(prompt, np.int32)
    P = len(prompt)
    if P < 1 or cap < 1:
        raise ValueError("empty prompt or cap < 1")
    seq = model.new_seq(P + cap)
    toks, margins = [], []
    finished = False
    try:
        lg = model.forward_rows([seq], np.zeros(P, np.int32), prompt, np.arange(P, dtype=np.int32),
                                (np.arange(P) == P - 1).astype(np.uint8))[0]
        for s in range(cap):
            u = 0.0 if temperature == 0 else float(draws[s])
            t, mg = sample_token(lg, temperature, u)
            toks.append(t)
            margins.append(mg)
            if t == eos_id or (target_len is not None and s + 1 >= target_len):
                finished = True
                break
            if s + 1 == cap:
                break
            lg = model.forward_rows([seq], [0], [t], [P + s])[0]
    finally:
        model.free_seq(seq)
    return dict(tokens=np.asarray(toks, np.int32), margins=np.asarray(margins, np.float64), length=len(toks),
                failed=not finished)


def next_token_on_prefix(model, prompt, emitted, temperature: float, u: float):
    """(token, margin) the definition yields after `prompt` followed by the tokens in `emitted`."""
    seq_toks = np.concatenate([np.asarray(prompt, np.int32), np.asarray(emitted, np.int32)])
    lg = model.teacher_forced(seq_toks, first=len(seq_toks) - 1)[0]
    return sample_token(lg, temperature, u)


# --------------------------------------------------------------------------- counter-based draws
_PHILOX_M = (0xD2511F53, 0xCD9E8D57)     # round multipliers
_PHILOX_W = (0x9E3779B9, 0xBB67AE85)     # key schedule increments (golden ratio, sqrt(3) - 1)
_MASK = 0xFFFFFFFF


def philox4x32_10(counter, key):
    """Ten rounds of the Philox 4x32 bijection: four 32-bit counter words, two key words -> four words."""
    c = [int(x) & _MASK for x in counter]
    k = [int(x) & _MASK for x in key]
    for _ in range(10):
        p0 = _PHILOX_M[0] * c[0]
        p1 = _PHILOX_M[1] * c[2]
        c = [(p1 >> 32) ^ c[1] ^ k[0], p1 & _MASK, (p0 >> 32) ^ c[3] ^ k[1], p0 & _MASK]
        k = [(k[0] + _PHILOX_W[0]) & _MASK, (k[1] + _PHILOX_W[1]) & _MASK]
    return tuple(c)


def generated_draw(seed: int, row_id: int, token_number: int) -> np.float32:
    """The draw in [0,1) for token `token_number` of the row with id `row_id` under the 64-bit `seed`."""
    x0 = philox4x32_10((token_number, row_id, 0, 0), (seed & _MASK, (seed >> 32) & _MASK))[0]
    return np.float32((x0 >> 8) * 2.0 ** -24)


def generated_draws(seed: int, row_ids, n_tokens: int) -> np.ndarray:
    """Table float32 [len(row_ids), n_tokens] of generated_draw."""
    return np.array([[generated_draw(seed, int(q), s) for s in range(n_tokens)] for q in row_ids], np.float32)
