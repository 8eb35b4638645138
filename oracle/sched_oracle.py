"""Scheduler and accounting oracle (TEST INFRASTRUCTURE ONLY): plain Python integers.

Follows Sec. 4.1 of the paper step by step:
  * sort the group by predicted length and split it into batches (Method, 3rd paragraph);
  * binning with a fixed cell size, rounding a length up to the bin that covers it
    (Binning paragraph; cell size 50 in Sec. 4.2);
  * FCR: the cap on newly generated tokens of a batch is the largest predicted length
    in it; rows that need more are failures, collected and recomputed after the group;
  * VBS: keep the number of tokens per batch constant, so the batch size is inversely
    proportional to the length (the printed fraction B0*L/L0 grows with L and contradicts
    the sentence before it and the 256*50/L of Sec. 4.2; it is read as B0*L0/L).
Readings of points the paper leaves open are listed next to each function.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

FLAGS = ("SORT", "BIN", "FCR", "VBS", "COMPACT")


def ceil_div(a: int, b: int) -> int:
    return -(-a // b)


def bin_upper(pred: int, w: int, l_max: int) -> int:
    """Upper edge of the bin holding ``pred`` (inclusive edge: 50 -> 50, 51 -> 100), never above
    the bin that holds l_max."""
    return min(w * ceil_div(pred, w), w * ceil_div(l_max, w))


def vbs_clamp_floor(length: int, base_batch: int, l_max: int, max_batch: int) -> int:
    """Constant tokens per batch: floor(B0 * L_max / L), kept within [B0, max_batch]."""
    return max(base_batch, min(max_batch, (base_batch * l_max) // length))


def vbs_paper_pow2(length: int) -> int:
    """Sec. 4.2: 16 for L >= 300, else 256*50/L rounded to the nearest power of two
    (nearest in linear distance, the lower one on a tie)."""
    if length >= 300:
        return 16
    x = 256.0 * 50.0 / float(length)
    lo = 1
    while lo * 2 <= x:
        lo *= 2
    hi = lo * 2
    return lo if (x - lo) <= (hi - x) else hi


@dataclass
class Policy:
    flags: Tuple[str, ...] = ()
    base_batch: int = 16
    l_max: int = 512
    max_batch: int = 256
    vbs_rule: str = "clamp_floor"      # or "paper_pow2"

    def has(self, f: str) -> bool:
        return f in self.flags

    def batch_for(self, length: int) -> int:
        if not self.has("VBS"):
            return self.base_batch
        if self.vbs_rule == "paper_pow2":
            return vbs_paper_pow2(length)
        return vbs_clamp_floor(length, self.base_batch, self.l_max, self.max_batch)


@dataclass
class MicroBatch:
    idx: List[int]
    cap: int


def _keys(pred: Sequence[int], w: int, pol: Policy) -> List[int]:
    """The length each query is scheduled by: its bin's upper edge, or its raw prediction."""
    if pol.has("BIN") and w > 0:
        return [bin_upper(int(p), w, pol.l_max) for p in pred]
    return [int(p) for p in pred]


def _chunk(order: List[int], key: List[int], pol: Policy, binned: bool, fcr: bool) -> List[MicroBatch]:
    out: List[MicroBatch] = []
    if binned:
        # every bin is chunked on its own; only its last chunk may be short; no merging across bins
        s = 0
        while s < len(order):
            e = s
            while e < len(order) and key[order[e]] == key[order[s]]:
                e += 1
            ub = key[order[s]]
            bsz = pol.batch_for(ub)
            for c in range(s, e, bsz):
                out.append(MicroBatch(order[c:min(e, c + bsz)], min(ub, pol.l_max) if fcr else pol.l_max))
            s = e
        return out
    s = 0
    while s < len(order):
        if pol.has("VBS"):
            # grow the chunk while its size still fits the batch size allowed for its longest prediction
            e = s + 1
            while e < len(order) and (e - s + 1) <= pol.batch_for(key[order[e]]):
                e += 1
        else:
            e = min(len(order), s + pol.base_batch)
        rows = order[s:e]
        cap = min(max(key[i] for i in rows), pol.l_max) if fcr else pol.l_max
        out.append(MicroBatch(rows, cap))
        s = e
    return out


def schedule(pred: Optional[Sequence[int]], n: int, w: int, pol: Policy) -> List[MicroBatch]:
    """First-pass plan.  pred None or no SORT flag = vanilla: arrival order, chunks of B0, cap L_max."""
    if pred is None or not pol.has("SORT"):
        return [MicroBatch(list(range(s, min(n, s + pol.base_batch))), pol.l_max)
                for s in range(0, n, pol.base_batch)]
    key = _keys(pred, w, pol)
    order = sorted(range(n), key=lambda i: (key[i], i))
    return _chunk(order, key, pol, pol.has("BIN") and w > 0, pol.has("FCR"))


def schedule_failures(pred: Sequence[int], failed: Sequence[int], w: int, pol: Policy) -> List[MicroBatch]:
    """The recomputation pass after the group: failures ordered by (scheduled length, index),
    fixed batch B0, cap L_max so that nothing can fail twice."""
    key = _keys(pred, w, pol)
    order = sorted(failed, key=lambda i: (key[i], i))
    return [MicroBatch(order[s:s + pol.base_batch], pol.l_max) for s in range(0, len(order), pol.base_batch)]


@dataclass
class Account:
    n_mb: int = 0
    steps: int = 0                 # forwards (one prompt forward + steps-1 decode forwards per micro-batch)
    padded_row_steps: int = 0      # sum B * steps
    live_row_steps: int = 0        # sum_i min(t_i, cap)
    rows: int = 0                  # sum B
    failed: List[int] = field(default_factory=list)
    per_mb: List[Dict[str, int]] = field(default_factory=list)


def account(plan: List[MicroBatch], t: Sequence[int]) -> Account:
    a = Account()
    for mb in plan:
        steps = min(mb.cap, max(int(t[i]) for i in mb.idx))
        live = sum(min(int(t[i]), mb.cap) for i in mb.idx)
        a.n_mb += 1
        a.steps += steps
        a.padded_row_steps += len(mb.idx) * steps
        a.live_row_steps += live
        a.rows += len(mb.idx)
        a.failed += [i for i in mb.idx if int(t[i]) > mb.cap]
        a.per_mb.append(dict(B=len(mb.idx), cap=mb.cap, steps=steps, live=live))
    return a


def run_group(pred: Optional[Sequence[int]], t: Sequence[int], w: int, pol: Policy) -> Dict[str, object]:
    """Whole-group accounting: first pass, then the failure pass (Sec. 4.1 FCR; metrics of Sec. 4.2)."""
    n = len(t)
    p1 = schedule(pred, n, w, pol)
    a1 = account(p1, t)
    p2 = schedule_failures(pred, a1.failed, w, pol) if a1.failed else []
    a2 = account(p2, t)
    assert not a2.failed
    rows = a1.rows + a2.rows
    padded = a1.padded_row_steps + a2.padded_row_steps
    return dict(
        plan=p1, failure_plan=p2, first=a1, second=a2,
        useful_tokens=sum(int(x) for x in t),
        steps=a1.steps + a2.steps,
        padded_row_steps=padded,
        live_row_steps=a1.live_row_steps + a2.live_row_steps,
        n_failed=len(a1.failed),
        failure_ratio=len(a1.failed) / n,
        avg_len_weighted=padded / rows,
        avg_len_unweighted=(sum(m["steps"] for m in a1.per_mb + a2.per_mb) / (a1.n_mb + a2.n_mb)),
        redundancy=1.0 - (sum(int(x) for x in t) / padded),
    )
