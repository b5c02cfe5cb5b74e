"""Oracle of the Hierarchical Groups Auto-Selection (test infrastructure only).

Plain Python, the paper's steps in the paper's order:

* GreedyProfileCkpt (appendix "Implementation Details of Hierarchical Groups Auto-Selection",
  GreedyProfileCkpt algorithm): profile the REMAINING memory with c_min and with c_max checkpointed
  layers, m_ave = (m2 - m1) / (c_max - c_min) per layer, c_o = c_max - m2 / m_ave.
* FindBestSpCkpt (same appendix, FindBestSpCkpt algorithm): for every SP degree take the layer count
  of GreedyProfileCkpt, profile the iteration time, return the argmin.
* Auto-Selection (Section 4.1, Algorithm 1): Stage 1 runs FindBestSpCkpt for every candidate length,
  j = argmin(P), (s_best, l_best) = (S[j], L[j]), (s_max, l_max) = (S[-1], L[-1]).  Stage 2:
  l_1 = floor(l_best / s_best.sp), l_2 = floor(l_max / s_max.sp); L_p = [l_1, l_best, l_2, l_max] if
  l_2 > l_best else [l_1, l_best, l_max].

Profiling is the caller's: `profile_memory(l, sp, ckpt)` returns the remaining memory (any unit;
negative: does not fit), `profile_time(l, sp, ckpt)` the iteration time (None or inf: cannot run).

Readings where the paper is silent (the same ones the C++ routine takes):
  - c_o is a layer count: the smallest integer c in [0, c_max] whose linearly extrapolated remaining
    memory m2 - m_ave (c_max - c) is >= 0, i.e. ceil(c_max - m2 / m_ave) clamped at 0 for m_ave > 0;
    for m_ave <= 0 (checkpointing frees nothing) 0 if the extrapolation at 0 fits, else infeasible.
    m2 < 0 (out of memory with c_max layers checkpointed): the (l, sp) pair is infeasible.
  - argmin takes the first minimum; infeasible entries count as +inf; a length with no feasible SP
    degree cannot win Stage 1; if the longest length has none, the selection fails.
  - L_p is reported without repeated lengths (the paper's own result for its tables is the two
    groups {16K, 128K}); a group derived by dividing by the SP degree (l_1, l_2) trains with SP = 1 and
    the checkpoint layers of the strategy it was derived from.
"""
from __future__ import annotations

import math
from typing import Callable, List, Optional, Sequence, Tuple


def greedy_profile_ckpt(l: int, sp: int, c_min: int, c_max: int, profile_memory: Callable) -> Optional[int]:
    if not (0 <= c_min < c_max):
        raise ValueError("need 0 <= c_min < c_max")
    m1 = profile_memory(l, sp, c_min)
    m2 = profile_memory(l, sp, c_max)
    if m2 < 0:
        return None
    m_ave = (m2 - m1) / (c_max - c_min)
    if m_ave > 0:
        c_o = c_max - m2 / m_ave
        return max(0, math.ceil(c_o))
    return 0 if m2 - m_ave * c_max >= 0 else None


def find_best_sp_ckpt(l: int, sp_set: Sequence[int], c_min: int, c_max: int, profile_memory: Callable,
                      profile_time: Callable) -> Optional[Tuple[int, int, float]]:
    p: List[float] = []
    o: List[Tuple[int, int]] = []
    for sp in sp_set:
        ckpt = greedy_profile_ckpt(l, sp, c_min, c_max, profile_memory)
        if ckpt is None:
            continue
        t = profile_time(l, sp, ckpt)
        if t is None or not (t < math.inf):
            continue
        p.append(t)
        o.append((sp, ckpt))
    if not p:
        return None
    j = p.index(min(p))
    return o[j][0], o[j][1], p[j]


def stage2(lengths: Sequence[int], strategies: Sequence[Optional[Tuple[int, int]]], times: Sequence[float]):
    """Stage 2 of Algorithm 1 from the per-length results of Stage 1.  Returns (groups, sp, ckpt, j)."""
    if strategies[-1] is None:
        raise ValueError("the longest length has no feasible strategy")
    finite = [t if strategies[i] is not None else math.inf for i, t in enumerate(times)]
    j = finite.index(min(finite))
    s_best, l_best = strategies[j], lengths[j]
    s_max, l_max = strategies[-1], lengths[-1]
    l_1 = l_best // s_best[0]
    l_2 = l_max // s_max[0]
    if l_2 > l_best:
        l_p = [(l_1, 1, s_best[1]), (l_best, s_best[0], s_best[1]), (l_2, 1, s_max[1]), (l_max, s_max[0], s_max[1])]
    else:
        l_p = [(l_1, 1, s_best[1]), (l_best, s_best[0], s_best[1]), (l_max, s_max[0], s_max[1])]
    out = []
    for g in l_p:  # a repeated length keeps its LAST entry (the length's own strategy)
        if out and out[-1][0] == g[0]:
            out[-1] = g
        else:
            out.append(g)
    return [g[0] for g in out], [g[1] for g in out], [g[2] for g in out], j


def auto_selection(lengths: Sequence[int], sp_set: Sequence[int], c_min: int, c_max: int,
                   profile_memory: Callable, profile_time: Callable):
    """Algorithm 1.  Returns {"groups", "sp", "ckpt", "j", "strategies": [(sp, ckpt) or None], "times"}."""
    if not lengths or not sp_set:
        raise ValueError("empty candidate set")
    if any(b <= a for a, b in zip(lengths, lengths[1:])) or lengths[0] <= 0:
        raise ValueError("lengths must be positive and strictly increasing")
    if any(sp <= 0 for sp in sp_set):
        raise ValueError("bad SP degree")
    strategies, times = [], []
    for l in lengths:
        best = find_best_sp_ckpt(l, sp_set, c_min, c_max, profile_memory, profile_time)
        strategies.append(None if best is None else (best[0], best[1]))
        times.append(math.inf if best is None else best[2])
    groups, sp, ckpt, j = stage2(lengths, strategies, times)
    return {"groups": groups, "sp": sp, "ckpt": ckpt, "j": j, "strategies": strategies, "times": times}
