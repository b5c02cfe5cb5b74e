"""Oracle of the Hierarchical Groups Auto-Selection (test infrastructure only).

Plain Python.  What each routine computes, as the paper defines it:

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
    """Fewest checkpointed layers that still fit, from a line through two memory probes.  Remaining memory
    is modelled as m(c) = m2 - m_ave (c_max - c); the answer is the smallest whole c >= 0 with m(c) >= 0."""
    if not (0 <= c_min < c_max):
        raise ValueError("need 0 <= c_min < c_max")
    m1, m2 = profile_memory(l, sp, c_min), profile_memory(l, sp, c_max)
    if m2 < 0:                                   # does not fit even with c_max layers checkpointed
        return None
    m_ave = (m2 - m1) / (c_max - c_min)          # memory freed per checkpointed layer
    if m_ave <= 0:                               # checkpointing frees nothing: all or nothing at c = 0
        return 0 if m2 - m_ave * c_max >= 0 else None
    return max(0, math.ceil(c_max - m2 / m_ave))  # zero crossing of the line, as a layer count


def find_best_sp_ckpt(l: int, sp_set: Sequence[int], c_min: int, c_max: int, profile_memory: Callable,
                      profile_time: Callable) -> Optional[Tuple[int, int, float]]:
    """argmin of the profiled iteration time over the feasible (sp, ckpt) pairs of length l, ckpt being
    GreedyProfileCkpt's layer count for that sp; the first of equal minima wins.  None: nothing fits."""
    feasible = []
    for position, sp in enumerate(sp_set):
        ckpt = greedy_profile_ckpt(l, sp, c_min, c_max, profile_memory)
        t = None if ckpt is None else profile_time(l, sp, ckpt)
        if t is not None and t < math.inf:
            feasible.append((t, position, sp, ckpt))
    if not feasible:
        return None
    t, _, sp, ckpt = min(feasible)
    return sp, ckpt, t


def stage2(lengths: Sequence[int], strategies: Sequence[Optional[Tuple[int, int]]], times: Sequence[float]):
    """Stage 2 of Algorithm 1 from the per-length results of Stage 1.  Returns (groups, sp, ckpt, j).

    The groups are the set {l_1, l_best, l_max}, plus l_2 when it lies above l_best, in ascending order,
    with l_1 = floor(l_best / sp_best) and l_2 = floor(l_max / sp_max).  l_best and l_max train with their
    own Stage 1 strategy; a derived length trains with SP 1 and the layer count of the strategy it comes
    from, unless it coincides with l_best or l_max."""
    if strategies[-1] is None:
        raise ValueError("the longest length has no feasible strategy")
    j = min((i for i in range(len(lengths)) if strategies[i] is not None), key=lambda i: (times[i], i))
    (sp_best, ckpt_best), l_best = strategies[j], lengths[j]
    (sp_max, ckpt_max), l_max = strategies[-1], lengths[-1]
    l_1, l_2 = l_best // sp_best, l_max // sp_max
    plan = {l_1: (1, ckpt_best)}
    if l_2 > l_best:
        plan[l_2] = (1, ckpt_max)
    plan[l_best] = (sp_best, ckpt_best)
    plan[l_max] = (sp_max, ckpt_max)
    groups = sorted(plan)
    return groups, [plan[l][0] for l in groups], [plan[l][1] for l in groups], j


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
