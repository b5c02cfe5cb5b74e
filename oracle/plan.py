"""Integer oracle of the single-pack planner (test infrastructure only).

Follows the paper where it speaks and a stated reading where it does not:

* Packing (Section 4.2 step 1, Algorithm 2): the paper allows any packer; the reading taken
  is an in-order greedy fill of ONE pack, the last sample truncated to the space left.
* Attention complexity of a pack (Section 3.1 worked example; Algorithm 7): a = sum len(x)^2.
* Attention Balance Sort (Algorithm 7) applied one level down: the units are (sample, tile)
  work items, their complexity is the exact number of causal (query, key) pairs they hold,
  and they are sorted longest first; ties fall back to (sample, tile) so the order is total.
* ABR (Section 3.1, ABR equation): sum(A_max - A_i) / (A_max * N).

Everything is Python integers; no code is shared with the C++ planner.
"""
from __future__ import annotations

from typing import List, Sequence, Tuple


def pack_cost(lengths: Sequence[int]) -> int:
    """Attention complexity of a pack: the sum of squared sample lengths."""
    return sum(int(s) * int(s) for s in lengths)


def balance_ratio(costs: Sequence[float]) -> float:
    """ABR over N units: sum(A_max - A_i) / (A_max * N)."""
    a_max = max(costs)
    return sum(a_max - a for a in costs) / (a_max * len(costs))


def pack_plan(lengths: Sequence[int], pack_len: int, tile_rows: int, kind: int):
    """Return (cu_seqlens, n_consumed, tiles, tile_cost, pack_cost).

    tiles: list of (sample, tile, row_begin, row_end) with rows absolute in the packed buffer.
    kind 0: query tiles, cost = number of pairs whose query row is in the tile.
    kind 1: key tiles,   cost = number of pairs whose key row is in the tile.
    """
    if pack_len <= 0 or tile_rows <= 0 or kind not in (0, 1):
        raise ValueError("bad argument")
    # a sample has at least one token: a length <= 0 anywhere in the list is an error, also behind the
    # point where the pack is already full (the paper is silent; the list as a whole is the input)
    if any(int(s) <= 0 for s in lengths):
        raise ValueError("non-positive length")
    taken: List[int] = []
    filled = 0
    consumed = 0
    for s in lengths:
        if filled == pack_len:
            break
        take = min(int(s), pack_len - filled)
        taken.append(take)
        filled += take
        consumed += 1
    cu = [0]
    for s in taken:
        cu.append(cu[-1] + s)
    items: List[Tuple[int, int, int, int, int]] = []
    for i, s in enumerate(taken):
        t = 0
        while t * tile_rows < s:
            lo = t * tile_rows
            hi = min(lo + tile_rows, s)
            if kind == 0:
                cost = sum(p + 1 for p in range(lo, hi))          # row p sees keys 0..p
            else:
                cost = sum(s - kk for kk in range(lo, hi))        # key kk is seen by rows kk..s-1
            items.append((cost, i, t, cu[i] + lo, cu[i] + hi))
            t += 1
    items.sort(key=lambda it: (-it[0], it[1], it[2]))
    tiles = [(i, t, b, e) for (_, i, t, b, e) in items]
    costs = [c for (c, _, _, _, _) in items]
    return cu, consumed, tiles, costs, pack_cost(taken)
