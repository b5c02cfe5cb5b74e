"""Oracle of the multi-level Balance Packing planner (test infrastructure only).

Plain Python integers and lists.  What each step computes, as the paper defines it:

* GroupData (Appendix "Implementation Details of Balance Packing", GroupData function):
  sample x goes to group D_i when len(x) lies in (l_{i-1}, l_i], l_0 = 0.
* Balance Packing (Section 4.2, Algorithm 2): for i = n down to 1:
  Packing(D_i, l_i), GreedyFill(G_i, l_i, [D_{i-1}, ..., D_1]), Balance Batching(G_i); the
  batches of all levels are shuffled at the end.
* GreedyFill (Appendix, GreedyFill function): for every pack g of G_i, for j = i-1 down to 1, for
  every x still in D_j (in order): if the pack's tokens + len(x) <= l_i, move x into the pack.
* Attention Balance Sort (Appendix, Attention Balance Sort function): a = sum len(x)^2 per pack,
  sort the packs by a, cut consecutive packs into mini-batches.
* Metrics (Section 3.1): DBR, PR, ABR, CR, Ave-T equations.

Readings where the paper is silent (the same ones the C++ planner takes):
  - Packing: "arbitrary packing methods are feasible" -> first-fit decreasing: samples by length
    descending (ties: input order), each into the first pack (in creation order) it fits.
  - Sort direction and ties: a descending, ties by pack creation order.
  - Mini-batches: `packs_per_batch[i]` consecutive packs of the sorted level; a short last batch
    is kept.
  - Shuffle: Fisher-Yates from the end, j = next() mod (k+1), next() = splitmix64 stream of the seed.
  - A sample longer than the largest group length, or of length <= 0, is an error.
  - Metrics are evaluated per batch (one pack = one device's input of an iteration) and averaged
    over the batches of full size; PR of a pack = (l_i - tokens) / l_i.

No code is shared with the C++ planner.
"""
from __future__ import annotations

from typing import Dict, List, Sequence

MASK64 = (1 << 64) - 1


def splitmix64_stream(seed: int):
    """The splitmix64 sequence (Steele, Lea, Flood 2014): state += golden gamma, then two xor-shift-multiplies."""
    state = seed & MASK64
    while True:
        state = (state + 0x9E3779B97F4A7C15) & MASK64
        z = state
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & MASK64
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & MASK64
        yield z ^ (z >> 31)


def group_data(lengths: Sequence[int], group_lens: Sequence[int]) -> List[List[int]]:
    """GroupData: D_i = samples (indices, input order) with length in (l_{i-1}, l_i]."""
    groups: List[List[int]] = [[] for _ in group_lens]
    for x, n in enumerate(lengths):
        if n <= 0:
            raise ValueError("non-positive length")
        placed = False
        lo = 0
        for i, hi in enumerate(group_lens):
            if lo < n <= hi:
                groups[i].append(x)
                placed = True
            lo = hi
        if not placed:
            raise ValueError("sample longer than the largest packing group")
    return groups


def packing_ffd(items: Sequence[int], lengths: Sequence[int], cap: int) -> List[List[int]]:
    """Packing(D_i, l_i), first-fit decreasing."""
    order = sorted(items, key=lambda x: (-lengths[x], x))
    packs: List[List[int]] = []
    used: List[int] = []
    for x in order:
        for p in range(len(packs)):
            if used[p] + lengths[x] <= cap:
                packs[p].append(x)
                used[p] += lengths[x]
                break
        else:
            packs.append([x])
            used.append(lengths[x])
    return packs


def take_what_fits(pool: List[int], room: int, lengths: Sequence[int]):
    """One pass over `pool` in its order with `room` tokens of space: a sample is taken when it fits the
    space that is left at the moment it is looked at.  Returns (taken, left over, space left)."""
    taken, left = [], []
    for x in pool:
        if lengths[x] <= room:
            taken.append(x)
            room -= lengths[x]
        else:
            left.append(x)
    return taken, left, room


def greedy_fill(packs: List[List[int]], cap: int, smaller: List[List[int]], lengths: Sequence[int]) -> None:
    """GreedyFill(G_i, l_i, [D_{i-1}, ..., D_1]): the residual space of every pack of level i is offered to
    the smaller groups, the nearest group first; the packs are served in creation order and a sample that
    went into a pack is gone from its group.  `smaller` is given nearest first and is edited in place."""
    for g in packs:
        room = cap - sum(lengths[s] for s in g)
        for level, pool in enumerate(smaller):
            taken, smaller[level][:], room = take_what_fits(pool, room, lengths)
            g.extend(taken)


def attention_complexity(pack: Sequence[int], lengths: Sequence[int]) -> int:
    """a = sum of len(x)^2 over the samples of a pack (Section 3.1; Attention Balance Sort)."""
    return sum(lengths[x] * lengths[x] for x in pack)


def attention_balance_sort(packs: List[List[int]], lengths: Sequence[int]) -> List[List[int]]:
    """The packs of one level ordered by attention complexity, largest first; equal ones keep their
    creation order (Python's sort is stable)."""
    return sorted(packs, key=lambda g: -attention_complexity(g, lengths))


def balance_packing(lengths: Sequence[int], group_lens: Sequence[int], packs_per_batch: Sequence[int],
                    shuffle_seed: int) -> List[Dict]:
    """Algorithm 2.  Returns the shuffled list of batches, each {"level": i (0-based), "packs": [[sample ids]]}."""
    n = len(group_lens)
    if n == 0 or len(packs_per_batch) != n:
        raise ValueError("bad argument")
    prev = 0
    for l in group_lens:
        if l <= prev:
            raise ValueError("group lengths must be positive and strictly increasing")
        prev = l
    if any(b <= 0 for b in packs_per_batch):
        raise ValueError("bad batch size")
    d = group_data(lengths, group_lens)
    batches: List[Dict] = []
    for i in range(n - 1, -1, -1):
        g = packing_ffd(d[i], lengths, group_lens[i])
        d[i] = []
        greedy_fill(g, group_lens[i], [d[j] for j in range(i - 1, -1, -1)], lengths)
        g = attention_balance_sort(g, lengths)
        b = packs_per_batch[i]
        for start in range(0, len(g), b):
            batches.append({"level": i, "packs": g[start:start + b]})
    rng = splitmix64_stream(shuffle_seed)
    for k in range(len(batches) - 1, 0, -1):
        j = next(rng) % (k + 1)
        batches[k], batches[j] = batches[j], batches[k]
    return batches


def ratio_to_max(values: Sequence[float]) -> float:
    """sum(v_max - v_i) / (v_max * N): the common form of the DBR, PR and ABR equations."""
    v_max = max(values)
    if v_max == 0:
        return 0.0
    return sum(v_max - v for v in values) / (v_max * len(values))


def metrics(batches: List[Dict], lengths: Sequence[int], group_lens: Sequence[int],
            packs_per_batch: Sequence[int], level_sp: Sequence[int]) -> Dict[str, float]:
    """DBR, PR, ABR (means over the full-size batches), CR and Ave-T (over all batches)."""
    dbr, abr, n_full = 0.0, 0.0, 0
    pad, cap, t_comm, t_all, devices = 0, 0, 0, 0, 0
    for b in batches:
        i = b["level"]
        tokens = [sum(lengths[x] for x in g) for g in b["packs"]]
        attn = [attention_complexity(g, lengths) for g in b["packs"]]
        if len(b["packs"]) == packs_per_batch[i]:
            dbr += ratio_to_max(tokens)
            abr += ratio_to_max(attn)
            n_full += 1
        pad += sum(group_lens[i] - t for t in tokens)
        cap += group_lens[i] * len(tokens)
        t_all += sum(tokens)
        devices += len(tokens)
        if level_sp[i] > 1:
            t_comm += sum(tokens)
    return {"DBR": dbr / n_full if n_full else 0.0, "ABR": abr / n_full if n_full else 0.0,
            "PR": pad / cap if cap else 0.0, "CR": t_comm / t_all if t_all else 0.0,
            "AveT": t_all / devices if devices else 0.0}
