"""Pins of the planner oracle: the paper's worked example, brute force, invariants."""
import os
import random

import pytest

from oracle import pack_plan, pack_cost, balance_ratio

GOLD = os.path.join(os.path.dirname(__file__), "golden", "paper_abr_example.txt")


def _read_golden():
    packs, abr = [], None
    for line in open(GOLD):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        a, b = [x.strip() for x in line.split(";")]
        if a == "ABR":
            abr = float(b)
        else:
            packs.append(([int(x) for x in a.split(",")], int(b)))
    return packs, abr


def test_paper_worked_example_cost_and_abr():
    # Section 3.1: {1K x4} -> 4K^2, {2K x2} -> 8K^2, ABR = 0.25
    packs, abr = _read_golden()
    K2 = 1024 * 1024
    costs = []
    for lengths, units in packs:
        assert pack_cost(lengths) == units * K2
        cu, consumed, tiles, tcost, pc = pack_plan(lengths, 4096, 128, 0)
        assert pc == units * K2 and cu[-1] == 4096 and consumed == len(lengths)
        costs.append(pc)
    assert balance_ratio(costs) == pytest.approx(abr, abs=0)


def test_tiny_pack_cu_seqlens():
    cu, consumed, tiles, cost, pc = pack_plan([512, 256, 128, 64, 64], 1024, 128, 0)
    assert cu == [0, 512, 768, 896, 960, 1024]
    assert consumed == 5
    assert pc == 512**2 + 256**2 + 128**2 + 2 * 64**2
    # 4 + 2 + 1 + 1 + 1 tiles
    assert len(tiles) == 9
    # the most expensive query tile is the last tile of the longest sample
    assert tiles[0] == (0, 3, 384, 512)
    assert cost[0] == sum(p + 1 for p in range(384, 512))


def test_truncation_and_underfull():
    cu, consumed, tiles, cost, pc = pack_plan([300, 300, 300], 700, 128, 0)
    assert cu == [0, 300, 600, 700] and consumed == 3
    cu, consumed, *_ = pack_plan([300, 300, 300], 600, 128, 0)
    assert cu == [0, 300, 600] and consumed == 2      # third sample untouched
    cu, consumed, *_ = pack_plan([100, 50], 4096, 128, 0)
    assert cu == [0, 100, 150] and consumed == 2      # under-full pack is legal, no padding
    with pytest.raises(ValueError):
        pack_plan([10, 0, 5], 64, 16, 0)
    with pytest.raises(ValueError):
        pack_plan([10], 0, 16, 0)
    # a non-positive length is an error wherever it stands, also behind the point where the pack is full
    with pytest.raises(ValueError):
        pack_plan([4, 4, 0], 4, 16, 0)
    with pytest.raises(ValueError):
        pack_plan([4, 4, -3], 8, 16, 1)


@pytest.mark.parametrize("kind", [0, 1])
def test_brute_force_pairs_and_partition(kind):
    rnd = random.Random(7)
    for trial in range(30):
        lengths = [rnd.randint(1, 70) for _ in range(rnd.randint(1, 9))]
        pack_len = rnd.randint(1, sum(lengths) + 20)
        B = rnd.choice([1, 3, 16, 32])
        cu, consumed, tiles, cost, pc = pack_plan(lengths, pack_len, B, kind)
        T = cu[-1]
        assert T == min(pack_len, sum(lengths))
        # brute force: enumerate every causal in-sample pair and charge it to its tile
        charge = {}
        for i in range(len(cu) - 1):
            for r in range(cu[i], cu[i + 1]):
                for k in range(cu[i], r + 1):
                    owner = r if kind == 0 else k
                    key = (i, (owner - cu[i]) // B)
                    charge[key] = charge.get(key, 0) + 1
        got = {(s, t): c for (s, t, _, _), c in zip(tiles, cost)}
        assert got == charge
        # tiles partition [0, T) and never straddle samples
        covered = sorted((b, e) for (_, _, b, e) in tiles)
        pos = 0
        for b, e in covered:
            assert b == pos and e > b
            pos = e
        assert pos == T
        for (s, t, b, e) in tiles:
            assert cu[s] <= b and e <= cu[s + 1] and e - b <= B and b == cu[s] + t * B
        # order: generic re-sort agrees
        order = sorted(range(len(tiles)), key=lambda j: (-cost[j], tiles[j][0], tiles[j][1]))
        assert order == list(range(len(tiles)))
        assert sum(cost) == sum(s * (s + 1) // 2 for s in [cu[i + 1] - cu[i] for i in range(len(cu) - 1)])
        assert pc == sum((cu[i + 1] - cu[i]) ** 2 for i in range(len(cu) - 1))


def test_closed_form_tile_costs():
    s, B = 1000, 128
    cu, _, tiles, cost, _ = pack_plan([s], s, B, 0)
    for (smp, t, b, e), c in zip(tiles, cost):
        lo, hi = b, e
        assert c == (hi * (hi + 1) - lo * (lo + 1)) // 2
    cu, _, tiles, cost, _ = pack_plan([s], s, B, 1)
    for (smp, t, b, e), c in zip(tiles, cost):
        n = e - b
        assert c == n * s - (b + e - 1) * n // 2
