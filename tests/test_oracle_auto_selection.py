"""Pins of the auto-selection oracle: the paper's printed tables and result, closed forms, hand cases."""
import math
import os

import pytest

from oracle import auto_selection as au

K = 1024
GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_auto_selection_tables.txt")


def read_golden():
    sec, out = None, {}
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        if line.startswith("["):
            sec = line.strip("[]")
            out[sec] = []
            continue
        out[sec].append([f.strip() for f in line.split(";")])
    return out


def test_stage2_on_the_papers_per_length_table_gives_the_papers_groups():
    """Appendix table of the best (SP, GC) per packing length -> argmin is 16K with (1, 28); l_1 = 16K,
    l_2 = 128K / 8 = 16K is not above l_best -> {16K, 128K} with SP {1, 8}: the auto row of the
    Section 5.3 table."""
    g = read_golden()
    lengths = [int(r[0]) * K for r in g["best_per_length"]]
    strategies = [(int(r[1]), int(r[2])) for r in g["best_per_length"]]
    times = [float(r[3]) for r in g["best_per_length"]]
    groups, sp, ckpt, j = au.stage2(lengths, strategies, times)
    want = {r[0]: [int(v) for v in r[1:]] for r in g["result"]}
    assert j == 1
    assert groups == [v * K for v in want["groups_k"]]
    assert sp == want["sp"]
    assert ckpt == [28, 28]


def test_find_best_sp_ckpt_on_the_papers_32k_table():
    """Appendix table at 32K: SP 1 does not fit, the fastest of the rest is SP 8 with 8 GC layers (2.82 s),
    the row the per-length table repeats for 32K."""
    g = read_golden()
    rows = {int(r[0]): (int(r[1]), None if r[2] == "OOM" else float(r[2])) for r in g["sp_at_32k"]}
    c_min, c_max = 20, 32

    def memory(l, sp, c):  # a linear model whose zero crossing is the table's GC layer count
        layers, t = rows[sp]
        if t is None:
            return -1.0 - (c_max - c)          # negative even with every layer checkpointed
        return 2.0 * (c - layers)              # 2 units per layer, zero remaining at `layers`

    def time(l, sp, c):
        layers, t = rows[sp]
        assert c == layers                     # the greedy estimate recovered the table's count
        return t

    assert au.find_best_sp_ckpt(32 * K, [1, 2, 4, 8, 16], c_min, c_max, memory, time) == (8, 8, 2.82)


def test_whole_algorithm_on_a_profile_built_from_the_papers_tables():
    g = read_golden()
    best = {int(r[0]) * K: (int(r[1]), int(r[2]), float(r[3])) for r in g["best_per_length"]}

    def memory(l, sp, c):
        return 1.5 * (c - best[l][1]) if sp >= best[l][0] else -5.0

    def time(l, sp, c):
        return best[l][2] * (1.0 + 0.1 * abs(math.log2(sp / best[l][0])))

    r = au.auto_selection(sorted(best), [1, 2, 4, 8, 16], 20, 32, memory, time)
    assert r["strategies"] == [best[l][:2] for l in sorted(best)]
    assert r["times"] == [best[l][2] for l in sorted(best)]
    assert (r["groups"], r["sp"], r["j"]) == ([16 * K, 128 * K], [1, 8], 1)


def test_greedy_ckpt_is_the_zero_crossing_of_the_linear_memory_model():
    """c_o = c_max - m2 / m_ave: exact for a linear model, rounded up to whole layers, never below 0."""
    for zero_at, slope in [(8, 2.0), (23, 0.7), (27.3, 1.9), (0, 3.0), (31.9, 0.5)]:
        mem = lambda l, sp, c: slope * (c - zero_at)
        assert au.greedy_profile_ckpt(32 * K, 2, 20, 32, mem) == math.ceil(zero_at - 1e-12)
    assert au.greedy_profile_ckpt(1, 1, 20, 32, lambda l, sp, c: 1.0 * (c + 5)) == 0         # fits with none
    assert au.greedy_profile_ckpt(1, 1, 20, 32, lambda l, sp, c: 1.0 * (c - 40)) is None     # OOM at c_max
    assert au.greedy_profile_ckpt(1, 1, 20, 32, lambda l, sp, c: 3.0) == 0                   # flat and fits
    # the appendix' own arithmetic: ave_m = (m1 - m2) / (32 - 20) with m1 at 32 layers, m2 at 20
    m_at = {32: 30.0, 20: 6.0}
    assert au.greedy_profile_ckpt(1, 1, 20, 32, lambda l, sp, c: m_at[c]) == 32 - math.floor(30.0 / ((30.0 - 6.0) / 12))


def test_stage2_four_groups_when_l2_exceeds_l_best_and_the_figure_example():
    """Section 4.1 figure: 32K with SP 2 -> every SP rank holds 16K, so l_1 = 16K.  With l_max = 128K at
    SP 2, l_2 = 64K > 32K: four groups."""
    groups, sp, ckpt, j = au.stage2([32 * K, 128 * K], [(2, 10), (2, 30)], [1.0, 2.0])
    assert (groups, sp, ckpt, j) == ([16 * K, 32 * K, 64 * K, 128 * K], [1, 2, 1, 2], [10, 10, 30, 30], 0)
    # floor division
    groups, sp, _, _ = au.stage2([1000, 3001], [(3, 0), (4, 0)], [1.0, 2.0])
    assert groups == [333, 1000, 3001] and sp == [1, 3, 4]


def test_degenerate_selections_collapse_repeated_lengths():
    assert au.stage2([8 * K], [(1, 4)], [1.0])[:2] == ([8 * K], [1])
    assert au.stage2([8 * K, 16 * K], [(1, 4), (2, 4)], [2.0, 1.0])[:2] == ([8 * K, 16 * K], [1, 2])
    assert au.stage2([8 * K, 16 * K], [(1, 4), (1, 9)], [1.0, 2.0]) == ([8 * K, 16 * K], [1, 1], [4, 9], 0)


def test_first_minimum_wins_infeasible_lengths_are_skipped_and_the_longest_must_fit():
    assert au.stage2([1, 2, 3], [(1, 0)] * 3, [2.0, 1.0, 1.0])[3] == 1
    assert au.stage2([4, 8, 16], [None, (2, 0), (4, 0)], [0.1, 1.0, 2.0])[3] == 1
    with pytest.raises(ValueError):
        au.stage2([4, 8], [(1, 0), None], [1.0, math.inf])
    t = lambda l, sp, c: {1: 5.0, 2: 3.0, 4: 3.0}[sp]
    assert au.find_best_sp_ckpt(8, [1, 2, 4], 1, 2, lambda l, sp, c: 1.0, t) == (2, 0, 3.0)
    assert au.find_best_sp_ckpt(8, [1, 2], 1, 2, lambda l, sp, c: -1.0, t) is None


def test_argument_checks():
    ok = (lambda l, sp, c: 1.0, lambda l, sp, c: 1.0)
    for lengths, sps in [([], [1]), ([8], []), ([8, 8], [1]), ([16, 8], [1]), ([0, 8], [1]), ([8], [0])]:
        with pytest.raises(ValueError):
            au.auto_selection(lengths, sps, 1, 2, *ok)
    with pytest.raises(ValueError):
        au.auto_selection([8], [1], 2, 2, *ok)
