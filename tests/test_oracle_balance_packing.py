"""Pins of the Balance Packing oracle: what the paper prints, hand-worked cases, invariants."""
import numpy as np
import pytest

from oracle import balance_packing as bp


def lognormal(n, median, sigma, lo, hi, seed):
    r = np.random.default_rng(seed)
    return [int(v) for v in np.clip(np.rint(np.exp(r.normal(np.log(median), sigma, n))), lo, hi)]


def test_paper_worked_example_abr():
    """Section 3.1: {1K x4} and {2K x2} fill a 4K pack alike, cost 4K^2 vs 8K^2, ABR = 0.25
    (tests/golden/paper_abr_example.txt holds the printed numbers)."""
    K = 1024
    lengths = [K] * 4 + [2 * K] * 2
    batches = bp.balance_packing(lengths, [4 * K], [2], shuffle_seed=0)
    assert len(batches) == 1 and len(batches[0]["packs"]) == 2
    costs = sorted(sum(lengths[x] ** 2 for x in g) for g in batches[0]["packs"])
    assert costs == [4 * K * K, 8 * K * K]
    m = bp.metrics(batches, lengths, [4 * K], [2], [1])
    assert m["ABR"] == pytest.approx(0.25, abs=1e-15)
    assert m["PR"] == 0.0 and m["DBR"] == 0.0 and m["CR"] == 0.0 and m["AveT"] == 4 * K


def test_group_data_intervals_are_half_open_on_the_left():
    """GroupData: len(x) in (l_{i-1}, l_i]."""
    g = bp.group_data([1, 4, 5, 8, 9, 16], [4, 8, 16])
    assert g == [[0, 1], [2, 3], [4, 5]]
    with pytest.raises(ValueError):
        bp.group_data([17], [4, 8, 16])
    with pytest.raises(ValueError):
        bp.group_data([0], [4])


def test_first_fit_decreasing_hand_case():
    # 7,5,4,3,2,2 into 10: 7 | 5 | 4 joins 5 | 3 joins 7 | 2 opens a third pack | 2 joins it
    assert bp.packing_ffd(list(range(6)), [7, 5, 4, 3, 2, 2], 10) == [[0, 3], [1, 2], [4, 5]]
    # ties keep input order
    assert bp.packing_ffd([0, 1, 2], [5, 5, 5], 10) == [[0, 1], [2]]


def test_greedy_fill_scans_packs_then_groups_downwards_then_samples_in_order():
    """GreedyFill: an exact fit is allowed (<= l_i); D_{i-1} is tried before D_{i-2}; a sample that does
    not fit is skipped, later ones are still tried; what is taken leaves its group."""
    lengths = [10, 9,      # level 2 samples (packs of 16)
               6, 5, 3,    # level 1 (len in (4, 8])
               4, 2, 1]    # level 0 (len <= 4)
    packs = [[0], [1]]
    d1, d0 = [2, 3, 4], [5, 6, 7]
    bp.greedy_fill(packs, 16, [d1, d0], lengths)
    # pack 0 (10): takes 6 -> 16, full.  pack 1 (9): 5 -> 14; 3 does not fit; then level 0: 4 no, 2 -> 16
    assert packs == [[0, 2], [1, 3, 6]]
    assert d1 == [4] and d0 == [5, 7]


def test_attention_balance_sort_orders_by_sum_of_squares():
    lengths = [4, 4, 8, 1, 7]
    packs = [[0, 1], [2], [3, 4]]           # a = 32, 64, 50
    assert bp.attention_balance_sort(packs, lengths) == [[2], [3, 4], [0, 1]]


def test_splitmix64_published_vectors():
    g = bp.splitmix64_stream(1234567)
    assert [next(g) for _ in range(3)] == [6457827717110365317, 3203168211198807973, 9817491932198370423]
    g = bp.splitmix64_stream(0)
    assert next(g) == 0xE220A8397B1DCDAF


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_invariants_on_mixed_lengths(seed):
    lengths = lognormal(3000, 600, 1.2, 16, 32768, seed)
    group_lens, per_batch = [4096, 16384, 32768], [8, 4, 2]
    batches = bp.balance_packing(lengths, group_lens, per_batch, shuffle_seed=seed)
    seen = []
    for b in batches:
        i = b["level"]
        assert 1 <= len(b["packs"]) <= per_batch[i]
        for g in b["packs"]:
            assert sum(lengths[x] for x in g) <= group_lens[i]
            lo = group_lens[i - 1] if i else 0
            assert lo < lengths[g[0]] <= group_lens[i]          # opened by a sample of its own group
            assert all(lengths[x] <= group_lens[i] for x in g)  # filled from its own or smaller groups
            seen += g
    assert sorted(seen) == list(range(len(lengths)))             # every sample exactly once
    # packs inside a batch are in descending attention complexity
    for b in batches:
        a = [sum(lengths[x] ** 2 for x in g) for g in b["packs"]]
        assert a == sorted(a, reverse=True)


def test_sorting_by_attention_complexity_lowers_abr():
    """The paper's point (Section 5.3 ablation: ABR 0.288 -> 0.002 with balance batching): batches of
    neighbouring packs after the sort are far better balanced than batches of packs in packing order."""
    lengths = lognormal(20000, 600, 1.2, 16, 4096, 7)
    cap, per_batch = 4096, 8
    packs = bp.packing_ffd(list(range(len(lengths))), lengths, cap)
    cost = lambda g: sum(lengths[x] ** 2 for x in g)
    def mean_abr(ps):
        full = [ps[s:s + per_batch] for s in range(0, len(ps) - per_batch + 1, per_batch)]
        return sum(bp.ratio_to_max([cost(g) for g in b]) for b in full) / len(full)
    r = np.random.default_rng(0)
    shuffled = [packs[i] for i in r.permutation(len(packs))]
    assert mean_abr(bp.attention_balance_sort(packs, lengths)) < 0.1 * mean_abr(shuffled)


def test_metrics_closed_forms():
    lengths = [8, 8, 4, 4, 4, 4]
    # level 1: two packs of 8+... ; build batches by hand
    batches = [{"level": 1, "packs": [[0], [1]]}, {"level": 0, "packs": [[2, 3], [4]]}, {"level": 0, "packs": [[5]]}]
    m = bp.metrics(batches, lengths, [8, 16], [2, 2], [1, 2])
    # level-1 batch: tokens 8,8 -> DBR 0, ABR 0.  level-0 full batch: tokens 8,4 -> DBR (8-4)/(8*2) = .25,
    # attention 32,16 -> ABR .25.  The short batch is left out of DBR/ABR.
    assert m["DBR"] == pytest.approx(0.125) and m["ABR"] == pytest.approx(0.125)
    # capacity 16+16 + 8+8 + 8 = 56, tokens 32 -> PR = 24/56; CR: level-1 tokens 16 of 32; Ave-T = 32/5
    assert m["PR"] == pytest.approx(24 / 56) and m["CR"] == pytest.approx(0.5) and m["AveT"] == pytest.approx(6.4)


def test_bad_arguments():
    with pytest.raises(ValueError):
        bp.balance_packing([1], [4, 4], [1, 1], 0)
    with pytest.raises(ValueError):
        bp.balance_packing([1], [4], [0], 0)
    with pytest.raises(ValueError):
        bp.balance_packing([1], [], [], 0)
