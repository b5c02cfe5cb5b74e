"""The C++ Balance Packing planner against the oracle: integer outputs bit-exact, metrics to rounding."""
import numpy as np
import pytest

import paper_2503_07680_amd as H
from oracle import balance_packing as bp


def lognormal(n, median, sigma, lo, hi, seed):
    r = np.random.default_rng(seed)
    return [int(v) for v in np.clip(np.rint(np.exp(r.normal(np.log(median), sigma, n))), lo, hi)]


def as_lists(batches, packs, items):
    out = []
    for b in batches:
        ps = []
        for p in packs[b["first_pack"]:b["first_pack"] + b["n_packs"]]:
            assert p["level"] == b["level"]
            ps.append([int(x) for x in items[p["first_item"]:p["first_item"] + p["n_items"]]])
        out.append({"level": int(b["level"]), "packs": ps})
    return out


CASES = [
    ([1024] * 4 + [2048] * 2, [4096], [2], [1], 0),
    (lognormal(500, 600, 1.2, 16, 4096, 0), [4096], [8], [1], 1),
    (lognormal(4000, 600, 1.2, 16, 32768, 1), [4096, 16384, 32768], [8, 4, 2], [1, 2, 4], 2),
    (lognormal(2500, 3000, 1.5, 1, 131072, 2), [2048, 8192, 32768, 131072], [16, 8, 4, 1], [1, 1, 4, 8], 3),
    ([5] * 37, [4, 8], [3, 3], [1, 1], 4),                       # an empty level, a short last batch
    ([1, 2, 3, 4, 4, 3, 2, 1], [4], [1], None, 5),                # batches of one pack
    ([], [16], [2], [1], 6),                                      # empty dataset
]


@pytest.mark.parametrize("lengths,group_lens,per_batch,sp,seed", CASES)
def test_planner_matches_oracle_bit_for_bit(lengths, group_lens, per_batch, sp, seed):
    batches, packs, items, m = H.hbp_balance_packing(lengths, group_lens, per_batch, sp, seed)
    want = bp.balance_packing(lengths, group_lens, per_batch, seed)
    assert as_lists(batches, packs, items) == want
    for p in packs:
        g = items[p["first_item"]:p["first_item"] + p["n_items"]]
        assert p["n_tokens"] == sum(lengths[x] for x in g)
        assert p["attn_cost"] == sum(lengths[x] ** 2 for x in g)
    wm = bp.metrics(want, lengths, group_lens, per_batch, sp if sp is not None else [1] * len(group_lens))
    for k in wm:
        assert m[k] == pytest.approx(wm[k], rel=1e-12, abs=1e-15), k
    nb, npk, none, m2 = H.hbp_balance_packing(lengths, group_lens, per_batch, sp, seed, lists=False)
    assert (nb, npk, none) == (len(batches), len(packs), None) and m2 == m


def test_size_query_capacity_and_argument_errors():
    import ctypes
    lib = H.load_library()
    L = np.array([3, 3, 3], dtype=np.int32)
    G = np.array([4], dtype=np.int32)
    B = np.array([1], dtype=np.int32)
    n_p, n_b = ctypes.c_int32(), ctypes.c_int32()
    call = lambda items, icap, packs, pcap, batches, bcap, g=G, b=B, l=L: lib.hbp_balance_packing(
        l.ctypes.data, l.size, g.ctypes.data, b.ctypes.data, None, g.size, 0, items, icap, packs, pcap,
        ctypes.byref(n_p), batches, bcap, ctypes.byref(n_b), None)
    assert call(None, 0, None, 0, None, 0) == 0 and (n_p.value, n_b.value) == (3, 3)
    items = np.zeros(3, np.int32)
    packs = np.zeros(3, H.binding.PACK_DTYPE)
    batches = np.zeros(3, H.binding.BATCH_DTYPE)
    assert call(items.ctypes.data, 3, packs.ctypes.data, 2, batches.ctypes.data, 3) == 4   # HBP_ERR_CAPACITY
    assert (n_p.value, n_b.value) == (3, 3)
    assert call(items.ctypes.data, 3, None, 3, batches.ctypes.data, 3) == 1                # one list missing
    assert call(None, 0, None, 0, None, 0, g=np.array([4, 4], np.int32), b=np.array([1, 1], np.int32)) == 1
    assert call(None, 0, None, 0, None, 0, b=np.array([0], np.int32)) == 1
    assert call(None, 0, None, 0, None, 0, l=np.array([5], np.int32)) == 1                 # longer than l_n
    assert call(None, 0, None, 0, None, 0, l=np.array([0], np.int32)) == 1


def test_a_hundred_thousand_samples_same_as_oracle_on_a_prefix_and_fast():
    """Structure check at size: every sample once, no pack over its length; the scan-free search
    trees give the oracle's answer (checked on a 6000-sample prefix, which the oracle does in seconds)."""
    lengths = lognormal(100000, 600, 1.2, 16, 32768, 11)
    group_lens, per_batch = [4096, 16384, 32768], [8, 4, 2]
    batches, packs, items, m = H.hbp_balance_packing(lengths, group_lens, per_batch, [1, 2, 4], 9)
    assert sorted(items.tolist()) == list(range(len(lengths)))
    L = np.asarray(lengths)
    for p in packs[:: max(1, len(packs) // 500)]:
        assert L[items[p["first_item"]:p["first_item"] + p["n_items"]]].sum() <= group_lens[p["level"]]
    assert m["PR"] < 0.02
    sub = lengths[:6000]
    b2, p2, i2, _ = H.hbp_balance_packing(sub, group_lens, per_batch, [1, 2, 4], 9)
    assert as_lists(b2, p2, i2) == bp.balance_packing(sub, group_lens, per_batch, 9)
