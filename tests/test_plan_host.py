"""hbp_pack_plan (C++, through the C ABI) against the integer oracle: bit-exact."""
import random

import numpy as np
import pytest

import hbp_workloads as wl
import paper_2503_07680_amd as H
from oracle import pack_plan as oracle_plan


def check(lengths, pack_len, rows, kind):
    cu, nc, tiles, cost, pc = H.hbp_pack_plan(lengths, pack_len, rows, kind)
    ocu, onc, otiles, ocost, opc = oracle_plan(lengths, pack_len, rows, kind)
    assert cu.dtype == np.int32 and cu.tolist() == ocu
    assert nc == onc and pc == opc
    assert [tuple(t) for t in tiles.tolist()] == otiles
    assert cost.tolist() == ocost


@pytest.mark.parametrize("kind", [H.HBP_TILES_QUERY, H.HBP_TILES_KEY])
def test_benchmark_packs_bit_exact(kind):
    for idx in (1, 2, 3, 4, 5):
        w = wl.workload(idx)
        check(list(w.lengths), w.pack_len, 128, kind)
    for seed in (1, 2):
        w = wl.workload(3, seed)
        check(list(w.lengths), w.pack_len, 128, kind)


@pytest.mark.parametrize("kind", [0, 1])
def test_random_lists_bit_exact(kind):
    rnd = random.Random(11 + kind)
    for _ in range(200):
        lengths = [rnd.choice([1, 2, 31, 32, 33, 127, 128, 129, rnd.randint(1, 700)])
                   for _ in range(rnd.randint(1, 40))]
        pack_len = rnd.randint(1, sum(lengths) + 50)
        check(lengths, pack_len, rnd.choice([1, 7, 32, 64, 128]), kind)


def test_tiny_pack_matches_expected_cu():
    cu, nc, tiles, cost, pc = H.hbp_pack_plan([512, 256, 128, 64, 64], 1024, 128, 0)
    assert cu.tolist() == [0, 512, 768, 896, 960, 1024]
    assert pc == 352256 and int(cost.sum()) == 176640


def test_many_tiny_samples_and_single_sample():
    check([1] * 1000, 1000, 128, 0)
    check([1] * 1000, 777, 128, 1)
    check([98304], 98304, 128, 1)
    check([5], 100, 128, 0)


def test_error_codes():
    for bad, pack_len in (([3, 0, 4], 64), ([3, -1], 64), ([4, 4, 0], 4), ([4, 4, -3], 8)):
        with pytest.raises(H.HbpError) as e:
            H.hbp_pack_plan(bad, pack_len, 16, 0)
        assert e.value.status == 1
        with pytest.raises(ValueError):          # the oracle rejects the same lists (also a bad length
            oracle_plan(bad, pack_len, 16, 0)    # that lies behind the point where the pack is full)
    for args in (([4], 0, 16, 0), ([4], 16, 0, 0), ([4], 16, 16, 2)):
        with pytest.raises(H.HbpError) as e:
            H.hbp_pack_plan(*args)
        assert e.value.status == 1
    # empty list: a legal empty plan
    cu, nc, tiles, cost, pc = H.hbp_pack_plan([], 16, 16, 0)
    assert cu.tolist() == [0] and nc == 0 and len(tiles) == 0 and pc == 0


def test_capacity_errors_through_raw_abi():
    import ctypes
    lib = H.load_library()
    L = (ctypes.c_int32 * 3)(100, 100, 100)
    ns, nc, nt = ctypes.c_int32(), ctypes.c_int32(), ctypes.c_int32()
    pc = ctypes.c_int64()
    cu = (ctypes.c_int32 * 2)()
    st = lib.hbp_pack_plan(L, 3, 300, 64, 0, cu, 2, ctypes.byref(ns), ctypes.byref(nc), None, None, 0,
                           ctypes.byref(nt), ctypes.byref(pc))
    assert st == 4 and ns.value == 3 and nt.value == 6          # HBP_ERR_CAPACITY, counts still set
    st = lib.hbp_pack_plan(L, 3, 300, 64, 0, None, 0, None, ctypes.byref(nc), None, None, 0,
                           ctypes.byref(nt), ctypes.byref(pc))
    assert st == 1
