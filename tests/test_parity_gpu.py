"""GPU parity: the HIP path (through the C ABI) against the fp64 oracle on the same seeded inputs."""
import numpy as np
import pytest

import hbp_workloads as wl
from parity_util import Case, run_gpu, check_plan, compare, check_dv_identity, sampled_rows

pytestmark = pytest.mark.gpu


def full(case):
    pa, dev, out = run_gpu(case)
    check_plan(case, pa)
    compare(case, pa, out)
    check_dv_identity(case, pa, dev, out)
    return pa, dev, out


def test_config1_tiny_pack_all_outputs():
    full(Case.from_workload(wl.workload(1)))


RAGGED = [1, 2, 31, 32, 33, 63, 64, 65, 127, 128, 129, 200, 257, 5, 300]


@pytest.mark.parametrize("Hq,Hkv,d,e", [(2, 2, 64, 64), (4, 1, 128, 128), (2, 2, 192, 128), (6, 2, 128, 128)])
def test_ragged_lengths_span_tiles_and_tails(Hq, Hkv, d, e):
    full(Case(RAGGED, sum(RAGGED), Hq, Hkv, d, e, seed=21, name="ragged-%d-%d-%d-%d" % (Hq, Hkv, d, e)))


def test_truncated_last_sample_and_underfull_pack():
    full(Case([300, 300, 300], 700, 4, 2, 128, 128, seed=22, name="truncated"))
    full(Case([100, 50], 4096, 2, 2, 64, 64, seed=23, name="underfull"))


def test_many_one_token_samples_and_single_sample():
    full(Case([1] * 300 + [2] * 50 + [3] * 20, 460, 4, 2, 128, 128, seed=24, name="tiny-samples"))
    full(Case([777], 777, 2, 1, 128, 128, seed=25, name="single-sample"))


def test_explicit_scale_and_small_sigma():
    full(Case([190, 66], 256, 4, 4, 64, 64, seed=26, sigma=0.5, scale=0.2, name="scale"))


def test_forward_is_bit_stable_and_untouched_rows_stay():
    import torch
    case = Case([260, 130], 390, 4, 2, 128, 128, seed=27, name="stable")
    pa, dev, out = run_gpu(case)
    o1, l1 = pa.o.clone(), pa.lse.clone()
    pa.forward(dev["q"], dev["k"], dev["v"])
    torch.cuda.synchronize()
    assert torch.equal(o1, pa.o) and torch.equal(l1, pa.lse)      # no atomics in the forward


def test_config2_short_heavy_8k_all_outputs():
    full(Case.from_workload(wl.workload(2)))


def test_config3_mixed_32k_sampled():
    case = Case.from_workload(wl.workload(3))
    pa, dev, out = run_gpu(case)
    check_plan(case, pa)
    check_dv_identity(case, pa, dev, out)
    rng = np.random.default_rng(3)
    rows = sampled_rows(pa.cu, 300, rng)
    # columns: every key of three short samples, plus the tail of the 16384 sample
    cols = list(range(int(pa.cu[1]), int(pa.cu[3]))) + list(range(int(pa.cu[-2]), int(pa.cu[-1])))
    cols += list(range(16384 - 160, 16384)) + [16384 - 1000, 16384 - 513]
    compare(case, pa, out, q_heads=[8, 9, 10, 11], rows=rows, cols=sorted(set(cols)), label="kv-group 2")
    compare(case, pa, out, q_heads=[0, 31], rows=rows[::4], label="first/last head")


def test_config5_mla_32k_sampled():
    case = Case.from_workload(wl.workload(5))
    pa, dev, out = run_gpu(case)
    check_plan(case, pa)
    check_dv_identity(case, pa, dev, out)
    rng = np.random.default_rng(5)
    rows = sampled_rows(pa.cu, 200, rng)
    big = int(np.argmax(np.diff(pa.cu)))
    end = int(pa.cu[big + 1])
    cols = list(range(int(pa.cu[4]), int(pa.cu[5]))) + list(range(end - 130, end))
    compare(case, pa, out, q_heads=[0, 77, 127], rows=rows, cols=sorted(set(cols)), label="heads 0,77,127")


@pytest.mark.timeout(900)
def test_config4_long_128k_sampled():
    case = Case.from_workload(wl.workload(4))
    pa, dev, out = run_gpu(case)
    check_plan(case, pa)
    check_dv_identity(case, pa, dev, out)
    rng = np.random.default_rng(4)
    rows = sorted(set([0, 1, 127, 128, 98303, 98304, 98305, 131071, 98304 + 4095, 65535, 65536]
                      + [int(x) for x in rng.integers(0, 131072, 40)]))
    cols = list(range(98304 - 96, 98304)) + list(range(131072 - 96, 131072)) + [131072 - 300]
    compare(case, pa, out, q_heads=list(range(24, 32)), rows=rows, cols=sorted(set(cols)), label="kv-group 3")
