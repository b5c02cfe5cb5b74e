"""Packed cross-entropy kernel against the fp64 oracle, through the C ABI."""
import numpy as np
import pytest

import hbp_workloads as wl

pytestmark = pytest.mark.gpu

# token losses are fp32 sums of up to 131072 terms over exactly representable bf16 inputs
TOKEN_LOSS_ABS = 2e-5
LOSS_REL = 2e-6
# Gradients are stored in bf16: 8 significant bits, so a stored value is off by up to 2^-8 = 3.9e-3 of itself.
# Entries round independently and the relative L2 error of a row usually comes out near 2^-8 / sqrt(3) / 1.5, but
# when the large entries of a gradient are all the same number (rows dominated by their one-hot term -w, with a
# weight w such as 1/13 that bf16 does not hold) the whole tensor carries that one rounding error; the bar is the
# bound itself plus the fp32 arithmetic in front of the rounding.
GRAD_REL_L2 = 4e-3


def make_case(lens, V, seed, sigma=2.0, p_mask=0.3, stride=None):
    r = np.random.default_rng([77, seed])
    T = int(sum(lens))
    bits = wl.f32_to_bf16_bits((r.normal(0, sigma, (T, V))).astype(np.float32))
    y = r.integers(0, V, T).astype(np.int32)
    y[r.random(T) < p_mask] = -100
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    return bits, y, cu


def run_gpu(bits, y, cu, mode, t_ave=0.0, want_grad=True, stride=None):
    import torch
    import paper_2503_07680_amd as H
    T, V = bits.shape
    st = stride or V
    host = np.zeros((T, st), dtype=np.uint16)
    host[:, :V] = bits
    logits = torch.from_numpy(host.view(np.int16)).cuda()
    labels = torch.from_numpy(y).cuda()
    cud = torch.from_numpy(cu).cuda()
    dl = torch.full((T, V), 0x7FC0, dtype=torch.int16, device="cuda") if want_grad else None   # NaN pattern: must be overwritten
    loss = torch.full((1,), float("nan"), device="cuda")
    tl = torch.full((max(T, 1),), float("nan"), device="cuda")
    ws = torch.empty(H.hbp_packed_ce_workspace_bytes(T, len(cu) - 1), dtype=torch.uint8, device="cuda")
    H.hbp_packed_ce(logits, st if stride else 0, T, V, labels, cud, len(cu) - 1, mode, t_ave, dl, loss, tl, ws,
                    int(torch.cuda.current_stream().cuda_stream))
    torch.cuda.synchronize()
    grad = wl.bf16_bits_to_f32(dl.cpu().numpy().view(np.uint16)) if want_grad else None
    return float(loss.item()), tl.cpu().numpy()[:T], grad


def check(bits, y, cu, mode, t_ave=0.0, stride=None):
    from oracle import loss as L
    z = wl.bf16_bits_to_f32(bits).astype(np.float64)
    want_loss, want_tl, want_dz = L.packed_ce(z, y, cu, mode, t_ave)
    loss, tl, dz = run_gpu(bits, y, cu, mode, t_ave, stride=stride)
    assert np.abs(tl - want_tl).max() <= TOKEN_LOSS_ABS
    assert abs(loss - want_loss) <= LOSS_REL * max(abs(want_loss), 1e-30) + 1e-7
    assert not dz[y < 0].any()
    num = np.sqrt(((dz - want_dz) ** 2).sum())
    den = np.sqrt((want_dz ** 2).sum())
    assert num <= GRAD_REL_L2 * den, (num, den)
    # every gradient row sums to ~0 (softmax minus one-hot), up to the bf16 rounding of its entries
    assert np.abs(dz.sum(axis=1)).max() <= 2e-2 * np.abs(want_dz).sum(axis=1).max() + 1e-12
    return loss


@pytest.mark.parametrize("mode", [0, 1, 2])
def test_small_vocab_all_normalisers(mode):
    bits, y, cu = make_case([37, 5, 1, 90], 4096, mode)
    check(bits, y, cu, mode, t_ave=21.5)


@pytest.mark.parametrize("V", [8, 8192, 8200, 16384 + 8, 65536])
def test_vocab_sizes_around_the_chunk_boundaries(V):
    bits, y, cu = make_case([9, 14], V, V % 97)
    check(bits, y, cu, 2, t_ave=7.0)


def test_large_vocabularies_held_in_registers_and_a_longer_row_streamed_twice():
    bits, y, cu = make_case([6, 3], 128256, 1)      # 16 chunks of 8192 held per row
    check(bits, y, cu, 0)
    bits, y, cu = make_case([4, 2], 151936, 2)      # 19 chunks: the 20-chunk form
    check(bits, y, cu, 1)
    bits, y, cu = make_case([3, 2], 163848, 6)      # > 163840: streamed, running maximum and sum
    check(bits, y, cu, 2, t_ave=2.0)


def test_row_stride_and_more_rows_than_workgroups():
    bits, y, cu = make_case([700, 300, 200], 512, 3)
    check(bits, y, cu, 0, stride=520)


@pytest.mark.parametrize("V,T", [(24576, 2400), (128256, 700)])
def test_several_rows_per_workgroup_with_the_row_held_in_many_chunks(V, T):
    # the steady state of the chunk pipeline: gradient of one row, refill and statistics of the next,
    # rows with and without a loss following each other (3 and 16 chunks per row)
    lens = [T // 3, T // 2, T - T // 3 - T // 2]
    bits, y, cu = make_case(lens, V, 8 + V % 7)
    check(bits, y, cu, 2, t_ave=float(T) / 4)


def test_many_rows_per_workgroup_and_uneven_masking():
    # several hundred rows per workgroup: the per-row scalars are staged more than once; a long masked
    # prefix and a dense tail: the ranges of rows per workgroup have very different lengths
    lens = [50000, 70000, 30000, 50000]
    bits, y, cu = make_case(lens, 64, 7, p_mask=0.2)
    y[:90000] = -100
    y[12345] = 3
    check(bits, y, cu, 0)
    check(bits, y, cu, 1)
    loss, tl, _ = run_gpu(bits, y, cu, 2, t_ave=100.0, want_grad=False)
    from oracle import loss as L
    want_loss, want_tl, _ = L.packed_ce(wl.bf16_bits_to_f32(bits).astype(np.float64), y, cu, 2, 100.0)
    assert np.abs(tl - want_tl).max() <= TOKEN_LOSS_ABS
    assert abs(loss - want_loss) <= LOSS_REL * abs(want_loss) + 1e-7


def test_sample_without_loss_tokens_and_all_masked():
    bits, y, cu = make_case([10, 12, 8], 1024, 4)
    y[10:22] = -1
    check(bits, y, cu, 1)
    y[:] = -5
    loss, tl, dz = run_gpu(bits, y, cu, 0)
    assert loss == 0.0 and not tl.any() and not dz.any()


def test_large_logits_and_out_of_range_label_is_ignored():
    bits, y, cu = make_case([16], 2048, 5, sigma=30.0, p_mask=0.0)
    check(bits, y, cu, 0)
    y2 = y.copy(); y2[3] = 2048                      # >= V: treated as no loss
    y3 = y.copy(); y3[3] = -1
    a = run_gpu(bits, y2, cu, 0)
    b = run_gpu(bits, y3, cu, 0)
    assert a[0] == b[0] and np.array_equal(a[1], b[1]) and np.array_equal(a[2], b[2])
    # the oracle takes the same reading of such a label: all three normalisers on ordinary logits
    bits, y, cu = make_case([9, 17], 2048, 6, p_mask=0.2)
    y[3] = 2048
    y[20] = 5000
    for mode in (0, 1, 2):
        check(bits, y, cu, mode, 3.0)


def test_loss_is_bit_stable_and_gradient_optional():
    bits, y, cu = make_case([333, 691], 32000, 6)
    a = run_gpu(bits, y, cu, 2, 100.0)
    b = run_gpu(bits, y, cu, 2, 100.0)
    assert a[0] == b[0] and np.array_equal(a[1], b[1]) and np.array_equal(a[2], b[2])
    c = run_gpu(bits, y, cu, 2, 100.0, want_grad=False)
    assert c[0] == a[0] and np.array_equal(c[1], a[1])


def test_empty_input():
    import torch
    import paper_2503_07680_amd as H
    loss = torch.full((1,), float("nan"), device="cuda")
    ws = torch.empty(H.hbp_packed_ce_workspace_bytes(0, 0), dtype=torch.uint8, device="cuda")
    H.hbp_packed_ce(None, 0, 0, 8, None, None, 0, 0, 0.0, None, loss, None, ws,
                    int(torch.cuda.current_stream().cuda_stream))
    torch.cuda.synchronize()
    assert float(loss.item()) == 0.0
