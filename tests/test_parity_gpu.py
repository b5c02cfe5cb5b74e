"""GPU parity: the HIP path (through the C ABI) against the fp64 oracle on the same seeded inputs."""
import numpy as np
import pytest

import hbp_workloads as wl
from parity_util import Case, run_gpu, check_plan, compare, compare_sample_dense, check_dv_identity, sampled_rows

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


def test_packs_of_one_token_samples_only():
    """dQ and dK are identically zero here (every probability is 1, dP = D); the kernels' values must vanish
    to rounding (see GRAD_ABS_RMS), dV = the sum of dO over the group, O = V, LSE = the one score."""
    for lengths, Hq, Hkv, d, e in (([1], 8, 1, 192, 128), ([1, 1, 1, 1, 1], 4, 2, 128, 128), ([1] * 70, 2, 2, 64, 64)):
        pa, dev, out = full(Case(lengths, len(lengths), Hq, Hkv, d, e, seed=29, name="ones-%d" % len(lengths)))
        assert np.abs(out["dq"]).max() <= 1e-4 and np.abs(out["dk"]).max() <= 1e-4


def test_explicit_scale_and_small_sigma():
    full(Case([190, 66], 256, 4, 4, 64, 64, seed=26, sigma=0.5, scale=0.2, name="scale"))


def test_peaked_softmax_with_large_logits():
    """Scores with a standard deviation of about 18 (Q, K drawn with sigma 4, scale 1/sqrt(d)): every row's
    softmax is dominated by a few keys, the running maximum moves often (the lazy rescale takes its slow
    path) and most probabilities underflow.  Relative bars on every tensor (the absolute bars on O are for
    values of unit scale), LSE to 1e-3 relative to its size."""
    import oracle
    from parity_util import rel_l2
    case = Case([700, 129, 33, 1, 260], 1123, 8, 2, 128, 128, seed=91, sigma=4.0, name="peaked")
    pa, dev, out = run_gpu(case)
    check_plan(case, pa)
    f32 = lambda w: wl.bf16_bits_to_f32(case.bits(w, pa.T))
    q, k, v, do = f32("q"), f32("k"), f32("v"), f32("do")
    cu = np.asarray(pa.cu, dtype=np.int32)
    O, LSE = oracle.attn_fwd(q, k, v, cu, None)
    dQ = oracle.attn_bwd_dq(q, k, v, do, cu, None)
    dK, dV = oracle.attn_bwd_dkdv(q, k, v, do, cu, None)
    res = {"o_rel": rel_l2(out["o"], O), "lse_rel": float(np.abs(out["lse"] - LSE).max() / np.abs(LSE).max()),
           "dq_rel": rel_l2(out["dq"], dQ), "dk_rel": rel_l2(out["dk"], dK), "dv_rel": rel_l2(out["dv"], dV)}
    print("[parity peaked]", " ".join("%s=%.3e" % kv for kv in res.items()), "max |LSE| %.1f" % np.abs(LSE).max(), flush=True)
    assert np.isfinite(out["o"]).all() and np.isfinite(out["dq"]).all() and np.isfinite(out["dk"]).all()
    assert res["o_rel"] <= 1e-2 and res["lse_rel"] <= 1e-3
    assert max(res["dq_rel"], res["dk_rel"], res["dv_rel"]) <= 1e-2, res


def test_scores_that_grow_along_the_sample_move_the_reference():
    """The forward takes every probability of a row against one reference, the maximum of the row's first 32
    keys, and moves it only when a later block would leave the range of fp32.  Here the keys grow along the
    sample (|K| rises from 1 to 40 times its start), so later scores exceed the first block's by hundreds of
    units and the reference must move, several times per row; a second sample has its large keys FIRST (the
    reference never moves and most later probabilities underflow).  Relative bars as in the peaked case."""
    import oracle
    import torch
    from paper_2503_07680_amd.runner import PackedAttention
    from parity_util import rel_l2
    lengths, Hq, Hkv, d, e = [900, 700, 70], 4, 2, 128, 128
    T = sum(lengths)
    rng = np.random.default_rng(93)
    ramp = np.concatenate([np.linspace(1.0, 40.0, 900), np.linspace(40.0, 1.0, 700), np.linspace(1.0, 25.0, 70)])
    bf = lambda x: wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(x.astype(np.float32)))
    q = bf(rng.standard_normal((T, Hq, d)))
    k = bf(rng.standard_normal((T, Hkv, d)) * ramp[:, None, None])
    v = bf(rng.standard_normal((T, Hkv, e)))
    do = bf(rng.standard_normal((T, Hq, e)))
    pa = PackedAttention(lengths, T, Hq, Hkv, d, e)
    dev = [pa.to_device_bf16(wl.f32_to_bf16_bits(x)) for x in (q, k, v, do)]
    pa.forward(*dev[:3])
    pa.backward(*dev)
    torch.cuda.synchronize()
    cu = np.asarray(pa.cu, dtype=np.int32)
    O, LSE = oracle.attn_fwd(q, k, v, cu, None)
    dQ = oracle.attn_bwd_dq(q, k, v, do, cu, None)
    dK, dV = oracle.attn_bwd_dkdv(q, k, v, do, cu, None)
    got = {n: t.float().cpu().numpy() for n, t in (("o", pa.o), ("dq", pa.dq), ("dk", pa.dk), ("dv", pa.dv))}
    lse = pa.lse.cpu().numpy()
    res = {"o_rel": rel_l2(got["o"], O), "lse_rel": float(np.abs(lse - LSE).max() / np.abs(LSE).max()),
           "dq_rel": rel_l2(got["dq"], dQ), "dk_rel": rel_l2(got["dk"], dK), "dv_rel": rel_l2(got["dv"], dV)}
    print("[parity growing-scores]", " ".join("%s=%.3e" % kv for kv in res.items()),
          "LSE from %.1f to %.1f" % (LSE.min(), LSE.max()), flush=True)
    assert all(np.isfinite(x).all() for x in got.values()) and np.isfinite(lse).all()
    assert res["o_rel"] <= 1e-2 and res["lse_rel"] <= 1e-3
    assert max(res["dq_rel"], res["dk_rel"], res["dv_rel"]) <= 1e-2, res


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
    # Key columns.  Every key of three short samples and of the last sample; in the 16384 sample (key tiles
    # of 128, taken 32 at a time by the workgroups of a kv head, every second set of 32 in the wrapped block
    # order) columns in all four sets: tiles 0, 16 (plain order), 32, 48, 63 (wrapped), 64, 95 (plain),
    # and the tail, 120..127 (wrapped), at tile edges and inside tiles.
    cols = list(range(int(pa.cu[1]), int(pa.cu[3]))) + list(range(int(pa.cu[-2]), int(pa.cu[-1])))
    cols += [0, 1, 100, 127, 128, 2049, 4095] + list(range(4096, 4101)) + [6207, 8191, 8192, 10000, 12287, 12288]
    cols += list(range(16384 - 160, 16384)) + [16384 - 1000, 16384 - 513]
    cols = sorted(set(cols))
    compare(case, pa, out, q_heads=[8, 9, 10, 11], rows=rows, cols=cols, label="kv-group 2")
    compare(case, pa, out, q_heads=[0, 31], rows=rows[::4], label="first/last head")
    print("[parity mixed-32k] sampled: %d of %d rows x 4+2 of 32 heads (O, LSE, dQ); %d of %d key columns x 1 of 8 kv "
          "heads (dK, dV), %d of them in the 16384 sample; sum-of-dV identity on every sample and head"
          % (len(rows), pa.T, len(cols), pa.T, sum(c < 16384 for c in cols)), flush=True)


def test_config3_long_sample_every_row_and_key_of_one_kv_group():
    """The 16384-token sample of the mixed pack carries 92 % of the pack's attention cost: every row and every
    key column of it, for one whole kv group (4 query heads), against the matrix-product oracle."""
    case = Case.from_workload(wl.workload(3))
    pa, dev, out = run_gpu(case)
    assert int(pa.cu[1]) == 16384
    compare_sample_dense(case, pa, out, sample=0, kv_head=5, label="16384 sample")


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
    print("[parity long-128k] GPU run and sum-of-dV identity done", flush=True)
    # the 32768 sample: every row and key column of one kv group (8 query heads)
    compare_sample_dense(case, pa, out, sample=1, kv_head=3, label="32768 sample")
    # the 98304 sample, kv group 3 (query heads 24..31).  Rows (O, LSE, dQ): sample and tile edges plus random
    # rows, 512 in all.  Key columns (dK, dV): a run inside key tile 735 (the 22nd set of 32 tiles: plain block
    # order), runs in tiles 736 and 750 and the sample's last 96 keys (23rd set: wrapped order).  The oracle
    # needs LSE and D of every row behind the first sampled column, which is what bounds how far down it goes.
    rng = np.random.default_rng(4)
    rows = set([0, 1, 31, 32, 127, 128, 255, 256, 4095, 4096, 49151, 49152, 65535, 65536, 98303 - 128, 98302, 98303])
    rows.update(int(x) for x in rng.integers(0, 98304, 512 - len(rows)))
    while len(rows) < 512:
        rows.add(int(rng.integers(0, 98304)))
    rows = sorted(rows)
    cols = list(range(94176, 94208)) + list(range(94208, 94224)) + list(range(96000, 96016)) + list(range(98304 - 96, 98304))
    compare(case, pa, out, q_heads=list(range(24, 32)), rows=rows, cols=cols, label="kv-group 3, 98304 sample")
    print("[parity long-128k] sampled: 32768 sample whole for 8 of 64 heads; 98304 sample %d of 98304 rows x 8 of 64 "
          "heads (O, LSE, dQ) and %d of 98304 key columns x 1 of 8 kv heads (dK, dV); sum-of-dV identity on both "
          "samples and every head" % (len(rows), len(cols)), flush=True)


@pytest.mark.parametrize("Hq,Hkv,d,e,pad_h", [(4, 2, 128, 128, 0), (2, 2, 64, 64, 8), (2, 1, 192, 128, 16)])
def test_strided_views_of_fused_buffers(Hq, Hkv, d, e, pad_h):
    """Q, K, V as column slices of one fused [T, W] projection buffer (and dQ, dK, dV of one fused
    gradient buffer), O and dO with padded heads: the descriptor's strides carry the layout.
    Results must equal the dense-layout run bit for bit, meet the oracle's bars, and no element
    outside the views may change."""
    import copy
    import torch
    from paper_2503_07680_amd import binding as B
    case = Case([150, 1, 290, 64, 33], 538, Hq, Hkv, d, e, seed=31, name="strided")
    pa, dev, dense = run_gpu(case)
    T, bf = pa.T, torch.bfloat16
    qh, kh, vh, oh = d + pad_h, d + pad_h, e + pad_h, e + pad_h      # head strides (elements)
    wq, wk, wv = Hq * qh, Hkv * kh, Hkv * vh
    W = wq + wk + wv + 24                                            # row stride of the fused buffer
    sentinel = 1.5
    fused = torch.full((T, W), sentinel, dtype=bf, device=pa.device)
    grads = torch.full((T, W), sentinel, dtype=bf, device=pa.device)
    o_buf = torch.full((T, Hq * oh + 8), sentinel, dtype=bf, device=pa.device)
    do_buf = torch.full((T, Hq * oh + 8), sentinel, dtype=bf, device=pa.device)

    def view(buf, col0, H, hs, dim):
        return buf[:, col0:col0 + H * hs].view(T, H, hs)[:, :, :dim]

    q_v, k_v, v_v = view(fused, 0, Hq, qh, d), view(fused, wq, Hkv, kh, d), view(fused, wq + wk, Hkv, vh, e)
    dq_v, dk_v, dv_v = view(grads, 0, Hq, qh, d), view(grads, wq, Hkv, kh, d), view(grads, wq + wk, Hkv, vh, e)
    o_v, do_v = view(o_buf, 0, Hq, oh, e), view(do_buf, 0, Hq, oh, e)
    q_v.copy_(dev["q"]); k_v.copy_(dev["k"]); v_v.copy_(dev["v"]); do_v.copy_(dev["do"])
    fused_before, do_before = fused.clone(), do_buf.clone()

    desc = copy.copy(pa.desc)
    desc.q_stride_t, desc.q_stride_h = W, qh
    desc.k_stride_t, desc.k_stride_h = W, kh
    desc.v_stride_t, desc.v_stride_h = W, vh
    desc.o_stride_t, desc.o_stride_h = o_buf.shape[1], oh
    lse = torch.zeros_like(pa.lse)
    stream = int(torch.cuda.current_stream().cuda_stream)
    B.hbp_varlen_attn_fwd(desc, q_v, k_v, v_v, pa.cu_dev, pa.fwd_tiles_dev, len(pa.fwd_tiles), o_v, lse,
                          pa.ws_fwd, None, stream)
    B.hbp_varlen_attn_bwd(desc, q_v, k_v, v_v, o_v, lse, do_v, pa.cu_dev, pa.q_tiles_dev, len(pa.q_tiles),
                          pa.kv_tiles_dev, len(pa.kv_tiles), dq_v, dk_v, dv_v, pa.ws_bwd, None, None, stream)
    torch.cuda.synchronize()

    assert torch.equal(fused, fused_before) and torch.equal(do_buf, do_before)      # inputs untouched
    for got, ref in ((o_v, pa.o), (lse, pa.lse), (dq_v, pa.dq), (dk_v, pa.dk), (dv_v, pa.dv)):
        assert torch.equal(got.contiguous(), ref)                                   # same as the dense layout
    out = {"o": o_v.float().cpu().numpy(), "lse": lse.cpu().numpy(), "dq": dq_v.float().cpu().numpy(),
           "dk": dk_v.float().cpu().numpy(), "dv": dv_v.float().cpu().numpy()}
    compare(case, pa, out, label="strided")
    # nothing outside the views was written
    for buf, views in ((grads, (dq_v, dk_v, dv_v)), (o_buf, (o_v,))):
        mask = torch.ones_like(buf, dtype=torch.bool)
        for vw, (col0, H, hs, dim) in zip(views, ((0, Hq, qh, d), (wq, Hkv, kh, d), (wq + wk, Hkv, vh, e))
                                          if buf is grads else ((0, Hq, oh, e),)):
            view(mask, col0, H, hs, dim).fill_(False)
        assert bool((buf[mask] == sentinel).all())


def test_descriptor_rejects_strides_that_break_alignment_or_overlap_rows():
    import copy
    import torch
    from paper_2503_07680_amd import binding as B
    case = Case([40], 40, 2, 2, 64, 64, seed=32, name="bad-strides")
    pa, dev, _ = run_gpu(case)
    stream = int(torch.cuda.current_stream().cuda_stream)
    for field, value in (("q_stride_h", 63), ("k_stride_t", 60), ("v_stride_h", 68), ("o_stride_t", 8)):
        desc = copy.copy(pa.desc)
        setattr(desc, field, value)
        with pytest.raises(B.HbpError):
            B.hbp_varlen_attn_fwd(desc, dev["q"], dev["k"], dev["v"], pa.cu_dev, pa.fwd_tiles_dev,
                                  len(pa.fwd_tiles), pa.o, pa.lse, pa.ws_fwd, None, stream)
    torch.cuda.synchronize()


@pytest.mark.parametrize("Hq,Hkv,d,e", [(3, 3, 128, 128), (3, 1, 64, 64), (2, 2, 192, 128)])
def test_odd_group_sizes_take_256_row_query_tiles_in_the_forward(Hq, Hkv, d, e):
    """With an odd number of query heads per kv head the forward pairs the two halves of a 256-row
    tile instead of two heads.  Both tile sizes must meet the oracle's bars and agree bit for bit
    (a row's arithmetic does not depend on which wavefronts share its K/V stream)."""
    import torch
    from paper_2503_07680_amd.runner import PackedAttention
    lengths = [700, 129, 256, 257, 31, 1, 400]
    case = Case(lengths, sum(lengths), Hq, Hkv, d, e, seed=33, name="tile256-%d-%d-%d" % (Hq, Hkv, d))
    pa, dev, out = run_gpu(case)
    assert pa.rows_fwd_pref == 256 and pa.desc.fwd_tile_rows == 256 and len(pa.fwd_tiles) < len(pa.q_tiles)
    check_plan(case, pa)
    compare(case, pa, out)
    small = PackedAttention(case.lengths, case.pack_len, Hq, Hkv, d, e, case.scale, fwd_tile_rows=128)
    assert small.desc.fwd_tile_rows == 0
    small.forward(dev["q"], dev["k"], dev["v"])
    torch.cuda.synchronize()
    assert torch.equal(small.o, pa.o) and torch.equal(small.lse, pa.lse)


def test_seeded_sweep_of_random_packs():
    """Two dozen seeded random packs: sample counts, lengths (many tiny, some spanning several tiles,
    lengths at and around the tile edges), head layouts (odd and even groups), all three head sizes,
    truncating and under-full pack lengths.  Every output against the oracle, plus the plan.  (Values stay
    at the workloads' scale, sigma <= 1: the absolute bar on O is about bf16 outputs of that magnitude.)"""
    rng = np.random.default_rng(2024)
    dims = [(64, 64), (128, 128), (192, 128)]
    edges = [1, 31, 32, 33, 63, 64, 65, 127, 128, 129, 255, 256, 257, 383, 384, 385]
    for i in range(24):
        n = int(rng.integers(1, 13))
        lengths = []
        for _ in range(n):
            kind = rng.random()
            if kind < 0.35:
                lengths.append(int(rng.integers(1, 40)))
            elif kind < 0.6:
                lengths.append(int(rng.choice(edges)))
            else:
                lengths.append(int(rng.integers(40, 700)))
        total = sum(lengths)
        pack_len = total if i % 3 else max(1, total - int(rng.integers(0, min(total, 200))))   # sometimes truncating
        if i % 5 == 0:
            pack_len = total + 77                                                              # under-full
        Hkv = int(rng.integers(1, 4))
        g = int(rng.integers(1, 5))
        d, e = dims[i % 3]
        scale = 0.0 if i % 4 else float(rng.uniform(0.05, 0.3))
        print("sweep case", i, lengths, pack_len, Hkv * g, Hkv, d, e, scale, flush=True)
        full(Case(lengths, pack_len, Hkv * g, Hkv, d, e, seed=100 + i, sigma=float(rng.choice([0.5, 1.0])),
                  scale=scale, name="sweep-%d" % i))


def test_seeded_sweep_of_larger_packs():
    """Ten seeded packs whose samples span many tiles (up to 2500 tokens: the unmasked hot loops of all three
    kernels, several query blocks per key tile, GQA groups of 1 to 8), with short samples in between and all
    three head sizes.  Every output of every head against the oracle, plus the plan and the dV identity."""
    rng = np.random.default_rng(4048)
    dims = [(128, 128), (64, 64), (192, 128)]
    for i in range(10):
        lengths = [int(rng.integers(600, 2500)) for _ in range(int(rng.integers(1, 3)))]
        lengths += [int(rng.integers(1, 300)) for _ in range(int(rng.integers(0, 5)))]
        order = rng.permutation(len(lengths))
        lengths = [lengths[j] for j in order]
        total = sum(lengths)
        pack_len = total if i % 2 else total - int(rng.integers(0, 100))
        Hkv = int(rng.choice([1, 2, 8]))
        g = int(rng.choice([1, 2, 4, 8])) if Hkv < 8 else int(rng.choice([1, 2]))
        d, e = dims[i % 3]
        print("larger sweep case", i, lengths, pack_len, Hkv * g, Hkv, d, e, flush=True)
        full(Case(lengths, pack_len, Hkv * g, Hkv, d, e, seed=300 + i, sigma=float(rng.choice([0.5, 1.0])),
                  name="sweep-large-%d" % i))


def test_long_sample_whose_later_key_tiles_start_below_the_top_and_wrap():
    """41 key tiles of one sample on 8 kv heads: 32 workgroups share a kv head, so key tiles 32..40 take
    their query blocks in the wrapped order (start below the sample's last block, skipped blocks last).
    A second, short sample rides along.  dK/dV of every key against the oracle."""
    full(Case([5197, 300], 5497, 8, 8, 64, 64, seed=41, name="wrap"))


def test_wrapped_block_order_with_a_group_of_four_heads_at_head_size_128():
    """The same 41-tile sample at the benchmark's head layout (32 query heads on 8 kv heads, d = 128): key
    tiles 32..40 take the wrapped order with the four heads of a group innermost.  Every key and row of two
    kv groups against the oracle, the sum-of-dV identity on all of them."""
    case = Case([5197, 300], 5497, 32, 8, 128, 128, seed=42, name="wrap-g4")
    pa, dev, out = run_gpu(case)
    check_plan(case, pa)
    check_dv_identity(case, pa, dev, out)
    compare_sample_dense(case, pa, out, sample=0, kv_head=0, label="group 0")
    compare(case, pa, out, q_heads=[20, 21, 22, 23], label="group 5")


@pytest.mark.parametrize("Hq,Hkv", [(8, 1), (12, 3), (8, 8)])
def test_few_kv_heads_split_their_query_heads_and_partial_tile_lists_leave_rows_alone(Hq, Hkv):
    """With fewer kv heads than dies the query heads of a kv head are dealt out in parts (dK/dV then come
    from partial sums and a reduce kernel).  All outputs against the oracle; and with a key-tile list
    that leaves tiles out, the dK/dV rows of those tiles keep what they held, in either form."""
    import torch
    from paper_2503_07680_amd import binding as B
    case = Case([700, 130, 1, 333], 1164, Hq, Hkv, 128, 128, seed=51, name="split-%d-%d" % (Hq, Hkv))
    pa, dev, out = full(case)
    keep = [i for i in range(len(pa.kv_tiles)) if i % 3 != 1]
    left_out = [pa.kv_tiles[i] for i in range(len(pa.kv_tiles)) if i % 3 == 1]
    tiles_dev = torch.from_numpy(np.ascontiguousarray(pa.kv_tiles[keep])).to(pa.device)
    sentinel = 3.0
    dk = torch.full_like(pa.dk, sentinel)
    dv = torch.full_like(pa.dv, sentinel)
    B.hbp_varlen_attn_bwd(pa.desc, dev["q"], dev["k"], dev["v"], pa.o, pa.lse, dev["do"], pa.cu_dev, pa.q_tiles_dev,
                          len(pa.q_tiles), tiles_dev, len(keep), pa.dq, dk, dv, pa.ws_bwd, None, None,
                          int(torch.cuda.current_stream().cuda_stream))
    torch.cuda.synchronize()
    covered = torch.zeros(pa.T, dtype=torch.bool, device=pa.device)
    for i in keep:
        covered[int(pa.kv_tiles[i][2]):int(pa.kv_tiles[i][3])] = True
    assert len(left_out) > 0 and bool((~covered).any())
    assert torch.equal(dk[covered], pa.dk[covered]) and torch.equal(dv[covered], pa.dv[covered])
    assert bool((dk[~covered] == sentinel).all()) and bool((dv[~covered] == sentinel).all())


@pytest.mark.parametrize("Hq,Hkv", [(24, 24), (40, 40), (34, 17)])
def test_head_counts_that_leave_dies_with_uneven_and_odd_numbers_of_kv_heads(Hq, Hkv):
    """24, 40 and 17 kv heads over 8 dies: 3, 5, and 2-or-3 kv heads per die, taken two at a time with a
    smaller last group.  Every head must be served exactly once (all outputs against the oracle)."""
    full(Case([300, 129, 64, 7], 500, Hq, Hkv, 64, 64, seed=61, name="heads-%d-%d" % (Hq, Hkv)))
