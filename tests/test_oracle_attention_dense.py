"""Pins of the matrix-product form of the attention oracle (``oracle/attention_dense.py``): torch fp64
autograd through the dense masked definition (a library routine), closed forms, the row-at-a-time C
oracle (independent code), invariants, and independence from the row ranges it streams."""
import numpy as np
import pytest
import torch

import hbp_workloads as wl
from oracle import attn_fwd, attn_bwd_dq, attn_bwd_dkdv
from oracle.attention_dense import sample_dense


def make(s, Hq, Hkv, d, e, seed=0, sigma=1.0):
    f = lambda w, H, D: wl.bf16_bits_to_f32(wl.tensor_bits(seed, w, s, H, D, sigma))
    return f("q", Hq, d), f("k", Hkv, d), f("v", Hkv, e), f("do", Hq, e)


def torch_reference(q, k, v, d_o, scale):
    s, Hq, d = q.shape
    g = Hq // k.shape[1]
    tq, tk, tv = (torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in (q, k, v))
    S = scale * torch.einsum("rhd,khd->hrk", tq, tk.repeat_interleave(g, dim=1))
    S = S.masked_fill(torch.triu(torch.ones(s, s, dtype=torch.bool), diagonal=1)[None], float("-inf"))
    O = torch.einsum("hrk,khe->rhe", torch.softmax(S, dim=-1), tv.repeat_interleave(g, dim=1))
    (O * torch.tensor(d_o, dtype=torch.float64)).sum().backward()
    return (O.detach().numpy(), torch.logsumexp(S, dim=-1).detach().numpy(), tq.grad.numpy(), tk.grad.numpy(),
            tv.grad.numpy())


@pytest.mark.parametrize("s,Hq,Hkv,d,e,step", [(97, 4, 2, 16, 24, 32), (64, 3, 3, 8, 8, 64), (150, 8, 1, 32, 16, 7)])
def test_matches_autograd_of_the_dense_definition(s, Hq, Hkv, d, e, step):
    q, k, v, d_o = make(s, Hq, Hkv, d, e, seed=11)
    scale = 0.37
    got = sample_dense(q, k, v, d_o, scale, rows_per_step=step)
    want = torch_reference(q, k, v, d_o, scale)
    for a, b, name in zip(got, want, ("O", "LSE", "dQ", "dK", "dV")):
        assert np.abs(a - b).max() < 1e-11, name


def test_matches_the_row_at_a_time_oracle_and_the_default_scale():
    q, k, v, d_o = make(211, 6, 2, 32, 32, seed=12)
    cu = np.array([0, 211], dtype=np.int32)
    O, LSE, dQ, dK, dV = sample_dense(q, k, v, d_o, None, rows_per_step=50)
    O2, LSE2 = attn_fwd(q, k, v, cu, None)
    dQ2 = attn_bwd_dq(q, k, v, d_o, cu, None)
    dK2, dV2 = attn_bwd_dkdv(q, k, v, d_o, cu, None)
    for a, b in ((O, O2), (LSE, LSE2), (dQ, dQ2), (dK, dK2), (dV, dV2)):
        assert np.abs(a - b).max() < 1e-11


def test_closed_forms():
    # Q = 0: uniform probabilities over the keys seen so far
    q, k, v, d_o = make(40, 2, 1, 8, 8, seed=13)
    q0 = np.zeros_like(q)
    O, LSE, dQ, dK, dV = sample_dense(q0, k, v, d_o, 0.5, rows_per_step=16)
    p = np.arange(1, 41, dtype=np.float64)
    assert np.abs(LSE - np.log(p)[None, :]).max() < 1e-13
    running_mean = np.cumsum(v[:, 0].astype(np.float64), axis=0) / p[:, None]
    assert np.abs(O - running_mean[:, None, :]).max() < 1e-13
    # dV[k] = sum_h sum_{r >= k} dO[r,h] / (r+1);  dK = 0 (Q = 0)
    w = d_o.astype(np.float64).sum(axis=1) / p[:, None]
    assert np.abs(dV[:, 0] - np.cumsum(w[::-1], axis=0)[::-1]).max() < 1e-12
    assert np.abs(dK).max() == 0.0
    # a single token: O = V, LSE = the one score, dQ = dK = 0, dV = sum of dO over the group
    q, k, v, d_o = make(1, 4, 2, 8, 8, seed=14)
    O, LSE, dQ, dK, dV = sample_dense(q, k, v, d_o, 0.25)
    assert np.array_equal(O[0, 0], v[0, 0].astype(np.float64)) and np.array_equal(O[0, 3], v[0, 1].astype(np.float64))
    assert LSE[2, 0] == pytest.approx(0.25 * float(q[0, 2].astype(np.float64) @ k[0, 1].astype(np.float64)), abs=1e-14)
    assert np.abs(dQ).max() < 1e-15 and np.abs(dK).max() < 1e-15
    assert np.abs(dV[0, 1] - d_o[0, 2:4].astype(np.float64).sum(axis=0)).max() < 1e-14


def test_invariants_and_independence_of_the_row_ranges():
    q, k, v, d_o = make(130, 4, 2, 16, 16, seed=15)
    ref = sample_dense(q, k, v, d_o, None, rows_per_step=130)
    for step in (1, 33, 64, 1000):
        for a, b in zip(sample_dense(q, k, v, d_o, None, rows_per_step=step), ref):
            assert np.abs(a - b).max() < 1e-12
    O, LSE, dQ, dK, dV = ref
    # rows of P sum to one: sum_k dV[k, kh] = sum over the group's heads and all rows of dO
    want = d_o.astype(np.float64).sum(axis=0).reshape(2, 2, 16).sum(axis=1)
    assert np.abs(dV.sum(axis=0) - want).max() < 1e-11
    # causality: changing the last key/value changes no earlier output row
    k2, v2 = k.copy(), v.copy()
    k2[-1] += 1.0
    v2[-1] -= 2.0
    O2 = sample_dense(q, k2, v2, d_o, None)[0]
    assert np.array_equal(O2[:-1], O[:-1]) and not np.array_equal(O2[-1], O[-1])
