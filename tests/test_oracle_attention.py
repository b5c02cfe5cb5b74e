"""Pins of the fp64 attention oracle against things other than itself:
brute-force dense masked softmax (numpy matrices), torch fp64 autograd of the dense
definition, central finite differences, closed forms and structural invariants."""
import numpy as np
import pytest
import torch

import hbp_workloads as wl
from oracle import attn_fwd, attn_bwd_dq, attn_bwd_dkdv, prob_row


def make(T_lengths, Hq, Hkv, d, e, seed=0, sigma=1.0):
    cu = np.concatenate([[0], np.cumsum(T_lengths)]).astype(np.int32)
    T = int(cu[-1])
    f = lambda w, H, D: wl.bf16_bits_to_f32(wl.tensor_bits(seed, w, T, H, D, sigma))
    return f("q", Hq, d), f("k", Hkv, d), f("v", Hkv, e), f("do", Hq, e), cu


def dense_numpy(q, k, v, cu, scale):
    """Different code path: whole T x T score matrix per head, boolean mask, matrix ops."""
    T, Hq, d = q.shape
    Hkv = k.shape[1]
    g = Hq // Hkv
    sid = np.zeros(T, dtype=np.int64)
    for i in range(len(cu) - 1):
        sid[cu[i]:cu[i + 1]] = i
    idx = np.arange(T)
    allowed = (sid[:, None] == sid[None, :]) & (idx[None, :] <= idx[:, None])
    O = np.zeros((T, Hq, v.shape[2]))
    LSE = np.zeros((Hq, T))
    for h in range(Hq):
        S = scale * (q[:, h].astype(np.float64) @ k[:, h // g].astype(np.float64).T)
        S = np.where(allowed, S, -np.inf)
        m = S.max(axis=1, keepdims=True)
        E = np.exp(S - m)
        Z = E.sum(axis=1, keepdims=True)
        O[:, h] = (E / Z) @ v[:, h // g].astype(np.float64)
        LSE[h] = (m + np.log(Z))[:, 0]
    return O, LSE


def dense_torch_grads(q, k, v, d_o, cu, scale):
    """Library pin: autograd through the dense masked definition in float64."""
    T, Hq, d = q.shape
    Hkv = k.shape[1]
    g = Hq // Hkv
    tq = torch.tensor(q, dtype=torch.float64, requires_grad=True)
    tk = torch.tensor(k, dtype=torch.float64, requires_grad=True)
    tv = torch.tensor(v, dtype=torch.float64, requires_grad=True)
    sid = torch.zeros(T, dtype=torch.long)
    for i in range(len(cu) - 1):
        sid[cu[i]:cu[i + 1]] = i
    idx = torch.arange(T)
    allowed = (sid[:, None] == sid[None, :]) & (idx[None, :] <= idx[:, None])
    kk = tk.repeat_interleave(g, dim=1)
    vv = tv.repeat_interleave(g, dim=1)
    S = scale * torch.einsum("rhd,khd->hrk", tq, kk)
    S = S.masked_fill(~allowed[None], float("-inf"))
    P = torch.softmax(S, dim=-1)
    O = torch.einsum("hrk,khe->rhe", P, vv)
    (O * torch.tensor(d_o, dtype=torch.float64)).sum().backward()
    return tq.grad.numpy(), tk.grad.numpy(), tv.grad.numpy()


@pytest.mark.parametrize("lengths,Hq,Hkv,d,e", [
    ([64, 37, 1, 90, 5], 4, 2, 16, 16),
    ([200, 56], 2, 2, 32, 24),
    ([1, 1, 1], 3, 1, 8, 8),
])
def test_forward_matches_dense_masked_softmax(lengths, Hq, Hkv, d, e):
    q, k, v, d_o, cu = make(lengths, Hq, Hkv, d, e, seed=3)
    scale = 1.0 / np.sqrt(d)
    O, LSE = attn_fwd(q, k, v, cu, scale)
    O2, LSE2 = dense_numpy(q, k, v, cu, scale)
    assert np.abs(O - O2).max() < 1e-12
    assert np.abs(LSE - LSE2).max() < 1e-12


def test_default_scale_is_inverse_sqrt_d():
    q, k, v, d_o, cu = make([40, 24], 2, 1, 16, 16, seed=5)
    O, LSE = attn_fwd(q, k, v, cu, None)
    O2, LSE2 = dense_numpy(q, k, v, cu, 0.25)
    assert np.abs(O - O2).max() < 1e-12 and np.abs(LSE - LSE2).max() < 1e-12


def test_packed_equals_each_sample_alone():
    lengths = [50, 17, 80]
    q, k, v, d_o, cu = make(lengths, 4, 2, 16, 16, seed=1)
    O, LSE = attn_fwd(q, k, v, cu, 0.3)
    dQ = attn_bwd_dq(q, k, v, d_o, cu, 0.3)
    dK, dV = attn_bwd_dkdv(q, k, v, d_o, cu, 0.3)
    for i, s in enumerate(lengths):
        a, b = cu[i], cu[i + 1]
        one = np.array([0, s], dtype=np.int32)
        Oi, Li = attn_fwd(q[a:b], k[a:b], v[a:b], one, 0.3)
        assert np.abs(O[a:b] - Oi).max() < 1e-12 and np.abs(LSE[:, a:b] - Li).max() < 1e-12
        dQi = attn_bwd_dq(q[a:b], k[a:b], v[a:b], d_o[a:b], one, 0.3)
        dKi, dVi = attn_bwd_dkdv(q[a:b], k[a:b], v[a:b], d_o[a:b], one, 0.3)
        assert np.abs(dQ[a:b] - dQi).max() < 1e-12
        assert np.abs(dK[a:b] - dKi).max() < 1e-12 and np.abs(dV[a:b] - dVi).max() < 1e-12


def test_probability_rows_sum_to_one():
    q, k, v, d_o, cu = make([70, 30], 2, 2, 16, 16, seed=2)
    for r in [0, 1, 35, 69, 70, 99]:
        for h in range(2):
            P = prob_row(q, k, v, cu, h, r, 0.25)
            start = 0 if r < 70 else 70
            assert len(P) == r - start + 1
            assert abs(P.sum() - 1.0) < 1e-13 and (P > 0).all()


def test_closed_forms_zero_query_single_token_constant_keys():
    lengths = [33, 1, 20]
    q, k, v, d_o, cu = make(lengths, 2, 1, 8, 8, seed=4)
    # Q = 0: uniform probabilities -> LSE = ln(p+1), O = running mean of V
    O, LSE = attn_fwd(np.zeros_like(q), k, v, cu, 0.7)
    for i, s in enumerate(lengths):
        a = cu[i]
        for p in range(s):
            assert np.abs(LSE[:, a + p] - np.log(p + 1)).max() < 1e-13
            mean = v[a:a + p + 1, 0].astype(np.float64).mean(axis=0)
            assert np.abs(O[a + p, 0] - mean).max() < 1e-13
            assert np.abs(O[a + p, 1] - mean).max() < 1e-13
    # sample of one token: O = V, LSE = the single score, dQ = dK = 0, dV = sum of dO over the group
    O, LSE = attn_fwd(q, k, v, cu, 0.7)
    r = cu[1]
    assert np.abs(O[r, 0] - v[r, 0]).max() == 0
    s00 = 0.7 * float(q[r, 1].astype(np.float64) @ k[r, 0].astype(np.float64))
    assert abs(LSE[1, r] - s00) < 1e-13
    dQ = attn_bwd_dq(q, k, v, d_o, cu, 0.7)
    dK, dV = attn_bwd_dkdv(q, k, v, d_o, cu, 0.7)
    assert np.abs(dQ[r]).max() < 1e-15 and np.abs(dK[r]).max() < 1e-15
    assert np.abs(dV[r, 0] - d_o[r].astype(np.float64).sum(axis=0)).max() < 1e-13
    # all keys of a sample equal: uniform again, LSE shifted by the common score; and since the
    # rows of dS sum to zero, dQ = scale * (sum_k dS) * K_const = 0
    kc = k.copy()
    kc[:] = k[0]
    O, LSE = attn_fwd(q, kc, v, cu, 0.7)
    for p in range(33):
        sc = 0.7 * float(q[p, 0].astype(np.float64) @ k[0, 0].astype(np.float64))
        assert abs(LSE[0, p] - (sc + np.log(p + 1))) < 1e-12
    dQ = attn_bwd_dq(q, kc, v, d_o, cu, 0.7)
    assert np.abs(dQ).max() < 1e-13


def test_causality_and_sample_isolation():
    q, k, v, d_o, cu = make([40, 25], 2, 2, 16, 16, seed=6)
    O, LSE = attn_fwd(q, k, v, cu, 0.25)
    k2, v2 = k.copy(), v.copy()
    k2[17] += 1.0
    v2[17] -= 2.0
    O2, LSE2 = attn_fwd(q, k2, v2, cu, 0.25)
    assert np.abs(O2[:17] - O[:17]).max() == 0 and np.abs(LSE2[:, :17] - LSE[:, :17]).max() == 0
    assert np.abs(O2[17:40] - O[17:40]).max() > 1e-3          # later rows of the same sample move
    assert np.abs(O2[40:] - O[40:]).max() == 0                # the other sample does not


def test_row_and_column_subsets_match_full():
    q, k, v, d_o, cu = make([60, 30, 10], 4, 2, 16, 8, seed=8)
    O, LSE = attn_fwd(q, k, v, cu, 0.2)
    dQ, D = attn_bwd_dq(q, k, v, d_o, cu, 0.2, return_D=True)
    dK, dV = attn_bwd_dkdv(q, k, v, d_o, cu, 0.2)
    rows = [0, 59, 60, 61, 89, 90, 99, 33]
    Os, Ls = attn_fwd(q, k, v, cu, 0.2, rows=rows)
    assert np.array_equal(Os, O[rows]) and np.array_equal(Ls, LSE[:, rows])
    dQs = attn_bwd_dq(q, k, v, d_o, cu, 0.2, rows=rows)
    assert np.array_equal(dQs, dQ[rows])
    dKs, dVs = attn_bwd_dkdv(q, k, v, d_o, cu, 0.2, cols=rows)
    assert np.array_equal(dKs, dK[rows]) and np.array_equal(dVs, dV[rows])
    # D is rowsum(dO * O)
    assert np.abs(D - np.einsum("rhe,rhe->hr", d_o.astype(np.float64), O)).max() < 1e-12


@pytest.mark.parametrize("lengths,Hq,Hkv,d,e", [
    ([30, 11, 1, 22], 4, 2, 16, 16),
    ([48], 6, 2, 8, 24),
])
def test_gradients_match_torch_autograd_of_dense_definition(lengths, Hq, Hkv, d, e):
    q, k, v, d_o, cu = make(lengths, Hq, Hkv, d, e, seed=9)
    scale = 0.31
    dQ = attn_bwd_dq(q, k, v, d_o, cu, scale)
    dK, dV = attn_bwd_dkdv(q, k, v, d_o, cu, scale)
    gq, gk, gv = dense_torch_grads(q, k, v, d_o, cu, scale)
    assert np.abs(dQ - gq).max() < 1e-12
    assert np.abs(dK - gk).max() < 1e-12
    assert np.abs(dV - gv).max() < 1e-12


def test_gradients_match_central_finite_differences():
    lengths = [9, 1, 14]
    q, k, v, d_o, cu = make(lengths, 2, 1, 4, 4, seed=10)
    scale = 0.5
    dQ = attn_bwd_dq(q, k, v, d_o, cu, scale)
    dK, dV = attn_bwd_dkdv(q, k, v, d_o, cu, scale)
    q64, k64, v64 = (x.astype(np.float64) for x in (q, k, v))

    def loss(qq, kk, vv):
        O, _ = dense_numpy(qq, kk, vv, cu, scale)   # fp64 inputs, independent forward
        return float((O * d_o).sum())

    h = 1e-5
    for name, base, grad in (("q", q64, dQ), ("k", k64, dK), ("v", v64, dV)):
        num = np.zeros_like(base)
        it = np.nditer(base, flags=["multi_index"])
        for _ in it:
            i = it.multi_index
            plus = base.copy(); plus[i] += h
            minus = base.copy(); minus[i] -= h
            args = {"q": (q64, k64, v64), "k": (q64, k64, v64), "v": (q64, k64, v64)}[name]
            args = list(args)
            args["qkv".index(name)] = plus
            lp = loss(*args)
            args["qkv".index(name)] = minus
            lm = loss(*args)
            num[i] = (lp - lm) / (2 * h)
        rel = np.abs(num - grad).max() / max(np.abs(grad).max(), 1e-30)
        assert rel < 1e-6, (name, rel)


def test_dv_column_sum_identity_and_gqa_equals_replicated_mha():
    lengths = [25, 40]
    q, k, v, d_o, cu = make(lengths, 4, 2, 8, 8, seed=11)
    dK, dV = attn_bwd_dkdv(q, k, v, d_o, cu, 0.4)
    # P rows sum to one => sum_k dV[k,kh] = sum over the group's heads and the sample's rows of dO
    for i in range(2):
        a, b = cu[i], cu[i + 1]
        for kh in range(2):
            want = d_o[a:b, 2 * kh:2 * kh + 2].astype(np.float64).sum(axis=(0, 1))
            assert np.abs(dV[a:b, kh].sum(axis=0) - want).max() < 1e-12
    # GQA == MHA with K/V replicated; dK/dV summed back over each group
    kr, vr = np.repeat(k, 2, axis=1), np.repeat(v, 2, axis=1)
    O1, L1 = attn_fwd(q, k, v, cu, 0.4)
    O2, L2 = attn_fwd(q, kr, vr, cu, 0.4)
    assert np.abs(O1 - O2).max() < 1e-13 and np.abs(L1 - L2).max() < 1e-13
    dK2, dV2 = attn_bwd_dkdv(q, kr, vr, d_o, cu, 0.4)
    assert np.abs(dK - dK2.reshape(-1, 2, 2, 8).sum(axis=2)).max() < 1e-12
    assert np.abs(dV - dV2.reshape(-1, 2, 2, 8).sum(axis=2)).max() < 1e-12


def test_oracle_rejects_bad_arguments():
    q, k, v, d_o, cu = make([8, 8], 2, 2, 4, 4)
    with pytest.raises(ValueError):
        attn_fwd(q, k, v, np.array([0, 9, 8, 16], dtype=np.int32))     # not monotone
    with pytest.raises(ValueError):
        attn_fwd(q, k, v, np.array([0, 8, 15], dtype=np.int32))        # does not end at T
    with pytest.raises(ValueError):
        attn_fwd(q, k, v, cu, rows=[16])
