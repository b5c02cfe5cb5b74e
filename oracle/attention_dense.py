"""fp64 oracle of causal attention over ONE sample, written with matrix products (test infrastructure only).

The same definition as ``attn_oracle.c`` (standard scaled-dot-product softmax attention, causal, inside
one sample of a pack; the paper fixes only that attention is per sample — Section 1, third paragraph —
and what it costs, Appendix D), stated with whole matrices instead of one row at a time so that a BLAS
``matmul`` carries the products and a whole kv group of a 32K-token sample can be checked in under a minute:

    S  = scale Q K^T  (keys k <= r only),   LSE = logsumexp_k S,   P = exp(S - LSE),   O = P V
    D  = rowsum(dO * O),   dP = dO V^T,   dS = P * (dP - D)
    dQ = scale dS K,   dK = scale sum_h dS^T Q,   dV = sum_h P^T dO      (h over the heads of the kv group)

The s x s matrices of a long sample do not fit memory at once, so the rows are taken in consecutive
ranges [a, b): every quantity of a row depends on that row only (and on keys 0..b-1), dK and dV are the
sums of the ranges' contributions.  Nothing else is blocked, no running maximum, no fusion.  fp64
throughout; inputs are float32 arrays holding bf16-representable values.  No code is shared with the HIP
library or with ``attn_oracle.c``; it is pinned on its own in ``tests/test_oracle_attention_dense.py``.
"""
from __future__ import annotations

from typing import Optional

import numpy as np


def _one_head(qh, kh, vh, doh, scale, rows_per_step):
    """All five outputs of one query head on its kv head.  qh [s,d], kh [s,d], vh [s,e], doh [s,e] fp64."""
    s, d = qh.shape
    e = vh.shape[1]
    O = np.empty((s, e))
    LSE = np.empty(s)
    dQ = np.empty((s, d))
    dK = np.zeros((s, d))
    dV = np.zeros((s, e))
    for a in range(0, s, rows_per_step):
        b = min(a + rows_per_step, s)
        S = qh[a:b] @ kh[:b].T                                     # [b-a, b]
        S *= scale
        # key after the query: excluded (only the columns a..b-1 hold such pairs)
        S[:, a:b][np.triu(np.ones((b - a, b - a), dtype=bool), k=1)] = -np.inf
        m = S.max(axis=1, keepdims=True)
        S -= m
        np.exp(S, out=S)
        Z = S.sum(axis=1, keepdims=True)
        P = S
        P /= Z                                                     # exp(S - LSE), LSE = m + ln Z
        o = P @ vh[:b]
        D = (doh[a:b] * o).sum(axis=1, keepdims=True)
        dS = doh[a:b] @ vh[:b].T                                   # dP
        dS -= D
        dS *= P
        O[a:b] = o
        LSE[a:b] = (m + np.log(Z))[:, 0]
        dQ[a:b] = scale * (dS @ kh[:b])
        dK[:b] += scale * (dS.T @ qh[a:b])
        dV[:b] += P.T @ doh[a:b]
    return O, LSE, dQ, dK, dV


def sample_dense(q, k, v, d_o, scale: Optional[float] = None, rows_per_step: int = 512):
    """One sample, any number of kv groups.  q [s,Hq,d], k [s,Hkv,d], v [s,Hkv,e], d_o [s,Hq,e].
    Returns O [s,Hq,e], LSE [Hq,s], dQ [s,Hq,d], dK [s,Hkv,d], dV [s,Hkv,e], all float64.
    The heads are taken one after the other from this one thread (the BLAS underneath may use every core:
    calling a multi-threaded BLAS from several Python threads at once gave wrong products on some hosts)."""
    s, Hq, d = q.shape
    Hkv, e = k.shape[1], v.shape[2]
    assert Hq % Hkv == 0 and k.shape == (s, Hkv, d) and v.shape == (s, Hkv, e) and d_o.shape == (s, Hq, e)
    g = Hq // Hkv
    sc = float(scale) if scale is not None and scale > 0 else 1.0 / float(np.sqrt(d))
    f64 = lambda x, h: np.ascontiguousarray(x[:, h], dtype=np.float64)

    def work(h):
        return _one_head(f64(q, h), f64(k, h // g), f64(v, h // g), f64(d_o, h), sc, rows_per_step)

    res = [work(h) for h in range(Hq)]
    O = np.stack([r[0] for r in res], axis=1)
    LSE = np.stack([r[1] for r in res], axis=0)
    dQ = np.stack([r[2] for r in res], axis=1)
    dK = np.zeros((s, Hkv, d))
    dV = np.zeros((s, Hkv, e))
    for h in range(Hq):                                            # the group's heads in order
        dK[:, h // g] += res[h][3]
        dV[:, h // g] += res[h][4]
    return O, LSE, dQ, dK, dV
