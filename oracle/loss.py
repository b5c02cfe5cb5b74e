"""fp64 oracle of the packed cross-entropy with the paper's loss normalisers (test infrastructure only).

Section 4.3, "Stable Loss Normalizer" (normaliser equation):
    L_token  = sum_i loss_i / sum_i T_i
    L_sample = (sum_i loss_i / T_i) / B_l
    L_stable = sum_i loss_i / (B_l * T_ave),   T_ave = sum over the GLOBAL batch of T_i / B_g
with loss_i the summed token cross-entropy of batch element i and T_i its number of loss tokens.
Reading: a batch element is one sample of the pack (rows cu[i] .. cu[i+1]), B_l the number of
samples of the pack, tokens whose label lies outside [0, V) (negative, or >= the vocabulary size)
carry no loss and are not counted in T_i, a sample without loss tokens contributes nothing (its
1/T_i term is dropped).

Plain numpy, one row at a time, the textbook definition
    CE(row) = logsumexp(z) - z[label],   d CE / d z = softmax(z) - onehot(label).
No code is shared with the GPU path.
"""
from __future__ import annotations

import numpy as np

TOKEN_MEAN, SAMPLE_MEAN, STABLE = 0, 1, 2


def token_weights(labels, cu_seqlens, normalizer: int, t_ave: float = 0.0, vocab=None) -> np.ndarray:
    """Weight of every token's cross-entropy in the loss, fp64 [T].  vocab: the vocabulary size V
    (labels >= V carry no loss); None: every non-negative label counts."""
    labels = np.asarray(labels)
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    n = len(cu) - 1
    w = np.zeros(len(labels), dtype=np.float64)
    valid = labels >= 0
    if vocab is not None:
        valid = valid & (labels < int(vocab))
    counts = [int(valid[cu[i]:cu[i + 1]].sum()) for i in range(n)]
    for i in range(n):
        rows = slice(cu[i], cu[i + 1])
        if normalizer == TOKEN_MEAN:
            wi = 1.0 / sum(counts) if sum(counts) else 0.0
        elif normalizer == SAMPLE_MEAN:
            wi = 1.0 / (counts[i] * n) if counts[i] else 0.0
        elif normalizer == STABLE:
            wi = 1.0 / (n * t_ave)
        else:
            raise ValueError("bad normalizer")
        w[rows] = np.where(valid[rows], wi, 0.0)
    return w


def packed_ce(logits, labels, cu_seqlens, normalizer: int, t_ave: float = 0.0):
    """Returns (loss, token_loss fp64 [T] (0 where no label), dlogits fp64 [T, V])."""
    z = np.asarray(logits, dtype=np.float64)
    labels = np.asarray(labels)
    T, V = z.shape
    w = token_weights(labels, cu_seqlens, normalizer, t_ave, vocab=V)
    token_loss = np.zeros(T, dtype=np.float64)
    dz = np.zeros((T, V), dtype=np.float64)
    for r in range(T):
        y = int(labels[r])
        if y < 0 or y >= V:          # no loss on this token: zero loss, zero gradient row
            continue
        m = z[r].max()
        e = np.exp(z[r] - m)
        s = e.sum()
        token_loss[r] = m + np.log(s) - z[r, y]
        p = e / s
        p[y] -= 1.0
        dz[r] = w[r] * p
    return float((w * token_loss).sum()), token_loss, dz
