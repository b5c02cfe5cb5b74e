"""Seeded synthetic workloads for packed varlen attention.

This module only *draws inputs*: sample-length lists and random bf16 tensors.  It holds
none of the method's arithmetic (no attention, no planning, no cost model), so both the
CPU oracle's tests and the HIP path's tests can feed from it without sharing any code
that is under test.

The five workloads stand in for the paper's hybrid short/long SFT data (Section 5.1:
a <=32K instruction set mixed with a <=128K long-context set): many short samples and a
few very long ones share one packed buffer.  Only the *length structure* is imitated,
through lognormal draws; no item of any dataset is reproduced.

Recipe
------
lengths : ``numpy.random.default_rng(seed)``; each draw is
          ``clip(rint(exp(normal(ln median, sigma))), lo, hi)``; draws continue until
          their running sum reaches ``pack_len`` (the planner truncates the last one).
tensors : tensor ``X[T, H, dim]`` is drawn head by head so that any subset of heads can be
          regenerated alone: head ``h`` of tensor number ``t`` (Q=0, K=1, V=2, dO=3) comes
          from ``default_rng([1000 + seed, t, h]).standard_normal((T, dim), float32) * sigma``
          and is then rounded to bf16 (round to nearest even).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Sequence

import numpy as np

TENSOR_ID = {"q": 0, "k": 1, "v": 2, "do": 3}


@dataclass(frozen=True)
class Workload:
    name: str
    lengths: tuple          # candidate sample lengths handed to the planner, in order
    pack_len: int
    n_q_heads: int
    n_kv_heads: int
    d_qk: int
    d_v: int
    sigma: float = 1.0
    seed: int = 0
    note: str = ""

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads


def lognormal_lengths(seed: int, median: float, sigma: float, lo: int, hi: int,
                      pack_len: int, first: Sequence[int] = ()) -> List[int]:
    """Draw sample lengths one at a time until they fill ``pack_len`` tokens."""
    rng = np.random.default_rng(seed)
    out = [int(x) for x in first]
    total = sum(out)
    mu = float(np.log(median))
    while total < pack_len:
        x = rng.normal(mu, sigma)
        n = int(np.clip(np.rint(np.exp(x)), lo, hi))
        out.append(n)
        total += n
    return out


def workload(index: int, seed: int = 0) -> Workload:
    """The five benchmark packs, numbered 1..5."""
    if index == 1:
        return Workload("tiny-1k", (512, 256, 128, 64, 64), 1024, 4, 4, 64, 64, 1.0, seed,
                        "5 samples, MHA, head_dim 64")
    if index == 2:
        L = lognormal_lengths(seed, 400, 1.0, 16, 4096, 8192)
        return Workload("short-heavy-8k", tuple(L), 8192, 32, 8, 128, 128, 1.0, seed,
                        "lognormal(400, 1.0) clipped [16,4096], GQA 32/8")
    if index == 3:
        L = lognormal_lengths(seed, 600, 1.2, 16, 4096, 32768, first=(16384,))
        return Workload("mixed-32k", tuple(L), 32768, 32, 8, 128, 128, 1.0, seed,
                        "one 16384 sample + lognormal(600, 1.2) clipped [16,4096], GQA 32/8")
    if index == 4:
        return Workload("long-128k", (98304, 32768), 131072, 64, 8, 128, 128, 0.5, seed,
                        "98304 + 32768, GQA 64/8, inputs N(0, 0.5)")
    if index == 5:
        L = lognormal_lengths(seed, 1000, 1.3, 32, 8192, 32768)
        return Workload("mla-32k", tuple(L), 32768, 128, 128, 192, 128, 1.0, seed,
                        "lognormal(1000, 1.3) clipped [32,8192], 128 heads, d_qk 192, d_v 128")
    raise ValueError("workload index must be 1..5")


# ----------------------------------------------------------------------------- bf16

def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns (uint16), round to nearest even.  Finite inputs only."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + bias) >> 16).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> the float32 with exactly that value."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def head_tensor(seed: int, which: str, head: int, n_tokens: int, dim: int,
                sigma: float = 1.0) -> np.ndarray:
    """One head ``[n_tokens, dim]`` of tensor ``which`` as bf16 bit patterns (uint16)."""
    rng = np.random.default_rng([1000 + seed, TENSOR_ID[which], head])
    x = rng.standard_normal((n_tokens, dim), dtype=np.float32)
    if sigma != 1.0:
        x *= np.float32(sigma)
    return f32_to_bf16_bits(x)


def tensor_bits(seed: int, which: str, n_tokens: int, n_heads: int, dim: int,
                sigma: float = 1.0, heads: Sequence[int] | None = None) -> np.ndarray:
    """Tensor ``[n_tokens, len(heads), dim]`` of bf16 bit patterns (all heads by default)."""
    hs = list(range(n_heads)) if heads is None else list(heads)
    out = np.empty((n_tokens, len(hs), dim), dtype=np.uint16)
    for j, h in enumerate(hs):
        out[:, j, :] = head_tensor(seed, which, h, n_tokens, dim, sigma)
    return out


def workload_dims(w: Workload, which: str):
    """(n_heads, dim) of tensor ``which`` for workload ``w``."""
    return {"q": (w.n_q_heads, w.d_qk), "k": (w.n_kv_heads, w.d_qk),
            "v": (w.n_kv_heads, w.d_v), "do": (w.n_q_heads, w.d_v)}[which]


def workload_tensor_bits(w: Workload, which: str, n_tokens: int,
                         heads: Sequence[int] | None = None) -> np.ndarray:
    nh, dim = workload_dims(w, which)
    return tensor_bits(w.seed, which, n_tokens, nh, dim, w.sigma, heads)
