"""Plumbing around the C ABI: torch device buffers for one pack, plan upload, fwd/bwd calls.

Holds no arithmetic: planning happens in ``hbp_pack_plan`` and all attention math in the HIP
kernels.  Used by the tests, the smoke check and the benchmark.
"""
from __future__ import annotations

from typing import Optional, Sequence

import numpy as np
import torch

from . import binding as B


class PackedAttention:
    """One packed buffer: plan on the host, buffers on ``cuda:0``, kernels through the C ABI."""

    def __init__(self, lengths: Sequence[int], pack_len: int, n_q_heads: int, n_kv_heads: int,
                 d_qk: int, d_v: int, softmax_scale: float = 0.0, device: str = "cuda:0",
                 with_profile: bool = False, fwd_tile_rows: Optional[int] = None, row_pad: int = 0):
        if not torch.cuda.is_available():
            raise RuntimeError("PackedAttention needs a GPU: there is no CPU fallback")
        B.load_library()
        self.device = torch.device(device)
        self.rows_fwd = B.hbp_tile_rows(d_qk, d_v, B.HBP_FWD)
        self.rows_bwd = B.hbp_tile_rows(d_qk, d_v, B.HBP_BWD)
        self.cu, self.n_consumed, self.q_tiles, self.q_cost, self.pack_cost = B.hbp_pack_plan(
            lengths, pack_len, self.rows_fwd, B.HBP_TILES_QUERY)
        # the forward's own list when the head layout prefers larger query tiles (odd group sizes)
        self.rows_fwd_pref = B.hbp_fwd_tile_rows(B.AttnDesc(n_q_heads=n_q_heads, n_kv_heads=n_kv_heads,
                                                            d_qk=d_qk, d_v=d_v))
        self.fwd_tiles, self.fwd_cost = self.q_tiles, self.q_cost
        if fwd_tile_rows is None:
            fwd_tile_rows = self.rows_fwd_pref
        if fwd_tile_rows != self.rows_fwd:
            _, _, self.fwd_tiles, self.fwd_cost, _ = B.hbp_pack_plan(lengths, pack_len, fwd_tile_rows,
                                                                     B.HBP_TILES_QUERY)
        _, _, self.kv_tiles, self.kv_cost, _ = B.hbp_pack_plan(
            lengths, pack_len, self.rows_bwd, B.HBP_TILES_KEY)
        self.T = int(self.cu[-1])
        self.n_samples = len(self.cu) - 1
        self.Hq, self.Hkv, self.d_qk, self.d_v = n_q_heads, n_kv_heads, d_qk, d_v
        self.desc = B.AttnDesc(total_tokens=self.T, n_samples=self.n_samples, n_q_heads=n_q_heads,
                               n_kv_heads=n_kv_heads, d_qk=d_qk, d_v=d_v,
                               softmax_scale=float(softmax_scale),
                               fwd_tile_rows=0 if fwd_tile_rows == self.rows_fwd else int(fwd_tile_rows))
        # row_pad: extra elements (a multiple of 8) at the end of every token row of every tensor, so that
        # the row stride is not a power of two; 0 = dense [T, H, dim]
        self.row_pad = int(row_pad)
        if self.row_pad:
            self.desc.q_stride_t = n_q_heads * d_qk + self.row_pad
            self.desc.k_stride_t = n_kv_heads * d_qk + self.row_pad
            self.desc.v_stride_t = n_kv_heads * d_v + self.row_pad
            self.desc.o_stride_t = n_q_heads * d_v + self.row_pad
        dev = self.device
        self.cu_dev = torch.from_numpy(self.cu).to(dev)
        self.q_tiles_dev = torch.from_numpy(self.q_tiles).to(dev)
        self.fwd_tiles_dev = (self.q_tiles_dev if self.fwd_tiles is self.q_tiles
                              else torch.from_numpy(self.fwd_tiles).to(dev))
        self.kv_tiles_dev = torch.from_numpy(self.kv_tiles).to(dev)
        self.ws_fwd = torch.empty(B.hbp_workspace_bytes(self.desc, B.HBP_FWD), dtype=torch.uint8, device=dev)
        self.ws_bwd = None
        self.prof_fwd = self.prof_bwd = self.prof_dq = None
        if with_profile:
            n = B.hbp_profile_capacity(self.desc, B.HBP_FWD)
            self.prof_fwd = torch.zeros(n * B.PROFILE_DTYPE.itemsize, dtype=torch.uint8, device=dev)
            n = B.hbp_profile_capacity(self.desc, B.HBP_BWD)
            self.prof_bwd = torch.zeros(n * B.PROFILE_DTYPE.itemsize, dtype=torch.uint8, device=dev)
            n = B.hbp_profile_capacity(self.desc, B.HBP_BWD_DQ)
            self.prof_dq = torch.zeros(n * B.PROFILE_DTYPE.itemsize, dtype=torch.uint8, device=dev)
        T = max(self.T, 1)
        bf = torch.bfloat16
        self.o = self.buffer(n_q_heads, d_v)
        self.lse = torch.zeros((n_q_heads, T), dtype=torch.float32, device=dev)
        self.dq = self.dk = self.dv = None

    # -- buffers ------------------------------------------------------------------------------
    def buffer(self, heads: int, dim: int) -> torch.Tensor:
        """Zeroed bf16 [T, heads, dim] tensor in this object's row layout (a view when rows are padded)."""
        T = max(self.T, 1)
        if not self.row_pad:
            return torch.zeros((T, heads, dim), dtype=torch.bfloat16, device=self.device)
        base = torch.zeros((T, heads * dim + self.row_pad), dtype=torch.bfloat16, device=self.device)
        return base[:, :heads * dim].view(T, heads, dim)

    # -- inputs -------------------------------------------------------------------------------
    def to_device_bf16(self, bits: np.ndarray) -> torch.Tensor:
        """uint16 bf16 bit patterns [T,H,dim] -> bf16 tensor on the device."""
        t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(self.device).view(torch.bfloat16)
        if not self.row_pad:
            return t
        out = self.buffer(t.shape[1], t.shape[2])
        out.copy_(t)
        return out

    # -- calls --------------------------------------------------------------------------------
    def _stream(self) -> int:
        return int(torch.cuda.current_stream(self.device).cuda_stream)

    def forward(self, q, k, v, profile: bool = False):
        B.hbp_varlen_attn_fwd(self.desc, q, k, v, self.cu_dev, self.fwd_tiles_dev, len(self.fwd_tiles),
                              self.o, self.lse, self.ws_fwd, self.prof_fwd if profile else None,
                              self._stream())
        return self.o, self.lse

    def alloc_backward(self):
        if self.ws_bwd is None:
            dev, bf, T = self.device, torch.bfloat16, max(self.T, 1)
            self.ws_bwd = torch.empty(B.hbp_workspace_bytes(self.desc, B.HBP_BWD), dtype=torch.uint8, device=dev)
            self.dq = self.buffer(self.Hq, self.d_qk)
            self.dk = self.buffer(self.Hkv, self.d_qk)
            self.dv = self.buffer(self.Hkv, self.d_v)

    def backward(self, q, k, v, d_o, profile: bool = False):
        self.alloc_backward()
        B.hbp_varlen_attn_bwd(self.desc, q, k, v, self.o, self.lse, d_o, self.cu_dev,
                              self.q_tiles_dev, len(self.q_tiles), self.kv_tiles_dev, len(self.kv_tiles),
                              self.dq, self.dk, self.dv, self.ws_bwd,
                              self.prof_bwd if profile else None, self.prof_dq if profile else None,
                              self._stream())
        return self.dq, self.dk, self.dv

    def profile_records(self, which: int) -> np.ndarray:
        buf = {B.HBP_FWD: self.prof_fwd, B.HBP_BWD: self.prof_bwd, B.HBP_BWD_DQ: self.prof_dq}[which]
        return np.frombuffer(buf.cpu().numpy().tobytes(), dtype=B.PROFILE_DTYPE)


def bf16_tensor_to_f32_numpy(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy()
