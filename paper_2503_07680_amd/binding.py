"""ctypes marshalling for the C ABI of ``include/hbp.h``.  No arithmetic of the method lives here.

Device buffers are passed as ``torch`` tensors (``data_ptr()``), or as raw integer addresses.
If ``libhbp.so`` is missing the binding raises: there is no CPU fallback.
"""
from __future__ import annotations

import ctypes
import os
from typing import Callable, Optional, Sequence

import numpy as np

HBP_FWD, HBP_BWD, HBP_BWD_DQ = 0, 1, 2
HBP_TILES_QUERY, HBP_TILES_KEY = 0, 1

EXPORTED_SYMBOLS = ["hbp_status_string", "hbp_pack_plan", "hbp_tile_rows", "hbp_fwd_tile_rows", "hbp_workspace_bytes",
                    "hbp_profile_capacity", "hbp_varlen_attn_fwd", "hbp_varlen_attn_bwd", "hbp_varlen_attn_bwd_static",
                    "hbp_set_kernel_events", "hbp_mfma_probe", "hbp_balance_packing",
                    "hbp_packed_ce_workspace_bytes", "hbp_packed_ce", "hbp_auto_select"]

# numpy views of hbp_pack / hbp_batch
PACK_DTYPE = np.dtype([("level", "<i4"), ("first_item", "<i4"), ("n_items", "<i4"), ("n_tokens", "<i4"),
                       ("attn_cost", "<i8")])
BATCH_DTYPE = np.dtype([("level", "<i4"), ("first_pack", "<i4"), ("n_packs", "<i4"), ("reserved", "<i4")])


PROFILE_FN = ctypes.CFUNCTYPE(ctypes.c_double, ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32)


class Profile(ctypes.Structure):
    """Mirror of ``hbp_profile``."""
    _fields_ = [("memory", PROFILE_FN), ("time", PROFILE_FN), ("ctx", ctypes.c_void_p)]


# numpy views of hbp_strategy / hbp_group
STRATEGY_DTYPE = np.dtype([("l", "<i4"), ("sp", "<i4"), ("ckpt", "<i4"), ("feasible", "<i4"), ("time", "<f8")])
GROUP_DTYPE = np.dtype([("l", "<i4"), ("sp", "<i4"), ("ckpt", "<i4"), ("reserved", "<i4")])


class PackMetrics(ctypes.Structure):
    """Mirror of ``hbp_pack_metrics``."""
    _fields_ = [("dbr", ctypes.c_double), ("pr", ctypes.c_double), ("abr", ctypes.c_double),
                ("cr", ctypes.c_double), ("ave_t", ctypes.c_double)]

# numpy view of hbp_profile_rec
PROFILE_DTYPE = np.dtype([("hw_id", "<u4"), ("xcc_id", "<u4"), ("n_items", "<u4"), ("reserved", "<u4"),
                          ("first_tick", "<u8"), ("last_tick", "<u8"), ("busy_ticks", "<u8")])

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "libhbp.so")
_lib = None


class HbpError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = int(status)
        super().__init__("%s: %s (status %d)" % (where, hbp_status_string(status), status))


class AttnDesc(ctypes.Structure):
    """Mirror of ``hbp_attn_desc``."""
    _fields_ = [("total_tokens", ctypes.c_int32), ("n_samples", ctypes.c_int32),
                ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
                ("d_qk", ctypes.c_int32), ("d_v", ctypes.c_int32),
                ("softmax_scale", ctypes.c_float), ("fwd_tile_rows", ctypes.c_int32),
                ("q_stride_t", ctypes.c_int64), ("q_stride_h", ctypes.c_int64),
                ("k_stride_t", ctypes.c_int64), ("k_stride_h", ctypes.c_int64),
                ("v_stride_t", ctypes.c_int64), ("v_stride_h", ctypes.c_int64),
                ("o_stride_t", ctypes.c_int64), ("o_stride_h", ctypes.c_int64)]


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libhbp.so; raises if it has not been built (no fallback path exists).  The environment
    variable HBP_LIBRARY names another build of the same library to load instead (the race-hunting
    build libhbp_racehunt.so, say); it is read once, at the first call."""
    global _lib, _LIB_PATH
    if _lib is not None:
        return _lib
    override = os.environ.get("HBP_LIBRARY")
    if override:
        _LIB_PATH = override if os.path.isabs(override) else os.path.join(_PKG, override)
    if not os.path.exists(_LIB_PATH):
        raise FileNotFoundError(
            "%s not found: build it with `python -m paper_2503_07680_amd.build`" % _LIB_PATH)
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i32, i32p, i64p = ctypes.c_void_p, ctypes.c_int32, ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int64)
    descp = ctypes.POINTER(AttnDesc)
    lib.hbp_status_string.restype = ctypes.c_char_p
    lib.hbp_status_string.argtypes = [i32]
    lib.hbp_pack_plan.restype = i32
    lib.hbp_pack_plan.argtypes = [i32p, i32, i32, i32, i32, i32p, i32, i32p, i32p, vp, i64p, i32, i32p, i64p]
    lib.hbp_tile_rows.restype = i32
    lib.hbp_tile_rows.argtypes = [i32, i32, i32, i32p]
    lib.hbp_fwd_tile_rows.restype = i32
    lib.hbp_fwd_tile_rows.argtypes = [descp, i32p]
    lib.hbp_workspace_bytes.restype = i32
    lib.hbp_workspace_bytes.argtypes = [descp, i32, ctypes.POINTER(ctypes.c_size_t)]
    lib.hbp_profile_capacity.restype = i32
    lib.hbp_profile_capacity.argtypes = [descp, i32, i32p]
    lib.hbp_varlen_attn_fwd.restype = i32
    lib.hbp_varlen_attn_fwd.argtypes = [descp, vp, vp, vp, vp, vp, i32, vp, vp, vp, ctypes.c_size_t, vp, vp]
    lib.hbp_varlen_attn_bwd.restype = i32
    lib.hbp_varlen_attn_bwd.argtypes = [descp, vp, vp, vp, vp, vp, vp, vp, vp, i32, vp, i32, vp, vp, vp, vp,
                                        ctypes.c_size_t, vp, vp, vp]
    lib.hbp_varlen_attn_bwd_static.restype = i32
    lib.hbp_varlen_attn_bwd_static.argtypes = [descp, vp, vp, vp, vp, vp, vp, vp, vp, i32, vp, i32, vp, vp, vp,
                                               vp, vp, vp]
    lib.hbp_set_kernel_events.restype = i32
    lib.hbp_set_kernel_events.argtypes = [i32, vp, vp]
    lib.hbp_balance_packing.restype = i32
    lib.hbp_balance_packing.argtypes = [vp, i32, vp, vp, vp, i32, ctypes.c_uint64, vp, i32, vp, i32, vp,
                                        vp, i32, vp, vp]
    lib.hbp_packed_ce_workspace_bytes.restype = i32
    lib.hbp_packed_ce_workspace_bytes.argtypes = [i32, i32, ctypes.POINTER(ctypes.c_size_t)]
    lib.hbp_packed_ce.restype = i32
    lib.hbp_packed_ce.argtypes = [vp, ctypes.c_int64, i32, i32, vp, vp, i32, i32, ctypes.c_float, vp, vp, vp,
                                  vp, ctypes.c_size_t, vp]
    lib.hbp_mfma_probe.restype = i32
    lib.hbp_mfma_probe.argtypes = [i32, i32, vp, vp]
    lib.hbp_auto_select.restype = i32
    lib.hbp_auto_select.argtypes = [vp, i32, vp, i32, i32, i32, ctypes.POINTER(Profile), vp, vp, i32p, i32p]
    _lib = lib
    return lib


def hbp_status_string(status: int) -> str:
    return load_library().hbp_status_string(int(status)).decode()


def _ptr(x) -> Optional[int]:
    """Device (or host) address of a torch tensor / int / None."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return int(x.data_ptr())


def _nbytes(x) -> int:
    return int(x.numel() * x.element_size())


def hbp_pack_plan(lengths: Sequence[int], pack_len: int, tile_rows: int, kind: int):
    """Returns (cu_seqlens int32[n+1], n_consumed, tiles int32[n_tiles,4], tile_cost int64[n_tiles],
    pack_cost).  Host only."""
    lib = load_library()
    L = np.ascontiguousarray(lengths, dtype=np.int32)
    Lp = L.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)) if L.size else None
    ns, nc, nt = ctypes.c_int32(), ctypes.c_int32(), ctypes.c_int32()
    pc = ctypes.c_int64()
    st = lib.hbp_pack_plan(Lp, int(L.size), int(pack_len), int(tile_rows), int(kind), None, 0,
                           ctypes.byref(ns), ctypes.byref(nc), None, None, 0, ctypes.byref(nt),
                           ctypes.byref(pc))
    if st != 0:
        raise HbpError(st, "hbp_pack_plan")
    cu = np.zeros(ns.value + 1, dtype=np.int32)
    tiles = np.zeros((nt.value, 4), dtype=np.int32)
    cost = np.zeros(nt.value, dtype=np.int64)
    st = lib.hbp_pack_plan(Lp, int(L.size), int(pack_len), int(tile_rows), int(kind),
                           cu.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), cu.size,
                           ctypes.byref(ns), ctypes.byref(nc), tiles.ctypes.data,
                           cost.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)), nt.value,
                           ctypes.byref(nt), ctypes.byref(pc))
    if st != 0:
        raise HbpError(st, "hbp_pack_plan")
    return cu, int(nc.value), tiles, cost, int(pc.value)


def hbp_balance_packing(lengths: Sequence[int], group_lens: Sequence[int], packs_per_batch: Sequence[int],
                        level_sp: Optional[Sequence[int]] = None, shuffle_seed: int = 0, lists: bool = True):
    """The multi-level Balance Packing planner.  Returns (batches BATCH_DTYPE[nb], packs PACK_DTYPE[np],
    pack_items int32[n_samples], metrics dict); with lists=False only the counts and metrics:
    (n_batches, n_packs, None, metrics).  Host only."""
    lib = load_library()
    L = np.ascontiguousarray(lengths, dtype=np.int32)
    G = np.ascontiguousarray(group_lens, dtype=np.int32)
    B = np.ascontiguousarray(packs_per_batch, dtype=np.int32)
    S = None if level_sp is None else np.ascontiguousarray(level_sp, dtype=np.int32)
    if B.size != G.size or (S is not None and S.size != G.size):
        raise HbpError(1, "hbp_balance_packing")
    n_p, n_b = ctypes.c_int32(), ctypes.c_int32()
    m = PackMetrics()
    ptr = lambda a: a.ctypes.data if a is not None and a.size else None
    args = (ptr(L), int(L.size), ptr(G), ptr(B), ptr(S), int(G.size), int(shuffle_seed) & (2 ** 64 - 1))
    st = lib.hbp_balance_packing(*args, None, 0, None, 0, ctypes.byref(n_p), None, 0, ctypes.byref(n_b),
                                 ctypes.byref(m))
    if st != 0:
        raise HbpError(st, "hbp_balance_packing")
    metrics = {"DBR": m.dbr, "PR": m.pr, "ABR": m.abr, "CR": m.cr, "AveT": m.ave_t}
    if not lists:
        return int(n_b.value), int(n_p.value), None, metrics
    items = np.zeros(max(int(L.size), 1), dtype=np.int32)
    packs = np.zeros(max(n_p.value, 1), dtype=PACK_DTYPE)
    batches = np.zeros(max(n_b.value, 1), dtype=BATCH_DTYPE)
    st = lib.hbp_balance_packing(*args, items.ctypes.data, int(L.size), packs.ctypes.data, n_p.value,
                                 ctypes.byref(n_p), batches.ctypes.data, n_b.value, ctypes.byref(n_b), None)
    if st != 0:
        raise HbpError(st, "hbp_balance_packing")
    return batches[:n_b.value], packs[:n_p.value], items[:L.size], metrics


def hbp_auto_select(lengths: Sequence[int], sp_set: Sequence[int], c_min: int, c_max: int,
                    profile_memory: Callable, profile_time: Callable):
    """Hierarchical Groups Auto-Selection.  ``profile_memory(l, sp, ckpt)`` returns the remaining memory
    (negative: does not fit), ``profile_time(l, sp, ckpt)`` the iteration time (None/inf: cannot run).
    Returns (groups GROUP_DTYPE[n], per_length STRATEGY_DTYPE[len(lengths)], best_index).  Host only."""
    lib = load_library()
    L = np.ascontiguousarray(lengths, dtype=np.int32)
    S = np.ascontiguousarray(sp_set, dtype=np.int32)

    def mem(_ctx, l, sp, c):
        return float(profile_memory(l, sp, c))

    def tim(_ctx, l, sp, c):
        t = profile_time(l, sp, c)
        return float("inf") if t is None else float(t)

    prof = Profile(PROFILE_FN(mem), PROFILE_FN(tim), None)
    per = np.zeros(max(int(L.size), 1), dtype=STRATEGY_DTYPE)
    groups = np.zeros(4, dtype=GROUP_DTYPE)
    n, j = ctypes.c_int32(), ctypes.c_int32(-1)
    st = lib.hbp_auto_select(L.ctypes.data if L.size else None, int(L.size), S.ctypes.data if S.size else None,
                             int(S.size), int(c_min), int(c_max), ctypes.byref(prof), per.ctypes.data,
                             groups.ctypes.data, ctypes.byref(n), ctypes.byref(j))
    if st != 0:
        raise HbpError(st, "hbp_auto_select")
    return groups[:n.value], per[:L.size], int(j.value)


def hbp_tile_rows(d_qk: int, d_v: int, which: int) -> int:
    out = ctypes.c_int32()
    st = load_library().hbp_tile_rows(int(d_qk), int(d_v), int(which), ctypes.byref(out))
    if st != 0:
        raise HbpError(st, "hbp_tile_rows")
    return int(out.value)


def hbp_fwd_tile_rows(desc: AttnDesc) -> int:
    """Preferred rows per query tile of the forward's list for this head layout."""
    out = ctypes.c_int32()
    st = load_library().hbp_fwd_tile_rows(ctypes.byref(desc), ctypes.byref(out))
    if st != 0:
        raise HbpError(st, "hbp_fwd_tile_rows")
    return int(out.value)


def hbp_workspace_bytes(desc: AttnDesc, which: int) -> int:
    out = ctypes.c_size_t()
    st = load_library().hbp_workspace_bytes(ctypes.byref(desc), int(which), ctypes.byref(out))
    if st != 0:
        raise HbpError(st, "hbp_workspace_bytes")
    return int(out.value)


def hbp_profile_capacity(desc: AttnDesc, which: int) -> int:
    out = ctypes.c_int32()
    st = load_library().hbp_profile_capacity(ctypes.byref(desc), int(which), ctypes.byref(out))
    if st != 0:
        raise HbpError(st, "hbp_profile_capacity")
    return int(out.value)


def hbp_varlen_attn_fwd(desc: AttnDesc, q, k, v, cu_seqlens, q_tiles, n_q_tiles: int, o, lse,
                        workspace, profile=None, stream: Optional[int] = None) -> None:
    """Enqueue the forward on ``stream`` (a raw hipStream_t handle, None = default stream)."""
    st = load_library().hbp_varlen_attn_fwd(
        ctypes.byref(desc), _ptr(q), _ptr(k), _ptr(v), _ptr(cu_seqlens), _ptr(q_tiles), int(n_q_tiles),
        _ptr(o), _ptr(lse), _ptr(workspace), 0 if workspace is None else _nbytes(workspace),
        _ptr(profile), stream)
    if st != 0:
        raise HbpError(st, "hbp_varlen_attn_fwd")


def hbp_varlen_attn_bwd(desc: AttnDesc, q, k, v, o, lse, d_o, cu_seqlens, q_tiles, n_q_tiles: int,
                        kv_tiles, n_kv_tiles: int, dq, dk, dv, workspace, profile=None, profile_dq=None,
                        stream: Optional[int] = None) -> None:
    """Enqueue the backward (prepass, dK/dV kernel, dQ kernel) on ``stream``."""
    st = load_library().hbp_varlen_attn_bwd(
        ctypes.byref(desc), _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), _ptr(d_o), _ptr(cu_seqlens),
        _ptr(q_tiles), int(n_q_tiles), _ptr(kv_tiles), int(n_kv_tiles), _ptr(dq), _ptr(dk), _ptr(dv),
        _ptr(workspace), 0 if workspace is None else _nbytes(workspace), _ptr(profile), _ptr(profile_dq),
        stream)
    if st != 0:
        raise HbpError(st, "hbp_varlen_attn_bwd")


HBP_STATIC_SCRATCH_BYTES = (64 << 20) + 4096
HBP_ERR_STATIC_LIMIT = 8


def hbp_varlen_attn_bwd_static(desc: AttnDesc, q, k, v, o, lse, d_o, cu_seqlens, q_tiles, n_q_tiles: int,
                               kv_tiles, n_kv_tiles: int, dq, dk, dv, profile=None, profile_dq=None,
                               stream: Optional[int] = None) -> None:
    """The backward with the library's static scratch array in place of a workspace (allocates nothing)."""
    st = load_library().hbp_varlen_attn_bwd_static(
        ctypes.byref(desc), _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), _ptr(d_o), _ptr(cu_seqlens),
        _ptr(q_tiles), int(n_q_tiles), _ptr(kv_tiles), int(n_kv_tiles), _ptr(dq), _ptr(dk), _ptr(dv),
        _ptr(profile), _ptr(profile_dq), stream)
    if st != 0:
        raise HbpError(st, "hbp_varlen_attn_bwd_static")


HBP_LOSS_TOKEN_MEAN, HBP_LOSS_SAMPLE_MEAN, HBP_LOSS_STABLE = 0, 1, 2
HBP_LOSS = 3


def hbp_packed_ce_workspace_bytes(total_tokens: int, n_samples: int) -> int:
    out = ctypes.c_size_t()
    st = load_library().hbp_packed_ce_workspace_bytes(int(total_tokens), int(n_samples), ctypes.byref(out))
    if st != 0:
        raise HbpError(st, "hbp_packed_ce_workspace_bytes")
    return int(out.value)


def hbp_packed_ce(logits, logit_stride_t: int, total_tokens: int, vocab: int, labels, cu_seqlens,
                  n_samples: int, normalizer: int, t_ave: float, dlogits, loss_out, token_loss, workspace,
                  stream=None) -> None:
    """Device pointers (torch tensors or ints); see include/hbp.h."""
    st = load_library().hbp_packed_ce(_ptr(logits), int(logit_stride_t), int(total_tokens), int(vocab),
                                      _ptr(labels), _ptr(cu_seqlens), int(n_samples), int(normalizer),
                                      float(t_ave), _ptr(dlogits), _ptr(loss_out), _ptr(token_loss),
                                      _ptr(workspace), _nbytes(workspace) if workspace is not None else 0,
                                      _ptr(stream))
    if st != 0:
        raise HbpError(st, "hbp_packed_ce")


def hbp_mfma_probe(n_cu: int, mfma_per_wave: int, sink, stream=None) -> None:
    """Launch the MFMA-only probe kernel (n_cu workgroups of 8 waves); the caller times it."""
    st = load_library().hbp_mfma_probe(int(n_cu), int(mfma_per_wave), _ptr(sink), _ptr(stream))
    if st != 0:
        raise HbpError(st, "hbp_mfma_probe")


def hbp_set_kernel_events(which: int, start_event: Optional[int], stop_event: Optional[int]) -> None:
    """Raw hipEvent_t handles (ints) recorded around the main kernel of later calls; None = off."""
    st = load_library().hbp_set_kernel_events(int(which), start_event, stop_event)
    if st != 0:
        raise HbpError(st, "hbp_set_kernel_events")
