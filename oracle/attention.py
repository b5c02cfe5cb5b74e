"""ctypes front end of ``attn_oracle.c`` (fp64 CPU oracle; test infrastructure only).

All tensor arguments are numpy float32 arrays holding bf16-representable values
(``Q [T,Hq,d]``, ``K [T,Hkv,d]``, ``V [T,Hkv,e]``, ``dO [T,Hq,e]``); results are float64.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "attn_oracle.c")
_LIB = os.path.join(_HERE, "libhbp_oracle.so")
_lib = None


def build_oracle(force: bool = False) -> str:
    """Compile the C oracle with gcc (plain -O2, OpenMP, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build_oracle())
    return _lib


def oracle_threads() -> int:
    return int(_load().hbp_oracle_threads())


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def _i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def _f64out(shape):
    a = np.zeros(shape, dtype=np.float64)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _dims(q, k, v, cu):
    T, Hq, d = q.shape
    Tk, Hkv, dk = k.shape
    Tv, Hkv2, e = v.shape
    assert T == Tk == Tv and d == dk and Hkv == Hkv2, "inconsistent Q/K/V shapes"
    n = len(cu) - 1
    return T, Hq, Hkv, d, e, n


def _scale(scale, d):
    return float(scale) if scale is not None and scale > 0 else 1.0 / float(np.sqrt(d))


def _check(rc, name):
    if rc != 0:
        raise ValueError("%s: oracle rejected its arguments (code %d)" % (name, rc))


def attn_fwd(q, k, v, cu_seqlens, scale: Optional[float] = None,
             rows: Optional[Sequence[int]] = None):
    """O ``[n_rows,Hq,e]`` and LSE ``[Hq,n_rows]`` (natural log of the scaled scores)."""
    q, qp = _f32(q); k, kp = _f32(k); v, vp = _f32(v); cu, cup = _i32(cu_seqlens)
    T, Hq, Hkv, d, e, n = _dims(q, k, v, cu)
    if rows is None:
        rp, nr = None, T
    else:
        rows, rp = _i32(rows); nr = len(rows)
    O, Op = _f64out((nr, Hq, e)); L, Lp = _f64out((Hq, nr))
    rc = _load().hbp_oracle_fwd(qp, kp, vp, cup, n, T, Hq, Hkv, d, e,
                                ctypes.c_double(_scale(scale, d)), rp, nr, Op, Lp)
    _check(rc, "attn_fwd")
    return O, L


def attn_bwd_dq(q, k, v, d_o, cu_seqlens, scale: Optional[float] = None,
                rows: Optional[Sequence[int]] = None, return_D: bool = False):
    """dQ ``[n_rows,Hq,d]`` (and optionally D ``[Hq,n_rows]``) for L = sum(O * dO)."""
    q, qp = _f32(q); k, kp = _f32(k); v, vp = _f32(v); d_o, dop = _f32(d_o)
    cu, cup = _i32(cu_seqlens)
    T, Hq, Hkv, d, e, n = _dims(q, k, v, cu)
    assert d_o.shape == (T, Hq, e)
    if rows is None:
        rp, nr = None, T
    else:
        rows, rp = _i32(rows); nr = len(rows)
    dQ, dQp = _f64out((nr, Hq, d)); D, Dp = _f64out((Hq, nr))
    rc = _load().hbp_oracle_bwd_dq(qp, kp, vp, dop, cup, n, T, Hq, Hkv, d, e,
                                   ctypes.c_double(_scale(scale, d)), rp, nr, dQp, Dp)
    _check(rc, "attn_bwd_dq")
    return (dQ, D) if return_D else dQ


def attn_bwd_dkdv(q, k, v, d_o, cu_seqlens, scale: Optional[float] = None,
                  cols: Optional[Sequence[int]] = None):
    """dK ``[n_cols,Hkv,d]`` and dV ``[n_cols,Hkv,e]`` for L = sum(O * dO)."""
    q, qp = _f32(q); k, kp = _f32(k); v, vp = _f32(v); d_o, dop = _f32(d_o)
    cu, cup = _i32(cu_seqlens)
    T, Hq, Hkv, d, e, n = _dims(q, k, v, cu)
    assert d_o.shape == (T, Hq, e)
    if cols is None:
        cp, nc = None, T
    else:
        cols, cp = _i32(cols); nc = len(cols)
    dK, dKp = _f64out((nc, Hkv, d)); dV, dVp = _f64out((nc, Hkv, e))
    rc = _load().hbp_oracle_bwd_dkdv(qp, kp, vp, dop, cup, n, T, Hq, Hkv, d, e,
                                     ctypes.c_double(_scale(scale, d)), cp, nc, dKp, dVp)
    _check(rc, "attn_bwd_dkdv")
    return dK, dV


def prob_row(q, k, v, cu_seqlens, h: int, r: int, scale: Optional[float] = None):
    """Softmax probabilities of packed row ``r``, head ``h`` over its sample's keys <= r."""
    q, qp = _f32(q); k, kp = _f32(k); v, vp = _f32(v); cu, cup = _i32(cu_seqlens)
    T, Hq, Hkv, d, e, n = _dims(q, k, v, cu)
    P, Pp = _f64out((T,))
    ln = ctypes.c_int(0)
    rc = _load().hbp_oracle_prob_row(qp, kp, vp, cup, n, T, Hq, Hkv, d, e,
                                     ctypes.c_double(_scale(scale, d)), int(h), int(r), Pp,
                                     ctypes.byref(ln))
    _check(rc, "prob_row")
    return P[: ln.value].copy()
