"""ctypes front end of the fp64 CPU oracle (oracle/fmha_oracle.c).

TEST INFRASTRUCTURE ONLY: tests, the smoke check and the benchmark's
cpu_baseline leg may import this; the HIP library and its binding never do.

The functions take float64 numpy arrays shaped [T, H, D] (packed tokens, see
Section IV-A-1 of the paper for the layout) and the int32 prefix-sum array.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fmha_oracle.c")
_LIB = os.path.join(_HERE, "libfmha_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
                               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int32)
        lib.oracle_fmha_varlen_fwd.argtypes = [dp, dp, dp, ip, ip, ctypes.c_int, ctypes.c_int,
                                               ctypes.c_int, ctypes.c_double, dp, dp]
        lib.oracle_fmha_varlen_fwd.restype = ctypes.c_int
        lib.oracle_fmha_varlen_bwd.argtypes = [dp, dp, dp, dp, ip, ip, ctypes.c_int, ctypes.c_int,
                                               ctypes.c_int, ctypes.c_double, dp, dp, dp]
        lib.oracle_fmha_varlen_bwd.restype = ctypes.c_int
        bp = ctypes.POINTER(ctypes.c_uint8)
        lp = ctypes.POINTER(ctypes.c_int64)
        lib.oracle_fmha_varlen_fwd_dropout.argtypes = [dp, dp, dp, ip, ip, ctypes.c_int, ctypes.c_int,
                                                       ctypes.c_int, ctypes.c_double, bp, lp,
                                                       ctypes.c_double, dp, dp]
        lib.oracle_fmha_varlen_fwd_dropout.restype = ctypes.c_int
        lib.oracle_fmha_varlen_bwd_dropout.argtypes = [dp, dp, dp, dp, ip, ip, ctypes.c_int,
                                                       ctypes.c_int, ctypes.c_int, ctypes.c_double,
                                                       bp, lp, ctypes.c_double, dp, dp, dp]
        lib.oracle_fmha_varlen_bwd_dropout.restype = ctypes.c_int
        lib.oracle_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def _d(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _i(a):
    return None if a is None else a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def _prep(x):
    x = np.ascontiguousarray(x, dtype=np.float64)
    assert x.ndim == 3
    return x


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def fwd(q, k, v, cu_seqlens, scale, seqused=None):
    """Returns (O [T,H,D] float64, LSE [H,T] float64)."""
    q, k, v = _prep(q), _prep(k), _prep(v)
    assert q.shape == k.shape == v.shape
    cu = np.ascontiguousarray(cu_seqlens, dtype=np.int32)
    su = None if seqused is None else np.ascontiguousarray(seqused, dtype=np.int32)
    t, h, d = q.shape
    assert cu[-1] == t
    o = np.zeros_like(q)
    lse = np.zeros((h, t), dtype=np.float64)
    rc = _load().oracle_fmha_varlen_fwd(_d(q), _d(k), _d(v), _i(cu), _i(su), len(cu) - 1, h, d,
                                        float(scale), _d(o), _d(lse))
    if rc:
        raise ValueError("oracle_fmha_varlen_fwd: bad arguments")
    return o, lse


def bwd(q, k, v, d_o, cu_seqlens, scale, seqused=None):
    """Returns (dQ, dK, dV), each [T,H,D] float64."""
    q, k, v, d_o = _prep(q), _prep(k), _prep(v), _prep(d_o)
    assert q.shape == k.shape == v.shape == d_o.shape
    cu = np.ascontiguousarray(cu_seqlens, dtype=np.int32)
    su = None if seqused is None else np.ascontiguousarray(seqused, dtype=np.int32)
    t, h, d = q.shape
    assert cu[-1] == t
    dq, dk, dv = np.zeros_like(q), np.zeros_like(q), np.zeros_like(q)
    rc = _load().oracle_fmha_varlen_bwd(_d(q), _d(k), _d(v), _d(d_o), _i(cu), _i(su),
                                        len(cu) - 1, h, d, float(scale), _d(dq), _d(dk), _d(dv))
    if rc:
        raise ValueError("oracle_fmha_varlen_bwd: bad arguments")
    return dq, dk, dv


def _flatten_masks(masks, cu, heads):
    """Per-sequence [H, L, L] keep masks -> one byte array + the offset of each sequence."""
    off = np.zeros(len(masks) + 1, dtype=np.int64)
    for i, m in enumerate(masks):
        n = int(cu[i + 1] - cu[i])
        assert m.shape == (heads, n, n), "mask of sequence %d must be [heads, L, L]" % i
        off[i + 1] = off[i] + m.size
    flat = np.zeros(max(int(off[-1]), 1), dtype=np.uint8)
    for i, m in enumerate(masks):
        flat[off[i]:off[i + 1]] = np.ascontiguousarray(m, dtype=np.uint8).ravel()
    return flat, off


def _b(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8))


def _l(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int64))


def fwd_dropout(q, k, v, cu_seqlens, scale, masks, keep_scale, seqused=None):
    """Forward with an explicit keep mask per sequence ([H, L, L], 1 = kept) on the
    probabilities and the factor keep_scale = 1 / (1 - p).  Returns (O, LSE)."""
    q, k, v = _prep(q), _prep(k), _prep(v)
    assert q.shape == k.shape == v.shape
    cu = np.ascontiguousarray(cu_seqlens, dtype=np.int32)
    su = None if seqused is None else np.ascontiguousarray(seqused, dtype=np.int32)
    t, h, d = q.shape
    assert cu[-1] == t and len(masks) == len(cu) - 1
    flat, off = _flatten_masks(masks, cu, h)
    o = np.zeros_like(q)
    lse = np.zeros((h, t), dtype=np.float64)
    rc = _load().oracle_fmha_varlen_fwd_dropout(_d(q), _d(k), _d(v), _i(cu), _i(su), len(cu) - 1,
                                                h, d, float(scale), _b(flat), _l(off),
                                                float(keep_scale), _d(o), _d(lse))
    if rc:
        raise ValueError("oracle_fmha_varlen_fwd_dropout: bad arguments")
    return o, lse


def bwd_dropout(q, k, v, d_o, cu_seqlens, scale, masks, keep_scale, seqused=None):
    """Backward of fwd_dropout for the same masks.  Returns (dQ, dK, dV)."""
    q, k, v, d_o = _prep(q), _prep(k), _prep(v), _prep(d_o)
    assert q.shape == k.shape == v.shape == d_o.shape
    cu = np.ascontiguousarray(cu_seqlens, dtype=np.int32)
    su = None if seqused is None else np.ascontiguousarray(seqused, dtype=np.int32)
    t, h, d = q.shape
    assert cu[-1] == t and len(masks) == len(cu) - 1
    flat, off = _flatten_masks(masks, cu, h)
    dq, dk, dv = np.zeros_like(q), np.zeros_like(q), np.zeros_like(q)
    rc = _load().oracle_fmha_varlen_bwd_dropout(_d(q), _d(k), _d(v), _d(d_o), _i(cu), _i(su),
                                                len(cu) - 1, h, d, float(scale), _b(flat), _l(off),
                                                float(keep_scale), _d(dq), _d(dk), _d(dv))
    if rc:
        raise ValueError("oracle_fmha_varlen_bwd_dropout: bad arguments")
    return dq, dk, dv
