"""CPU checker (``gnnagg_ref.c``) loaded through ctypes on numpy arrays.

TEST INFRASTRUCTURE ONLY.  Nothing in the GPU package imports this module;
it is used by the tests, by the smoke check and by the benchmark's
CPU-baseline leg.  It shares no code with the GPU path.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gnnagg_ref.c")
_LIB = os.path.join(_HERE, "libgnnagg_ref.so")

SUM, WSUM, MEAN, MAX, SUM_SCALED = 0, 1, 2, 3, 4
F32, BF16 = 0, 1
SELF_LOOPS, NORM_SYM = 1, 2


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-Wall", "-shared", "-fPIC", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        i64, i32, u32, f32, ci, vp = (ctypes.c_int64, ctypes.c_int32, ctypes.c_uint32, ctypes.c_float,
                                      ctypes.c_int, ctypes.c_void_p)
        lib.gnnagg_ref_build_csr.restype = ci
        lib.gnnagg_ref_build_csr.argtypes = [i64, i64, vp, vp, u32, vp, vp, vp, vp, ci]
        lib.gnnagg_ref_aggregate.restype = ci
        lib.gnnagg_ref_aggregate.argtypes = [ci, i64, vp, vp, vp, vp, ci, vp, i32, i32, ci, ci]
        lib.gnnagg_ref_aggregate_rows.restype = ci
        lib.gnnagg_ref_aggregate_rows.argtypes = [ci, i64, vp, vp, vp, vp, vp, ci, vp, i32, ci]
        lib.gnnagg_ref_gat_attention.restype = ci
        lib.gnnagg_ref_gat_attention.argtypes = [i64, vp, vp, vp, vp, vp, i32, i32, f32, vp, vp, ci]
        lib.gnnagg_ref_gat_attention_rows.restype = ci
        lib.gnnagg_ref_gat_attention_rows.argtypes = [i64, vp, vp, vp, vp, vp, vp, i32, i32, f32, vp, ci]
        lib.gnnagg_ref_combine.restype = ci
        lib.gnnagg_ref_combine.argtypes = [i64, vp, ci, i32, vp, vp, i32, ci, vp, ci]
        lib.gnnagg_ref_update.restype = ci
        lib.gnnagg_ref_update.argtypes = [i64, i32, vp, vp, ci, vp]
        lib.gnnagg_ref_gcn_factors.restype = ci
        lib.gnnagg_ref_gcn_factors.argtypes = [i64, vp, vp]
        lib.gnnagg_ref_scale_rows.restype = ci
        lib.gnnagg_ref_scale_rows.argtypes = [i64, i32, vp, ci, vp, vp]
        _lib = lib
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dt):
    a = np.ascontiguousarray(a, dtype=dt)
    return a


def build_csr(N, src, dst, flags=0, want_w=False, want_perm=False, threads=1):
    """-> (rowptr int64 [N+1], colidx int32 [nnz], edge_w float32|None, perm int64|None)"""
    src = _c(src, np.int32)
    dst = _c(dst, np.int32)
    E = src.shape[0]
    nnz = E + (N if flags & SELF_LOOPS else 0)
    rowptr = np.empty(N + 1, dtype=np.int64)
    colidx = np.empty(nnz, dtype=np.int32)
    w = np.empty(nnz, dtype=np.float32) if want_w else None
    perm = np.empty(nnz, dtype=np.int64) if want_perm else None
    rc = _load().gnnagg_ref_build_csr(N, E, _p(src), _p(dst), flags, _p(rowptr), _p(colidx), _p(w), _p(perm),
                                      threads)
    if rc != 0:
        raise ValueError("gnnagg_ref_build_csr failed: %d" % rc)
    return rowptr, colidx, w, perm


def _xinfo(X):
    if X.dtype == np.float32:
        return F32
    if X.dtype == np.uint16:
        return BF16
    raise TypeError("X must be float32 or uint16 (bf16 bits)")


def aggregate(op, rowptr, colidx, edge_w, X, f_chunk=0, form=0, threads=1):
    """Full aggregation; X is float32 [N,F] or uint16 (bf16 bits) [N,F]."""
    X = np.ascontiguousarray(X)
    N, F = X.shape
    assert rowptr.shape[0] == N + 1
    out = np.empty((N, F), dtype=np.float32)
    rc = _load().gnnagg_ref_aggregate(op, N, _p(rowptr), _p(colidx), _p(edge_w), _p(X), _xinfo(X), _p(out), F,
                                      f_chunk, form, threads)
    if rc != 0:
        raise ValueError("gnnagg_ref_aggregate failed: %d" % rc)
    return out


def aggregate_rows(op, rows, rowptr, colidx, edge_w, X, threads=1):
    X = np.ascontiguousarray(X)
    F = X.shape[1]
    rows = _c(rows, np.int64)
    out = np.empty((rows.shape[0], F), dtype=np.float32)
    rc = _load().gnnagg_ref_aggregate_rows(op, rows.shape[0], _p(rows), _p(rowptr), _p(colidx), _p(edge_w), _p(X),
                                           _xinfo(X), _p(out), F, threads)
    if rc != 0:
        raise ValueError("gnnagg_ref_aggregate_rows failed: %d" % rc)
    return out


def gat_attention(rowptr, colidx, H, a_src, a_dst, negative_slope=0.2, want_alpha=True, want_out=True, threads=1):
    """H float32 [N,heads,C]; -> (alpha [nnz,heads]|None, out [N,heads,C]|None)"""
    H = _c(H, np.float32)
    N, heads, C = H.shape
    a_src = _c(a_src, np.float32)
    a_dst = _c(a_dst, np.float32)
    assert a_src.shape == (heads, C) and a_dst.shape == (heads, C)
    nnz = int(rowptr[N])
    alpha = np.empty((nnz, heads), dtype=np.float32) if want_alpha else None
    out = np.empty((N, heads, C), dtype=np.float32) if want_out else None
    rc = _load().gnnagg_ref_gat_attention(N, _p(rowptr), _p(colidx), _p(H), _p(a_src), _p(a_dst), heads, C,
                                          negative_slope, _p(alpha), _p(out), threads)
    if rc != 0:
        raise ValueError("gnnagg_ref_gat_attention failed: %d" % rc)
    return alpha, out


def gat_attention_rows(rows, rowptr, colidx, H, a_src, a_dst, negative_slope=0.2, threads=1):
    """Attention output for the listed destination rows only: -> out [len(rows), heads, C]."""
    H = _c(H, np.float32)
    N, heads, C = H.shape
    a_src = _c(a_src, np.float32)
    a_dst = _c(a_dst, np.float32)
    rows = _c(rows, np.int64)
    out = np.empty((rows.shape[0], heads, C), dtype=np.float32)
    rc = _load().gnnagg_ref_gat_attention_rows(rows.shape[0], _p(rows), _p(rowptr), _p(colidx), _p(H), _p(a_src),
                                               _p(a_dst), heads, C, negative_slope, _p(out), threads)
    if rc != 0:
        raise ValueError("gnnagg_ref_gat_attention_rows failed: %d" % rc)
    return out


def combine(X, W, bias=None, relu=False, threads=1):
    """out [N,H] float32 = act(X @ W + bias); X float32 or uint16 (bf16 bits) [N,F], W float32 [F,H]."""
    X = np.ascontiguousarray(X)
    W = _c(W, np.float32)
    N, F = X.shape
    assert W.shape[0] == F
    H = W.shape[1]
    bias = None if bias is None else _c(bias, np.float32)
    out = np.empty((N, H), dtype=np.float32)
    rc = _load().gnnagg_ref_combine(N, _p(X), _xinfo(X), F, _p(W), _p(bias), H, int(bool(relu)), _p(out), threads)
    if rc != 0:
        raise ValueError("gnnagg_ref_combine failed: %d" % rc)
    return out


def update(A, bias=None, relu=False):
    """out [N,F] float32 = act(A + bias): the Update step without a weight matrix on an aggregated matrix."""
    A = _c(A, np.float32)
    N, F = A.shape
    bias = None if bias is None else _c(bias, np.float32)
    out = np.empty((N, F), dtype=np.float32)
    rc = _load().gnnagg_ref_update(N, F, _p(A), _p(bias), int(bool(relu)), _p(out))
    if rc != 0:
        raise ValueError("gnnagg_ref_update failed: %d" % rc)
    return out


def gcn_factors(rowptr):
    """s[i] = 1/sqrt(deg(i)) as float32, 0 for an empty row."""
    rowptr = _c(rowptr, np.int64)
    N = rowptr.shape[0] - 1
    s = np.empty(N, dtype=np.float32)
    if _load().gnnagg_ref_gcn_factors(N, _p(rowptr), _p(s)) != 0:
        raise ValueError("gnnagg_ref_gcn_factors failed")
    return s


def scale_rows(X, scale):
    """out[j, :] = scale[j] * X[j, :] as float32; X float32 or uint16 (bf16 bits)."""
    X = np.ascontiguousarray(X)
    N, F = X.shape
    scale = _c(scale, np.float32)
    assert scale.shape[0] == N
    out = np.empty((N, F), dtype=np.float32)
    if _load().gnnagg_ref_scale_rows(N, F, _p(X), _xinfo(X), _p(scale), _p(out)) != 0:
        raise ValueError("gnnagg_ref_scale_rows failed")
    return out
