"""numpy front end of the fp64 CPU oracle (TEST INFRASTRUCTURE ONLY).

Every function converts its inputs to contiguous int32 / float64 arrays, calls the C
routine of the same name in ftc_oracle.c and returns numpy arrays.  No arithmetic of the
method is done in this file.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.LIB
        if not os.path.exists(path):
            _build.build()
        _lib = C.CDLL(path)
        _lib.oracle_set_threads.restype = C.c_int
        _lib.oracle_tile_capacity.restype = C.c_int64
        _lib.oracle_tile_capacity.argtypes = [C.c_int64, C.c_int32, C.c_int32]
    return _lib


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _f64(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float64)


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def set_threads(t):
    return lib().oracle_set_threads(C.c_int(int(t)))


def gcn_norm(row_ptr, col_idx):
    """-> (vals fp64 [nnz], dinv fp64 [n])"""
    row_ptr, col_idx = _i32(row_ptr), _i32(col_idx)
    n = row_ptr.size - 1
    vals = np.empty(col_idx.size, dtype=np.float64)
    dinv = np.empty(n, dtype=np.float64)
    lib().oracle_gcn_norm(C.c_int32(n), _p(row_ptr), _p(col_idx), _p(vals), _p(dinv))
    return vals, dinv


def build_windows(row_ptr, col_idx, blk_h=16, blk_w=8):
    """-> dict of the index arrays; win_cols trimmed to sum of unique columns."""
    row_ptr, col_idx = _i32(row_ptr), _i32(col_idx)
    n = row_ptr.size - 1
    nnz = col_idx.size
    n_win = (n + blk_h - 1) // blk_h
    e2r = np.empty(nnz, dtype=np.int32)
    e2c = np.empty(nnz, dtype=np.int32)
    bp = np.empty(n_win, dtype=np.int32)
    wcp = np.empty(n_win + 1, dtype=np.int32)
    wc = np.empty(max(nnz, 1), dtype=np.int32)
    summary = np.zeros(2, dtype=np.int64)
    lib().oracle_build_windows(C.c_int32(n), _p(row_ptr), _p(col_idx), C.c_int32(blk_h),
                               C.c_int32(blk_w), _p(e2r), _p(e2c), _p(bp), _p(wcp), _p(wc),
                               _p(summary))
    return dict(blk_h=blk_h, blk_w=blk_w, n_windows=n_win, edge_to_row=e2r, edge_to_col=e2c,
                block_partition=bp, win_col_ptr=wcp, win_cols=wc[:int(summary[0])].copy(),
                summary=summary)


def spmm(row_ptr, col_idx, vals, X):
    """-> (out, abs) both fp64 [n, D]"""
    row_ptr, col_idx, vals, X = _i32(row_ptr), _i32(col_idx), _f64(vals), _f64(X)
    n = row_ptr.size - 1
    D = X.shape[1]
    out = np.zeros((n, D), dtype=np.float64)
    ab = np.zeros((n, D), dtype=np.float64)
    lib().oracle_spmm(C.c_int32(n), _p(row_ptr), _p(col_idx), _p(vals), _p(X), C.c_int64(D),
                      C.c_int32(D), _p(out), _p(ab), C.c_int64(D))
    return out, ab


def sddmm(row_ptr, col_idx, X, Y, rs=None, cs=None, alpha=1.0):
    """-> (s, abs) both fp64 [nnz]"""
    row_ptr, col_idx, X, Y = _i32(row_ptr), _i32(col_idx), _f64(X), _f64(Y)
    rs, cs = _f64(rs), _f64(cs)
    n = row_ptr.size - 1
    D = X.shape[1]
    assert Y.shape[1] == D
    s = np.zeros(col_idx.size, dtype=np.float64)
    ab = np.zeros(col_idx.size, dtype=np.float64)
    lib().oracle_sddmm(C.c_int32(n), _p(row_ptr), _p(col_idx), _p(X), _p(Y), C.c_int64(D),
                       C.c_int32(D), _p(rs), _p(cs), C.c_double(alpha), _p(s), _p(ab))
    return s, ab


def row_rnorm(H):
    H = _f64(H)
    rinv = np.empty(H.shape[0], dtype=np.float64)
    lib().oracle_row_rnorm(C.c_int32(H.shape[0]), _p(H), C.c_int64(H.shape[1]),
                           C.c_int32(H.shape[1]), _p(rinv))
    return rinv


def edge_softmax(row_ptr, s):
    row_ptr, s = _i32(row_ptr), _f64(s)
    p = np.zeros_like(s)
    lib().oracle_edge_softmax(C.c_int32(row_ptr.size - 1), _p(row_ptr), _p(s), _p(p))
    return p


def gemm(X, W):
    """-> (Z, abs) fp64 [n, d_out]"""
    X, W = _f64(X), _f64(W)
    n, d_in = X.shape
    d_out = W.shape[1]
    Z = np.zeros((n, d_out), dtype=np.float64)
    ab = np.zeros((n, d_out), dtype=np.float64)
    lib().oracle_gemm(C.c_int32(n), C.c_int32(d_in), C.c_int32(d_out), _p(X), C.c_int64(d_in),
                      _p(W), C.c_int64(d_out), _p(Z), _p(ab), C.c_int64(d_out))
    return Z, ab


def gcn_layer(row_ptr, col_idx, vals, X, W, relu=False):
    """-> (out, abs) fp64 [n, d_out]"""
    row_ptr, col_idx, vals, X, W = _i32(row_ptr), _i32(col_idx), _f64(vals), _f64(X), _f64(W)
    n, d_in = X.shape
    d_out = W.shape[1]
    Z = np.zeros((n, d_out), dtype=np.float64)
    Zabs = np.zeros((n, d_out), dtype=np.float64)
    out = np.zeros((n, d_out), dtype=np.float64)
    ab = np.zeros((n, d_out), dtype=np.float64)
    lib().oracle_gcn_layer(C.c_int32(n), _p(row_ptr), _p(col_idx), _p(vals), _p(X),
                           C.c_int64(d_in), C.c_int32(d_in), _p(W), C.c_int32(d_out),
                           C.c_int32(1 if relu else 0), _p(Z), _p(Zabs), _p(out), _p(ab))
    return out, ab


def agnn_layer(row_ptr, col_idx, H, beta=1.0):
    """-> (out fp64 [n, D], abs fp64 [n, D], p fp64 [nnz])"""
    row_ptr, col_idx, H = _i32(row_ptr), _i32(col_idx), _f64(H)
    n, D = H.shape
    rinv = np.empty(n, dtype=np.float64)
    p = np.zeros(col_idx.size, dtype=np.float64)
    out = np.zeros((n, D), dtype=np.float64)
    ab = np.zeros((n, D), dtype=np.float64)
    lib().oracle_agnn_layer(C.c_int32(n), _p(row_ptr), _p(col_idx), _p(H), C.c_int64(D),
                            C.c_int32(D), C.c_double(beta), _p(rinv), _p(p), _p(out), _p(ab))
    return out, ab, p


def tile_capacity(block_counter, blk_h=16, blk_w=8):
    return int(lib().oracle_tile_capacity(int(block_counter), blk_h, blk_w))
