"""ctypes front end of the C oracle (oracle/molora_oracle.c).

TEST INFRASTRUCTURE, NOT THE PRODUCT.  Every function takes and returns numpy arrays;
bf16 tensors travel as uint16 bit patterns.  The arithmetic lives in the C file; this
module only marshals arguments.
"""
import ctypes
import os

import numpy as np

from . import build as _build

_LIB = None


def _lib():
    global _LIB
    if _LIB is None:
        path = _build.LIB
        if not os.path.exists(path):
            _build.build()
        lib = ctypes.CDLL(path)
        i64, i32, vp = ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p
        lib.oracle_route_gate.argtypes = [vp, vp, vp, i64, i32, i32]
        lib.oracle_route_gate.restype = ctypes.c_int
        lib.oracle_gate_logits.argtypes = [vp, vp, vp, i64, i32, i32]
        lib.oracle_gate_logits.restype = ctypes.c_int
        lib.oracle_route_vocab.argtypes = [vp, vp, i32, vp, i64]
        lib.oracle_route_vocab.restype = None
        lib.oracle_bucket.argtypes = [vp, vp, vp, i64, i32]
        lib.oracle_bucket.restype = i64
        lib.oracle_apply_rows.argtypes = [vp, vp, vp, vp, vp, vp, i64, vp, i64, i32, i32, i32, i32]
        lib.oracle_apply_rows.restype = ctypes.c_int
        lib.oracle_num_threads.argtypes = []
        lib.oracle_num_threads.restype = ctypes.c_int
        _LIB = lib
    return _LIB


def _c(a, dtype, shape=None):
    a = np.ascontiguousarray(a, dtype=dtype)
    if shape is not None and tuple(a.shape) != tuple(shape):
        raise ValueError(f"expected shape {shape}, got {a.shape}")
    return a


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def num_threads():
    return int(_lib().oracle_num_threads())


def route_gate(x_bits, G_bits):
    """r[i] = argmax_c (x_i . G[:, c]) in fp32, ascending-k sums, lowest index on ties."""
    x = _c(x_bits, np.uint16)
    N, d_in = x.shape
    G = _c(G_bits, np.uint16)
    if G.shape[0] != d_in:
        raise ValueError("G must be [d_in][C]")
    C = G.shape[1]
    r = np.empty(N, dtype=np.int32)
    if _lib().oracle_route_gate(_p(x), _p(G), _p(r), N, d_in, C) != 0:
        raise MemoryError
    return r


def gate_logits(x_bits, G_bits):
    x = _c(x_bits, np.uint16)
    N, d_in = x.shape
    G = _c(G_bits, np.uint16, (d_in, np.shape(G_bits)[1]))
    C = G.shape[1]
    out = np.empty((N, C), dtype=np.float32)
    if _lib().oracle_gate_logits(_p(x), _p(G), _p(out), N, d_in, C) != 0:
        raise MemoryError
    return out


def route_vocab(v, breaks):
    v = _c(v, np.int32)
    b = _c(breaks, np.int32)
    M = b.shape[0] - 1
    if M < 1:
        raise ValueError("need at least two breaks")
    r = np.empty(v.shape[0], dtype=np.int32)
    _lib().oracle_route_vocab(_p(v), _p(b), M, _p(r), v.shape[0])
    return r


def bucket(r, C):
    """Returns (offsets[C+1], perm[N], number of out-of-range tokens)."""
    r = _c(r, np.int32)
    N = r.shape[0]
    offsets = np.empty(C + 1, dtype=np.int32)
    perm = np.empty(N, dtype=np.int32)
    bad = _lib().oracle_bucket(_p(r), _p(offsets), _p(perm), N, C)
    if bad < 0:
        raise MemoryError
    return offsets, perm, int(bad)


def apply_rows(x_bits, W_bits, A_bits, B_bits, r, rows=None):
    """h rows (fp32) for the listed tokens (all tokens when rows is None)."""
    x = _c(x_bits, np.uint16)
    N, d_in = x.shape
    W = _c(W_bits, np.uint16)
    d_out = W.shape[1]
    if W.shape[0] != d_in:
        raise ValueError("W must be [d_in][d_out]")
    A = _c(A_bits, np.uint16)
    C, _, rank = A.shape
    if A.shape[1] != d_in:
        raise ValueError("A must be [C][d_in][rank]")
    B = _c(B_bits, np.uint16, (C, rank, d_out))
    r = _c(r, np.int32, (N,))
    if rows is None:
        rows_arr, n_rows, rows_p = None, N, None
    else:
        rows_arr = _c(rows, np.int64)
        if rows_arr.size and (rows_arr.min() < 0 or rows_arr.max() >= N):
            raise ValueError("row index out of range")
        n_rows, rows_p = rows_arr.shape[0], _p(rows_arr)
    h = np.empty((n_rows, d_out), dtype=np.float32)
    rc = _lib().oracle_apply_rows(_p(x), _p(W), _p(A), _p(B), _p(r), rows_p, n_rows, _p(h),
                                  N, d_in, d_out, C, rank)
    if rc != 0:
        raise MemoryError
    return h


def apply(x_bits, W_bits, A_bits, B_bits, r):
    return apply_rows(x_bits, W_bits, A_bits, B_bits, r, None)
