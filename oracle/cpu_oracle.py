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
        f32 = ctypes.c_float
        lib.oracle_expf.argtypes = [f32]
        lib.oracle_expf.restype = f32
        lib.oracle_gelu.argtypes = [f32]
        lib.oracle_gelu.restype = f32
        lib.oracle_mlp_logits.argtypes = [vp, vp, vp, vp, vp, vp, i64, i32, i32, i32]
        lib.oracle_mlp_logits.restype = ctypes.c_int
        lib.oracle_topk_softmax.argtypes = [vp, vp, vp, i64, i32, i32]
        lib.oracle_topk_softmax.restype = None
        lib.oracle_apply_mix.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, i64, i32, i32, i32, i32, i32]
        lib.oracle_apply_mix.restype = ctypes.c_int
        lib.oracle_route_compose.argtypes = [vp, vp, vp, i32, i32, vp, i64]
        lib.oracle_route_compose.restype = None
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


def expf(y):
    return float(_lib().oracle_expf(float(y)))


def gelu(u):
    return float(_lib().oracle_gelu(float(u)))


def mlp_logits(x_bits, W1_bits, b1, W2_bits, b2):
    """Router logits W2^T GELU(W1^T x + b1) + b2, fp32 [N][K]."""
    x = _c(x_bits, np.uint16)
    N, d = x.shape
    W1 = _c(W1_bits, np.uint16)
    H = W1.shape[1]
    if W1.shape[0] != d:
        raise ValueError("W1 must be [d][H]")
    W2 = _c(W2_bits, np.uint16)
    K = W2.shape[1]
    if W2.shape[0] != H:
        raise ValueError("W2 must be [H][K]")
    b1 = _c(b1, np.float32, (H,))
    b2 = _c(b2, np.float32, (K,))
    logits = np.empty((N, K), dtype=np.float32)
    if _lib().oracle_mlp_logits(_p(x), _p(W1), _p(b1), _p(W2), _p(b2), _p(logits), N, d, H, K) != 0:
        raise MemoryError
    return logits


def topk_softmax(logits, k):
    """(idx [N][k] int32 in descending logit order, w [N][k] fp32 softmax over the selected)."""
    l = _c(logits, np.float32)
    N, K = l.shape
    if not 1 <= k <= K:
        raise ValueError("k must be in [1, K]")
    idx = np.empty((N, k), dtype=np.int32)
    w = np.empty((N, k), dtype=np.float32)
    _lib().oracle_topk_softmax(_p(l), _p(idx), _p(w), N, K, k)
    return idx, w


def apply_mix(x_bits, W_bits, A_bits, B_bits, idx, w=None, slots=None, C=None):
    """h_i = x_i W + sum_j w_ij (x_i A_s) B_s, s = slots[idx_ij] (slots None: s = idx_ij).
    A, B are pools [S][...]; C (number of targets) defaults to S."""
    x = _c(x_bits, np.uint16)
    N, d_in = x.shape
    W = _c(W_bits, np.uint16)
    d_out = W.shape[1]
    A = _c(A_bits, np.uint16)
    S, _, rank = A.shape
    B = _c(B_bits, np.uint16, (S, rank, d_out))
    idx = _c(idx, np.int32)
    if idx.ndim == 1:
        idx = idx.reshape(N, 1)
    k = idx.shape[1]
    wp = None
    if w is not None:
        w = _c(w, np.float32, (N, k))
        wp = _p(w)
    sp = None
    if slots is not None:
        slots = _c(slots, np.int32)
        if slots.size and (slots.min() < 0 or slots.max() >= S):
            raise ValueError("slot out of range")
        sp = _p(slots)
        C = slots.shape[0] if C is None else C
    C = S if C is None else C
    h = np.empty((N, d_out), dtype=np.float32)
    if _lib().oracle_apply_mix(_p(x), _p(W), _p(A), _p(B), _p(idx), wp, sp, _p(h), N, d_in, d_out,
                               C, rank, k) != 0:
        raise MemoryError
    return h


def route_compose(v, adapter, breaks, n_adapters):
    """c = adapter * M + modality(v); -1 when either part is out of range."""
    v = _c(v, np.int32)
    N = v.shape[0]
    adapter = _c(adapter, np.int32, (N,))
    b = _c(breaks, np.int32)
    M = b.shape[0] - 1
    r = np.empty(N, dtype=np.int32)
    _lib().oracle_route_compose(_p(v), _p(adapter), _p(b), M, n_adapters, _p(r), N)
    return r
