"""Thin ctypes binding of libmolora.so (the C ABI of include/molora.h).

Argument marshalling only: torch supplies device memory and the current HIP stream, every
step of the path runs in the library's kernels.  There is no fallback: if the library is
not built, the first call raises.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmolora.so")

MOLORA_OK = 0
EXPORTS = ["molora_route", "molora_route_vocab", "molora_bucket", "molora_apply_workspace_bytes",
           "molora_apply", "molora_apply_bucketed", "molora_shrink", "molora_shrink_workspace_bytes",
           "molora_base_expand",
           "molora_base_expand_fixed", "molora_init", "molora_dense_shrink_supported", "molora_bucket_shrink",
           "molora_gate_dispatch_shrink", "molora_base_expand_dense", "molora_apply_static", "molora_static_workspace_bytes",
           "molora_route_mlp_workspace_bytes", "molora_route_mlp", "molora_route_compose",
           "molora_gate_dispatch",
           "molora_apply_mix_workspace_bytes", "molora_apply_mix",
           "molora_graph_begin", "molora_graph_end", "molora_graph_launch", "molora_graph_destroy",
           "molora_status_string", "molora_version"]

_lib = None


class MoloraError(RuntimeError):
    def __init__(self, status, what):
        self.status = status
        super().__init__(f"{what}: {status_string(status)} ({status})")


def load():
    """dlopen the library and declare the prototypes (no GPU needed for this)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} is not built; run `python -m paper_2603_15965_amd.build` "
            "(or __graft_entry__.build()) first")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i64, i32, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_size_t
    lib.molora_route.argtypes = [vp, vp, vp, i64, i32, i32, vp]
    lib.molora_route.restype = ctypes.c_int
    lib.molora_route_vocab.argtypes = [vp, ctypes.POINTER(i32), i32, vp, i64, vp]
    lib.molora_route_vocab.restype = ctypes.c_int
    lib.molora_bucket.argtypes = [vp, vp, vp, i64, i32, vp, vp]
    lib.molora_bucket.restype = ctypes.c_int
    lib.molora_apply_workspace_bytes.argtypes = [i64, i32, i32, i32, i32]
    lib.molora_apply_workspace_bytes.restype = sz
    lib.molora_apply.argtypes = [vp, vp, vp, vp, vp, vp, i64, i32, i32, i32, i32, vp, sz, vp]
    lib.molora_apply.restype = ctypes.c_int
    lib.molora_apply_bucketed.argtypes = [vp, vp, vp, vp, vp, vp, vp, i64, i32, i32, i32, i32, vp, sz, vp]
    lib.molora_apply_bucketed.restype = ctypes.c_int
    lib.molora_shrink.argtypes = [vp, vp, vp, vp, vp, i64, i32, i32, i32, vp, sz, vp]
    lib.molora_shrink.restype = ctypes.c_int
    lib.molora_shrink_workspace_bytes.argtypes = [i64, i32, i32, i32]
    lib.molora_shrink_workspace_bytes.restype = sz
    lib.molora_base_expand.argtypes = [vp, vp, vp, vp, vp, vp, vp, i64, i32, i32, i32, i32, vp]
    lib.molora_base_expand.restype = ctypes.c_int
    lib.molora_base_expand_fixed.argtypes = [vp, vp, vp, vp, vp, vp, vp, i64, i32, i32, i32, i32, i32, vp]
    lib.molora_base_expand_fixed.restype = ctypes.c_int
    lib.molora_apply_static.argtypes = [vp, vp, vp, vp, vp, vp, i64, i32, i32, i32, i32, vp]
    lib.molora_apply_static.restype = ctypes.c_int
    lib.molora_static_workspace_bytes.argtypes = []
    lib.molora_static_workspace_bytes.restype = sz
    lib.molora_dense_shrink_supported.argtypes = [i64, i32, i32, i32]
    lib.molora_dense_shrink_supported.restype = ctypes.c_int32
    lib.molora_bucket_shrink.argtypes = [vp, vp, vp, vp, vp, vp, i64, i32, i32, i32, vp, vp]
    lib.molora_bucket_shrink.restype = ctypes.c_int
    lib.molora_gate_dispatch_shrink.argtypes = [vp, vp, ctypes.POINTER(i32), i32, i32, vp, vp, vp, vp, vp, vp,
                                                i64, i32, i32, vp, vp]
    lib.molora_gate_dispatch_shrink.restype = ctypes.c_int
    lib.molora_base_expand_dense.argtypes = [vp, vp, vp, vp, vp, vp, vp, i64, i32, i32, i32, i32, vp]
    lib.molora_base_expand_dense.restype = ctypes.c_int
    lib.molora_init.argtypes = []
    lib.molora_init.restype = ctypes.c_int
    lib.molora_route_mlp_workspace_bytes.argtypes = [i64, i32]
    lib.molora_route_mlp_workspace_bytes.restype = sz
    lib.molora_route_mlp.argtypes = [vp, vp, vp, vp, vp, vp, vp, i64, i32, i32, i32, i32, vp, sz, vp]
    lib.molora_route_mlp.restype = ctypes.c_int
    lib.molora_route_compose.argtypes = [vp, vp, ctypes.POINTER(i32), i32, i32, vp, i64, vp]
    lib.molora_route_compose.restype = ctypes.c_int
    lib.molora_gate_dispatch.argtypes = [vp, vp, ctypes.POINTER(i32), i32, i32, vp, vp, vp, i64, vp, vp]
    lib.molora_gate_dispatch.restype = ctypes.c_int
    lib.molora_apply_mix_workspace_bytes.argtypes = [i64, i32, i32, i32, i32, i32]
    lib.molora_apply_mix_workspace_bytes.restype = sz
    lib.molora_apply_mix.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, i64, i32, i32, i32, i32, i32, vp, sz, vp]
    lib.molora_apply_mix.restype = ctypes.c_int
    lib.molora_graph_begin.argtypes = [vp]
    lib.molora_graph_begin.restype = ctypes.c_int
    lib.molora_graph_end.argtypes = [vp, ctypes.POINTER(vp)]
    lib.molora_graph_end.restype = ctypes.c_int
    lib.molora_graph_launch.argtypes = [vp, vp]
    lib.molora_graph_launch.restype = ctypes.c_int
    lib.molora_graph_destroy.argtypes = [vp]
    lib.molora_graph_destroy.restype = None
    lib.molora_status_string.argtypes = [ctypes.c_int]
    lib.molora_status_string.restype = ctypes.c_char_p
    lib.molora_version.argtypes = []
    lib.molora_version.restype = ctypes.c_char_p
    _lib = lib
    return lib


def status_string(status):
    return load().molora_status_string(int(status)).decode()


def version():
    return load().molora_version().decode()


def _check(status, what):
    if status != MOLORA_OK:
        raise MoloraError(status, what)


def _dev(t, dtype, name):
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{name} must be a device tensor")
    if t.dtype != dtype:
        raise TypeError(f"{name} must be {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def molora_route(x, G, r=None, stream=None):
    """r[i] = argmax_c x[i] . G[:, c] (fp32 ascending-k chain, lowest index on ties)."""
    N, d_in = x.shape
    C = G.shape[1]
    if G.shape[0] != d_in:
        raise ValueError("G must be [d_in][C]")
    if r is None:
        r = torch.empty(N, dtype=torch.int32, device=x.device)
    st = load().molora_route(_dev(x, torch.bfloat16, "x"), _dev(G, torch.bfloat16, "G"),
                             _dev(r, torch.int32, "r"), N, d_in, C, _stream(stream))
    _check(st, "molora_route")
    return r


def molora_route_vocab(v, breaks, r=None, stream=None):
    """r[i] = m with breaks[m] <= v[i] < breaks[m+1], else -1.  breaks: host ints."""
    N = v.shape[0]
    b = [int(t) for t in breaks]
    M = len(b) - 1
    arr = (ctypes.c_int32 * len(b))(*b)
    if r is None:
        r = torch.empty(N, dtype=torch.int32, device=v.device)
    st = load().molora_route_vocab(_dev(v, torch.int32, "v"), arr, M, _dev(r, torch.int32, "r"), N,
                                   _stream(stream))
    _check(st, "molora_route_vocab")
    return r


def molora_bucket(r, C, offsets=None, perm=None, err_flag=None, stream=None):
    """Stable grouping of tokens by target: returns (offsets[C+1], perm[N])."""
    N = r.shape[0]
    if offsets is None:
        offsets = torch.empty(C + 1, dtype=torch.int32, device=r.device)
    if perm is None:
        perm = torch.empty(max(N, 1), dtype=torch.int32, device=r.device)[:N]
    st = load().molora_bucket(_dev(r, torch.int32, "r"), _dev(offsets, torch.int32, "offsets"),
                              _dev(perm, torch.int32, "perm"), N, C,
                              None if err_flag is None else _dev(err_flag, torch.int32, "err_flag"),
                              _stream(stream))
    _check(st, "molora_bucket")
    return offsets, perm


def molora_apply_workspace_bytes(N, d_in, d_out, C, rank):
    return int(load().molora_apply_workspace_bytes(N, d_in, d_out, C, rank))


def _shapes(x, W, A, B):
    N, d_in = x.shape
    d_out = W.shape[1]
    C, _, rank = A.shape
    if W.shape[0] != d_in or A.shape[1] != d_in or tuple(B.shape) != (C, rank, d_out):
        raise ValueError("expected W [d_in][d_out], A [C][d_in][rank], B [C][rank][d_out]")
    return N, d_in, d_out, C, rank


def new_workspace(N, d_in, d_out, C, rank, device="cuda"):
    nbytes = molora_apply_workspace_bytes(N, d_in, d_out, C, rank)
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)


def molora_apply(x, W, A, B, r, h=None, workspace=None, stream=None):
    """h[i] = x[i] W + (x[i] A[r[i]]) B[r[i]]  (fp32 [N][d_out])."""
    N, d_in, d_out, C, rank = _shapes(x, W, A, B)
    if h is None:
        h = torch.empty((N, d_out), dtype=torch.float32, device=x.device)
    if workspace is None:
        workspace = new_workspace(N, d_in, d_out, C, rank, x.device)
    bf = torch.bfloat16
    st = load().molora_apply(_dev(x, bf, "x"), _dev(W, bf, "W"), _dev(A, bf, "A"), _dev(B, bf, "B"),
                             _dev(r, torch.int32, "r"), _dev(h, torch.float32, "h"),
                             N, d_in, d_out, C, rank, _dev(workspace, torch.uint8, "workspace"),
                             workspace.numel(), _stream(stream))
    _check(st, "molora_apply")
    return h


def molora_apply_static(x, W, A, B, r, h, stream=None):
    """molora_apply on the library's own fixed scratch array: no workspace argument and no
    allocation anywhere in the call, so h must be supplied."""
    N, d_in, d_out, C, rank = _shapes(x, W, A, B)
    bf = torch.bfloat16
    st = load().molora_apply_static(_dev(x, bf, "x"), _dev(W, bf, "W"), _dev(A, bf, "A"),
                                    _dev(B, bf, "B"), _dev(r, torch.int32, "r"),
                                    _dev(h, torch.float32, "h"), N, d_in, d_out, C, rank,
                                    _stream(stream))
    _check(st, "molora_apply_static")
    return h


def molora_apply_bucketed(x, W, A, B, offsets, perm, h=None, workspace=None, stream=None):
    """molora_apply for a caller that already holds molora_bucket's output."""
    N, d_in, d_out, C, rank = _shapes(x, W, A, B)
    if h is None:
        h = torch.empty((N, d_out), dtype=torch.float32, device=x.device)
    if workspace is None:
        workspace = new_workspace(N, d_in, d_out, C, rank, x.device)
    bf = torch.bfloat16
    st = load().molora_apply_bucketed(
        _dev(x, bf, "x"), _dev(W, bf, "W"), _dev(A, bf, "A"), _dev(B, bf, "B"),
        _dev(offsets, torch.int32, "offsets"), _dev(perm, torch.int32, "perm"),
        _dev(h, torch.float32, "h"), N, d_in, d_out, C, rank,
        _dev(workspace, torch.uint8, "workspace"), workspace.numel(), _stream(stream))
    _check(st, "molora_apply_bucketed")
    return h


def molora_shrink_workspace(N, d_in, C, rank, device="cuda"):
    """Scratch for molora_shrink (None when these sizes need none)."""
    nbytes = int(load().molora_shrink_workspace_bytes(N, d_in, C, rank))
    return torch.empty(nbytes, dtype=torch.uint8, device=device) if nbytes else None


def molora_shrink(x, A, offsets, perm, t=None, workspace="auto", stream=None):
    """t[p] = x[perm[p]] A_c as [hi | lo] bf16 halves, [N][2*rank].  workspace: a tensor from
    molora_shrink_workspace, None (never split K over workgroups) or "auto" (allocate)."""
    N, d_in = x.shape
    C, _, rank = A.shape
    if t is None:
        t = torch.empty((N, 2 * rank), dtype=torch.bfloat16, device=x.device)
    if isinstance(workspace, str):
        workspace = molora_shrink_workspace(N, d_in, C, rank, x.device)
    bf = torch.bfloat16
    st = load().molora_shrink(_dev(x, bf, "x"), _dev(A, bf, "A"), _dev(offsets, torch.int32, "offsets"),
                              _dev(perm, torch.int32, "perm"), _dev(t, bf, "t"), N, d_in, C, rank,
                              None if workspace is None else _dev(workspace, torch.uint8, "workspace"),
                              0 if workspace is None else workspace.numel(), _stream(stream))
    _check(st, "molora_shrink")
    return t


def molora_base_expand(x, W, B, t, offsets, perm, h=None, stream=None, tile_rows=None):
    """h[perm[p]] = x[perm[p]] W + t_p B_c, every row written once.  tile_rows (64, 128 or
    256) forces the row-tile height (molora_base_expand_fixed, for the tiling ablation)."""
    N, d_in = x.shape
    d_out = W.shape[1]
    C, rank, _ = B.shape
    if h is None:
        h = torch.empty((N, d_out), dtype=torch.float32, device=x.device)
    bf = torch.bfloat16
    args = [_dev(x, bf, "x"), _dev(W, bf, "W"), _dev(B, bf, "B"), _dev(t, bf, "t"),
            _dev(offsets, torch.int32, "offsets"), _dev(perm, torch.int32, "perm"),
            _dev(h, torch.float32, "h"), N, d_in, d_out, C, rank]
    if tile_rows is None:
        st = load().molora_base_expand(*args, _stream(stream))
    else:
        st = load().molora_base_expand_fixed(*args, int(tile_rows), _stream(stream))
    _check(st, "molora_base_expand")
    return h


def molora_dense_shrink_supported(N, d_in, C, rank):
    """Whether dispatch and shrink can run in one launch for these sizes (C * rank <= 64, N > 512)."""
    return bool(load().molora_dense_shrink_supported(N, d_in, C, rank))


def molora_bucket_shrink(r, x, A, offsets=None, perm=None, t=None, err_flag=None, stream=None):
    """Dispatch (r given) and token-order shrink in one launch: (offsets, perm, t [N][2*C*rank])."""
    N, d_in = x.shape
    C, _, rank = A.shape
    if offsets is None:
        offsets = torch.empty(C + 1, dtype=torch.int32, device=x.device)
    if perm is None:
        perm = torch.empty(N, dtype=torch.int32, device=x.device)
    if t is None:
        t = torch.empty((N, 2 * C * rank), dtype=torch.bfloat16, device=x.device)
    bf = torch.bfloat16
    st = load().molora_bucket_shrink(_dev(r, torch.int32, "r"), _dev(x, bf, "x"), _dev(A, bf, "A"),
                                     _dev(offsets, torch.int32, "offsets"), _dev(perm, torch.int32, "perm"),
                                     _dev(t, bf, "t"), N, d_in, C, rank,
                                     None if err_flag is None else _dev(err_flag, torch.int32, "err_flag"),
                                     _stream(stream))
    _check(st, "molora_bucket_shrink")
    return offsets, perm, t


def molora_gate_dispatch_shrink(v, breaks, x, A, adapter=None, n_adapters=1, r=None, offsets=None, perm=None,
                                t=None, err_flag=None, stream=None):
    """Vocabulary / compositional gating, dispatch and token-order shrink in one launch:
    (r, offsets, perm, t [N][2*C*rank]) with C = n_adapters * M."""
    N, d_in = x.shape
    C, _, rank = A.shape
    b = [int(q) for q in breaks]
    M = len(b) - 1
    if C != n_adapters * M:
        raise ValueError("A must hold n_adapters * M adapters")
    arr = (ctypes.c_int32 * len(b))(*b)
    if r is None:
        r = torch.empty(N, dtype=torch.int32, device=x.device)
    if offsets is None:
        offsets = torch.empty(C + 1, dtype=torch.int32, device=x.device)
    if perm is None:
        perm = torch.empty(N, dtype=torch.int32, device=x.device)
    if t is None:
        t = torch.empty((N, 2 * C * rank), dtype=torch.bfloat16, device=x.device)
    bf = torch.bfloat16
    st = load().molora_gate_dispatch_shrink(
        _dev(v, torch.int32, "v"), None if adapter is None else _dev(adapter, torch.int32, "adapter"), arr, M,
        n_adapters, _dev(x, bf, "x"), _dev(A, bf, "A"), _dev(r, torch.int32, "r"),
        _dev(offsets, torch.int32, "offsets"), _dev(perm, torch.int32, "perm"), _dev(t, bf, "t"), N, d_in, rank,
        None if err_flag is None else _dev(err_flag, torch.int32, "err_flag"), _stream(stream))
    _check(st, "molora_gate_dispatch_shrink")
    return r, offsets, perm, t


def molora_base_expand_dense(x, W, B, t, offsets, perm, h=None, stream=None):
    """molora_base_expand reading the token-order intermediate of the two calls above."""
    N, d_in = x.shape
    d_out = W.shape[1]
    C, rank, _ = B.shape
    if h is None:
        h = torch.empty((N, d_out), dtype=torch.float32, device=x.device)
    bf = torch.bfloat16
    st = load().molora_base_expand_dense(_dev(x, bf, "x"), _dev(W, bf, "W"), _dev(B, bf, "B"), _dev(t, bf, "t"),
                                         _dev(offsets, torch.int32, "offsets"), _dev(perm, torch.int32, "perm"),
                                         _dev(h, torch.float32, "h"), N, d_in, d_out, C, rank, _stream(stream))
    _check(st, "molora_base_expand_dense")
    return h


def molora_init():
    """Once-per-device set-up (needed only before a stream capture made with the HIP API)."""
    _check(load().molora_init(), "molora_init")


def bf16_tensor(bits, device="cuda"):
    """numpy uint16 bit patterns -> torch.bfloat16 tensor on the device (same bits)."""
    import numpy as np
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16))
    return t.to(device).view(torch.bfloat16)


def molora_route_mlp(x, W1, b1, W2, b2, k, idx=None, w=None, workspace=None, stream=None):
    """Router MLP + top-k + softmax: returns (idx [N][k] int32, w [N][k] fp32)."""
    N, d_in = x.shape
    H, K = W2.shape
    if W1.shape != (d_in, H):
        raise ValueError("W1 must be [d_in][H]")
    if idx is None:
        idx = torch.empty((N, k), dtype=torch.int32, device=x.device)
    if w is None:
        w = torch.empty((N, k), dtype=torch.float32, device=x.device)
    if workspace is None:
        nbytes = int(load().molora_route_mlp_workspace_bytes(N, H))
        workspace = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=x.device)
    bf = torch.bfloat16
    st = load().molora_route_mlp(_dev(x, bf, "x"), _dev(W1, bf, "W1"), _dev(b1, torch.float32, "b1"),
                                 _dev(W2, bf, "W2"), _dev(b2, torch.float32, "b2"),
                                 _dev(idx, torch.int32, "idx"), _dev(w, torch.float32, "w"),
                                 N, d_in, H, K, k, _dev(workspace, torch.uint8, "workspace"),
                                 workspace.numel(), _stream(stream))
    _check(st, "molora_route_mlp")
    return idx, w


def molora_route_compose(v, adapter, breaks, n_adapters, r=None, stream=None):
    """r[i] = adapter[i] * M + modality(v[i]), -1 when either part is out of range."""
    N = v.shape[0]
    b = [int(t) for t in breaks]
    M = len(b) - 1
    arr = (ctypes.c_int32 * len(b))(*b)
    if r is None:
        r = torch.empty(N, dtype=torch.int32, device=v.device)
    st = load().molora_route_compose(_dev(v, torch.int32, "v"), _dev(adapter, torch.int32, "adapter"),
                                     arr, M, n_adapters, _dev(r, torch.int32, "r"), N, _stream(stream))
    _check(st, "molora_route_compose")
    return r


def molora_gate_dispatch(v, breaks, adapter=None, n_adapters=1, r=None, offsets=None, perm=None,
                         err_flag=None, stream=None):
    """Vocabulary / compositional gating and bucketing in one launch: (r, offsets, perm)."""
    N = v.shape[0]
    b = [int(t) for t in breaks]
    M = len(b) - 1
    arr = (ctypes.c_int32 * len(b))(*b)
    C = n_adapters * M
    if r is None:
        r = torch.empty(N, dtype=torch.int32, device=v.device)
    if offsets is None:
        offsets = torch.empty(C + 1, dtype=torch.int32, device=v.device)
    if perm is None:
        perm = torch.empty(max(N, 1), dtype=torch.int32, device=v.device)[:N]
    st = load().molora_gate_dispatch(
        _dev(v, torch.int32, "v"), None if adapter is None else _dev(adapter, torch.int32, "adapter"),
        arr, M, n_adapters, _dev(r, torch.int32, "r"), _dev(offsets, torch.int32, "offsets"),
        _dev(perm, torch.int32, "perm"), N,
        None if err_flag is None else _dev(err_flag, torch.int32, "err_flag"), _stream(stream))
    _check(st, "molora_gate_dispatch")
    return r, offsets, perm


def molora_apply_mix(x, W, A, B, idx, w=None, slots=None, C=None, h=None, workspace=None, stream=None):
    """h[i] = x[i] W + sum_j w[i][j] (x[i] A_s) B_s, s = slots[idx[i][j]] (slots None: idx)."""
    N, d_in, d_out, S, rank = _shapes(x, W, A, B)
    if idx.dim() == 1:
        idx = idx.reshape(N, 1)
    k = idx.shape[1]
    if C is None:
        C = S if slots is None else slots.shape[0]
    if h is None:
        h = torch.empty((N, d_out), dtype=torch.float32, device=x.device)
    if workspace is None:
        nbytes = int(load().molora_apply_mix_workspace_bytes(N, d_in, d_out, C, rank, k))
        workspace = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=x.device)
    bf = torch.bfloat16
    st = load().molora_apply_mix(
        _dev(x, bf, "x"), _dev(W, bf, "W"), _dev(A, bf, "A"), _dev(B, bf, "B"),
        _dev(idx, torch.int32, "idx"), None if w is None else _dev(w, torch.float32, "w"),
        None if slots is None else _dev(slots, torch.int32, "slots"), _dev(h, torch.float32, "h"),
        N, d_in, d_out, C, rank, k, _dev(workspace, torch.uint8, "workspace"), workspace.numel(),
        _stream(stream))
    _check(st, "molora_apply_mix")
    return h


class Graph:
    """A recorded sequence of molora_* calls.

        g = Graph(stream)            # a torch.cuda.Stream other than the default one
        with g.capture():
            molora_route(..., stream=stream); molora_bucket(..., stream=stream); ...
        g.launch()                   # replays on `stream`
    """

    def __init__(self, stream):
        self.stream = stream
        self._handle = None

    def capture(self):
        graph = self

        class _Capture:
            def __enter__(self):
                _check(load().molora_graph_begin(_stream(graph.stream)), "molora_graph_begin")

            def __exit__(self, et, ev, tb):
                h = ctypes.c_void_p()
                st = load().molora_graph_end(_stream(graph.stream), ctypes.byref(h))
                if et is None:
                    _check(st, "molora_graph_end")
                    graph._handle = h
                elif st == MOLORA_OK:
                    load().molora_graph_destroy(h)
                return False

        return _Capture()

    def launch(self, stream=None):
        if self._handle is None:
            raise RuntimeError("nothing captured")
        _check(load().molora_graph_launch(self._handle, _stream(stream or self.stream)),
               "molora_graph_launch")

    def destroy(self):
        if self._handle is not None:
            load().molora_graph_destroy(self._handle)
            self._handle = None
