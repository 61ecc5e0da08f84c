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
           "molora_gate_dispatch_shrink", "molora_base_expand_dense", "molora_bucket_shrink_small_supported",
           "molora_bucket_shrink_small", "molora_shrink_base_small", "molora_expand_small",
           "molora_pack_w_cols", "molora_pack_w", "molora_shrink_base_small_packed", "molora_expand_small_packed", "molora_apply_static", "molora_static_workspace_bytes",
           "molora_route_mlp_workspace_bytes", "molora_route_mlp", "molora_route_compose",
           "molora_gate_dispatch",
           "molora_apply_mix_workspace_bytes", "molora_apply_mix",
           "molora_graph_begin", "molora_graph_end", "molora_graph_launch", "molora_graph_destroy",
           "molora_launch_timer_create", "molora_launch_timer_arm", "molora_launch_timer_elapsed_us",
           "molora_launch_timer_destroy",
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
    lib.molora_bucket_shrink_small_supported.argtypes = [i64, i32, i32, i32]
    lib.molora_bucket_shrink_small_supported.restype = ctypes.c_int32
    lib.molora_bucket_shrink_small.argtypes = [vp, vp, vp, vp, vp, vp, i64, i32, i32, i32, vp, sz, vp, vp]
    lib.molora_bucket_shrink_small.restype = ctypes.c_int
    lib.molora_shrink_base_small.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, i64, i32, i32, i32, i32, vp, vp]
    lib.molora_shrink_base_small.restype = ctypes.c_int
    lib.molora_shrink_base_small_packed.argtypes = lib.molora_shrink_base_small.argtypes
    lib.molora_shrink_base_small_packed.restype = ctypes.c_int
    lib.molora_pack_w_cols.argtypes = [i32]
    lib.molora_pack_w_cols.restype = ctypes.c_int
    lib.molora_pack_w.argtypes = [vp, vp, i32, i32, vp]
    lib.molora_pack_w.restype = ctypes.c_int
    lib.molora_expand_small.argtypes = [vp, vp, vp, vp, vp, i64, i32, i32, i32, vp]
    lib.molora_expand_small.restype = ctypes.c_int
    lib.molora_expand_small_packed.argtypes = lib.molora_expand_small.argtypes
    lib.molora_expand_small_packed.restype = ctypes.c_int
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
    lib.molora_launch_timer_create.argtypes = [ctypes.POINTER(vp)]
    lib.molora_launch_timer_create.restype = ctypes.c_int
    lib.molora_launch_timer_arm.argtypes = [vp]
    lib.molora_launch_timer_arm.restype = ctypes.c_int
    lib.molora_launch_timer_elapsed_us.argtypes = [vp, ctypes.POINTER(ctypes.c_double)]
    lib.molora_launch_timer_elapsed_us.restype = ctypes.c_int
    lib.molora_launch_timer_destroy.argtypes = [vp]
    lib.molora_launch_timer_destroy.restype = None
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


class _T:
    """A tensor argument: what the library will take it for (dtype, shape), checked by _call."""

    def __init__(self, t, dtype, name, shape=None):
        self.t, self.dtype, self.name = t, dtype, name
        self.shape = None if shape is None else tuple(int(q) for q in shape)


def _dev(t, dtype, name, shape=None):
    return _T(t, dtype, name, shape)


def _call(fn, *args):
    """Call the library function `fn` with tensors given as _T.  The C ABI gets plain pointers
    and sizes: a tensor smaller than the sizes passed beside it would be read or written past
    its end by the kernels, so every tensor's type, shape and layout is checked first, for all
    arguments (host tensors included: shape errors come before the complaint that a tensor is
    not on the device), and nothing is launched unless all of them pass."""
    specs = [a for a in args if isinstance(a, _T)]
    for a in specs:
        if not isinstance(a.t, torch.Tensor):
            raise TypeError(f"{a.name} must be a tensor")
        if a.shape is not None and tuple(a.t.shape) != a.shape:
            raise ValueError(f"{a.name} must have shape {a.shape}, got {tuple(a.t.shape)}")
        if a.t.dtype != a.dtype:
            raise TypeError(f"{a.name} must be {a.dtype}, got {a.t.dtype}")
        if not a.t.is_contiguous():
            raise ValueError(f"{a.name} must be contiguous")
    for a in specs:
        if not a.t.is_cuda:
            raise TypeError(f"{a.name} must be a device tensor")
    raw = [a.t.data_ptr() if isinstance(a, _T) else _stream_now(a.stream) if isinstance(a, _S) else a
           for a in args]
    st = getattr(load(), fn)(*raw)
    if st != MOLORA_OK:
        raise MoloraError(st, fn)


def _stream_now(stream):
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


class _S:
    """The stream argument of a _call, resolved after the tensors have been checked."""

    def __init__(self, stream):
        self.stream = stream


def _stream(stream):
    return _S(stream)


def _two(t, name):
    if not isinstance(t, torch.Tensor) or t.dim() != 2:
        raise ValueError(f"{name} must be a 2-D tensor")
    return int(t.shape[0]), int(t.shape[1])


def _three(t, name):
    if not isinstance(t, torch.Tensor) or t.dim() != 3:
        raise ValueError(f"{name} must be a 3-D tensor")
    return int(t.shape[0]), int(t.shape[1]), int(t.shape[2])


def _breaks(breaks):
    b = [int(q) for q in breaks]
    if len(b) < 2:
        raise ValueError("breaks must hold at least two boundaries")
    return (ctypes.c_int32 * len(b))(*b), len(b) - 1


def _opt(t, dtype, name, shape=None):
    return None if t is None else _dev(t, dtype, name, shape)


def molora_route(x, G, r=None, stream=None):
    """r[i] = argmax_c x[i] . G[:, c] (fp32 ascending-k chain, lowest index on ties)."""
    N, d_in = _two(x, "x")
    C = _two(G, "G")[1]
    if r is None:
        r = torch.empty(N, dtype=torch.int32, device=x.device)
    _call("molora_route", _dev(x, torch.bfloat16, "x"), _dev(G, torch.bfloat16, "G", (d_in, C)),
                             _dev(r, torch.int32, "r", (N,)), N, d_in, C, _stream(stream))
    return r


def molora_route_vocab(v, breaks, r=None, stream=None):
    """r[i] = m with breaks[m] <= v[i] < breaks[m+1], else -1.  breaks: host ints."""
    N = int(v.shape[0])
    arr, M = _breaks(breaks)
    if r is None:
        r = torch.empty(N, dtype=torch.int32, device=v.device)
    _call("molora_route_vocab", _dev(v, torch.int32, "v", (N,)), arr, M, _dev(r, torch.int32, "r", (N,)), N,
                                   _stream(stream))
    return r


def molora_bucket(r, C, offsets=None, perm=None, err_flag=None, stream=None):
    """Stable grouping of tokens by target: returns (offsets[C+1], perm[N])."""
    N = int(r.shape[0])
    C = int(C)
    if offsets is None:
        offsets = torch.empty(C + 1, dtype=torch.int32, device=r.device)
    if perm is None:
        perm = torch.empty(max(N, 1), dtype=torch.int32, device=r.device)[:N]
    _call("molora_bucket", _dev(r, torch.int32, "r", (N,)), _dev(offsets, torch.int32, "offsets", (C + 1,)),
                              _dev(perm, torch.int32, "perm", (N,)), N, C,
                              _opt(err_flag, torch.int32, "err_flag"), _stream(stream))
    return offsets, perm


def molora_apply_workspace_bytes(N, d_in, d_out, C, rank):
    return int(load().molora_apply_workspace_bytes(N, d_in, d_out, C, rank))


def _shapes(x, W, A, B):
    N, d_in = _two(x, "x")
    d_out = _two(W, "W")[1]
    C, _, rank = _three(A, "A")
    _three(B, "B")
    if W.shape[0] != d_in or A.shape[1] != d_in or tuple(B.shape) != (C, rank, d_out):
        raise ValueError("expected W [d_in][d_out], A [C][d_in][rank], B [C][rank][d_out]")
    return N, d_in, d_out, C, rank


def new_workspace(N, d_in, d_out, C, rank, device="cuda"):
    nbytes = molora_apply_workspace_bytes(N, d_in, d_out, C, rank)
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)


def _flat_bytes(t, name):
    if not isinstance(t, torch.Tensor) or t.dim() != 1:
        raise ValueError(f"{name} must be a 1-D uint8 tensor")
    return _dev(t, torch.uint8, name), t.numel()


def molora_apply(x, W, A, B, r, h=None, workspace=None, stream=None):
    """h[i] = x[i] W + (x[i] A[r[i]]) B[r[i]]  (fp32 [N][d_out])."""
    N, d_in, d_out, C, rank = _shapes(x, W, A, B)
    if h is None:
        h = torch.empty((N, d_out), dtype=torch.float32, device=x.device)
    if workspace is None:
        workspace = new_workspace(N, d_in, d_out, C, rank, x.device)
    bf = torch.bfloat16
    ws, ws_bytes = _flat_bytes(workspace, "workspace")
    _call("molora_apply", _dev(x, bf, "x"), _dev(W, bf, "W"), _dev(A, bf, "A"), _dev(B, bf, "B"),
                             _dev(r, torch.int32, "r", (N,)), _dev(h, torch.float32, "h", (N, d_out)),
                             N, d_in, d_out, C, rank, ws, ws_bytes, _stream(stream))
    return h


def molora_apply_static(x, W, A, B, r, h, stream=None):
    """molora_apply on the library's own fixed scratch array: no workspace argument and no
    allocation anywhere in the call, so h must be supplied."""
    N, d_in, d_out, C, rank = _shapes(x, W, A, B)
    bf = torch.bfloat16
    _call("molora_apply_static", _dev(x, bf, "x"), _dev(W, bf, "W"), _dev(A, bf, "A"),
                                    _dev(B, bf, "B"), _dev(r, torch.int32, "r", (N,)),
                                    _dev(h, torch.float32, "h", (N, d_out)), N, d_in, d_out, C, rank,
                                    _stream(stream))
    return h


def molora_apply_bucketed(x, W, A, B, offsets, perm, h=None, workspace=None, stream=None):
    """molora_apply for a caller that already holds molora_bucket's output."""
    N, d_in, d_out, C, rank = _shapes(x, W, A, B)
    if h is None:
        h = torch.empty((N, d_out), dtype=torch.float32, device=x.device)
    if workspace is None:
        workspace = new_workspace(N, d_in, d_out, C, rank, x.device)
    bf = torch.bfloat16
    ws, ws_bytes = _flat_bytes(workspace, "workspace")
    _call("molora_apply_bucketed", 
        _dev(x, bf, "x"), _dev(W, bf, "W"), _dev(A, bf, "A"), _dev(B, bf, "B"),
        _dev(offsets, torch.int32, "offsets", (C + 1,)), _dev(perm, torch.int32, "perm", (N,)),
        _dev(h, torch.float32, "h", (N, d_out)), N, d_in, d_out, C, rank, ws, ws_bytes, _stream(stream))
    return h


def molora_shrink_workspace(N, d_in, C, rank, device="cuda"):
    """Scratch for molora_shrink (None when these sizes need none)."""
    nbytes = int(load().molora_shrink_workspace_bytes(N, d_in, C, rank))
    return torch.empty(nbytes, dtype=torch.uint8, device=device) if nbytes else None


def molora_shrink(x, A, offsets, perm, t=None, workspace="auto", stream=None):
    """t[p] = x[perm[p]] A_c as [hi | lo] bf16 halves, [N][2*rank].  workspace: a tensor from
    molora_shrink_workspace, None (never split K over workgroups) or "auto" (allocate)."""
    N, d_in = _two(x, "x")
    C, _, rank = _three(A, "A")
    if t is None:
        t = torch.empty((N, 2 * rank), dtype=torch.bfloat16, device=x.device)
    if isinstance(workspace, str):
        workspace = molora_shrink_workspace(N, d_in, C, rank, x.device)
    bf = torch.bfloat16
    ws, ws_bytes = (None, 0) if workspace is None else _flat_bytes(workspace, "workspace")
    _call("molora_shrink", _dev(x, bf, "x"), _dev(A, bf, "A", (C, d_in, rank)),
                              _dev(offsets, torch.int32, "offsets", (C + 1,)),
                              _dev(perm, torch.int32, "perm", (N,)), _dev(t, bf, "t", (N, 2 * rank)),
                              N, d_in, C, rank, ws, ws_bytes, _stream(stream))
    return t


def _base_expand_args(x, W, B, t, offsets, perm, h, t_cols):
    N, d_in = _two(x, "x")
    d_out = _two(W, "W")[1]
    C, rank, _ = _three(B, "B")
    if h is None:
        h = torch.empty((N, d_out), dtype=torch.float32, device=x.device)
    bf = torch.bfloat16
    args = [_dev(x, bf, "x"), _dev(W, bf, "W", (d_in, d_out)), _dev(B, bf, "B", (C, rank, d_out)),
            _dev(t, bf, "t", (N, t_cols(C, rank))), _dev(offsets, torch.int32, "offsets", (C + 1,)),
            _dev(perm, torch.int32, "perm", (N,)), _dev(h, torch.float32, "h", (N, d_out)),
            N, d_in, d_out, C, rank]
    return args, h


def molora_base_expand(x, W, B, t, offsets, perm, h=None, stream=None, tile_rows=None):
    """h[perm[p]] = x[perm[p]] W + t_p B_c, every row written once.  tile_rows (64, 128 or
    256) forces the row-tile height (molora_base_expand_fixed, for the tiling ablation)."""
    args, h = _base_expand_args(x, W, B, t, offsets, perm, h, lambda C, rank: 2 * rank)
    if tile_rows is None:
        _call("molora_base_expand", *args, _stream(stream))
    else:
        _call("molora_base_expand_fixed", *args, int(tile_rows), _stream(stream))
    return h


def molora_dense_shrink_supported(N, d_in, C, rank):
    """Whether dispatch and shrink can run in one launch for these sizes (C * rank <= 64, N > 512)."""
    return bool(load().molora_dense_shrink_supported(N, d_in, C, rank))


def _dense_outputs(N, C, rank, offsets, perm, t, device):
    if offsets is None:
        offsets = torch.empty(C + 1, dtype=torch.int32, device=device)
    if perm is None:
        perm = torch.empty(N, dtype=torch.int32, device=device)
    if t is None:
        t = torch.empty((N, 2 * C * rank), dtype=torch.bfloat16, device=device)
    return offsets, perm, t


def molora_bucket_shrink(r, x, A, offsets=None, perm=None, t=None, err_flag=None, stream=None):
    """Dispatch (r given) and token-order shrink in one launch: (offsets, perm, t [N][2*C*rank])."""
    N, d_in = _two(x, "x")
    C, _, rank = _three(A, "A")
    offsets, perm, t = _dense_outputs(N, C, rank, offsets, perm, t, x.device)
    bf = torch.bfloat16
    _call("molora_bucket_shrink", _dev(r, torch.int32, "r", (N,)), _dev(x, bf, "x"),
                                     _dev(A, bf, "A", (C, d_in, rank)),
                                     _dev(offsets, torch.int32, "offsets", (C + 1,)),
                                     _dev(perm, torch.int32, "perm", (N,)),
                                     _dev(t, bf, "t", (N, 2 * C * rank)), N, d_in, C, rank,
                                     _opt(err_flag, torch.int32, "err_flag"), _stream(stream))
    return offsets, perm, t


def molora_bucket_shrink_small_supported(N, d_in, C, rank):
    """Whether dispatch and shrink of a batch can run in one launch (N <= 64, rank above 32)."""
    return bool(load().molora_bucket_shrink_small_supported(N, d_in, C, rank))


def molora_bucket_shrink_small(r, x, A, offsets=None, perm=None, t=None, workspace="auto", err_flag=None,
                               stream=None):
    """molora_bucket + molora_shrink of a batch of at most 64 tokens in one launch:
    (offsets, perm, t [N][2*rank] in bucket order, as molora_shrink writes it)."""
    N, d_in = _two(x, "x")
    C, _, rank = _three(A, "A")
    if offsets is None:
        offsets = torch.empty(C + 1, dtype=torch.int32, device=x.device)
    if perm is None:
        perm = torch.empty(N, dtype=torch.int32, device=x.device)
    if t is None:
        t = torch.empty((N, 2 * rank), dtype=torch.bfloat16, device=x.device)
    if isinstance(workspace, str):
        workspace = molora_shrink_workspace(N, d_in, C, rank, x.device)
    bf = torch.bfloat16
    ws, ws_bytes = (None, 0) if workspace is None else _flat_bytes(workspace, "workspace")
    _call("molora_bucket_shrink_small", _dev(r, torch.int32, "r", (N,)), _dev(x, bf, "x"),
          _dev(A, bf, "A", (C, d_in, rank)), _dev(offsets, torch.int32, "offsets", (C + 1,)),
          _dev(perm, torch.int32, "perm", (N,)), _dev(t, bf, "t", (N, 2 * rank)), N, d_in, C, rank,
          ws, ws_bytes, _opt(err_flag, torch.int32, "err_flag"), _stream(stream))
    return offsets, perm, t


def molora_pack_w_cols(d_out):
    """Columns per group of the packed form of a base weight with d_out columns (0: none)."""
    return int(load().molora_pack_w_cols(int(d_out)))


def molora_pack_w(W, Wp=None, stream=None):
    """W [d_in][d_out] -> Wp, the same elements in the order molora_shrink_base_small(packed=True)
    streams: pieces of 64 rows, and inside a piece groups of molora_pack_w_cols(d_out) columns one
    after the other (done once per weight).  Wp has W's shape; row 64 u starts piece u."""
    d_in, d_out = _two(W, "W")
    if molora_pack_w_cols(d_out) == 0:
        raise ValueError(f"a base weight with {d_out} columns has no packed form")
    if Wp is None:
        Wp = torch.empty_like(W)
    bf = torch.bfloat16
    _call("molora_pack_w", _dev(W, bf, "W"), _dev(Wp, bf, "Wp", (d_in, d_out)), d_in, d_out, _stream(stream))
    return Wp


def molora_shrink_base_small(r, x, W, A, offsets=None, perm=None, t=None, h=None, err_flag=None, stream=None,
                             packed=False):
    """A batch of at most 64 tokens: dispatch, shrink and h = x W in one launch:
    (offsets, perm, t [N][2*rank] in bucket order, h [N][d_out] holding the base projection).
    packed=True: W is the output of molora_pack_w."""
    N, d_in = _two(x, "x")
    d_out = _two(W, "W")[1]
    if packed and molora_pack_w_cols(d_out) == 0:
        raise ValueError(f"a base weight with {d_out} columns has no packed form")
    C, _, rank = _three(A, "A")
    if offsets is None:
        offsets = torch.empty(C + 1, dtype=torch.int32, device=x.device)
    if perm is None:
        perm = torch.empty(N, dtype=torch.int32, device=x.device)
    if t is None:
        t = torch.empty((N, 2 * rank), dtype=torch.bfloat16, device=x.device)
    if h is None:
        h = torch.empty((N, d_out), dtype=torch.float32, device=x.device)
    bf = torch.bfloat16
    _call("molora_shrink_base_small_packed" if packed else "molora_shrink_base_small",
          _dev(r, torch.int32, "r", (N,)), _dev(x, bf, "x"),
          _dev(W, bf, "W", (d_in, d_out)), _dev(A, bf, "A", (C, d_in, rank)),
          _dev(offsets, torch.int32, "offsets", (C + 1,)), _dev(perm, torch.int32, "perm", (N,)),
          _dev(t, bf, "t", (N, 2 * rank)), _dev(h, torch.float32, "h", (N, d_out)), N, d_in, d_out, C, rank,
          _opt(err_flag, torch.int32, "err_flag"), _stream(stream))
    return offsets, perm, t, h


def molora_pack_b(B, Bp=None, stream=None):
    """B [C][rank][d_out] -> the same elements in the order molora_expand_small(packed=True) streams
    (molora_pack_w on the stacked [C * rank][d_out] matrix; rank a multiple of 16)."""
    C, rank, d_out = _three(B, "B")
    if rank % 16 != 0:
        raise ValueError(f"a packed B needs a rank that is a multiple of 16, not {rank}")
    if Bp is None:
        Bp = torch.empty_like(B)
    _three(Bp, "Bp")
    if tuple(Bp.shape) != tuple(B.shape):
        raise ValueError(f"Bp has shape {tuple(Bp.shape)}, B {tuple(B.shape)}")
    molora_pack_w(B.view(C * rank, d_out), Bp.view(C * rank, d_out), stream=stream)
    return Bp


def molora_expand_small(B, t, offsets, perm, h, stream=None, packed=False):
    """h[perm[p]] += t_p B_c (a batch of at most 64 tokens; after molora_shrink_base_small).
    packed=True: B is the output of molora_pack_b."""
    C, rank, d_out = _three(B, "B")
    N = int(h.shape[0])
    if packed and (rank % 16 != 0 or molora_pack_w_cols(d_out) == 0):
        raise ValueError(f"no packed form of B for rank {rank}, {d_out} columns")
    bf = torch.bfloat16
    _call("molora_expand_small_packed" if packed else "molora_expand_small", _dev(B, bf, "B"),
          _dev(t, bf, "t", (N, 2 * rank)),
          _dev(offsets, torch.int32, "offsets", (C + 1,)), _dev(perm, torch.int32, "perm", (N,)),
          _dev(h, torch.float32, "h", (N, d_out)), N, d_out, C, rank, _stream(stream))
    return h


def molora_gate_dispatch_shrink(v, breaks, x, A, adapter=None, n_adapters=1, r=None, offsets=None, perm=None,
                                t=None, err_flag=None, stream=None):
    """Vocabulary / compositional gating, dispatch and token-order shrink in one launch:
    (r, offsets, perm, t [N][2*C*rank]) with C = n_adapters * M."""
    N, d_in = _two(x, "x")
    C, _, rank = _three(A, "A")
    arr, M = _breaks(breaks)
    if C != n_adapters * M:
        raise ValueError("A must hold n_adapters * M adapters")
    if r is None:
        r = torch.empty(N, dtype=torch.int32, device=x.device)
    offsets, perm, t = _dense_outputs(N, C, rank, offsets, perm, t, x.device)
    bf = torch.bfloat16
    _call("molora_gate_dispatch_shrink", 
        _dev(v, torch.int32, "v", (N,)), _opt(adapter, torch.int32, "adapter", (N,)), arr, M,
        n_adapters, _dev(x, bf, "x"), _dev(A, bf, "A", (C, d_in, rank)), _dev(r, torch.int32, "r", (N,)),
        _dev(offsets, torch.int32, "offsets", (C + 1,)), _dev(perm, torch.int32, "perm", (N,)),
        _dev(t, bf, "t", (N, 2 * C * rank)), N, d_in, rank,
        _opt(err_flag, torch.int32, "err_flag"), _stream(stream))
    return r, offsets, perm, t


def molora_base_expand_dense(x, W, B, t, offsets, perm, h=None, stream=None):
    """molora_base_expand reading the token-order intermediate of the two calls above."""
    args, h = _base_expand_args(x, W, B, t, offsets, perm, h, lambda C, rank: 2 * C * rank)
    _call("molora_base_expand_dense", *args, _stream(stream))
    return h


def molora_init():
    """Once-per-device set-up (needed only before a stream capture made with the HIP API)."""
    _check(load().molora_init(), "molora_init")


def bf16_tensor(bits, device="cuda"):
    """numpy uint16 bit patterns -> torch.bfloat16 tensor on the device (same bits).  Anything
    but uint16 is refused: reinterpreting wider elements would silently change the shape."""
    import numpy as np
    bits = np.ascontiguousarray(bits)
    if bits.dtype != np.uint16:
        raise TypeError(f"bf16_tensor takes uint16 bit patterns, got {bits.dtype}")
    t = torch.from_numpy(bits.view(np.int16))
    return t.to(device).view(torch.bfloat16)


def molora_route_mlp(x, W1, b1, W2, b2, k, idx=None, w=None, workspace=None, stream=None):
    """Router MLP + top-k + softmax: returns (idx [N][k] int32, w [N][k] fp32)."""
    N, d_in = _two(x, "x")
    H, K = _two(W2, "W2")
    k = int(k)
    if idx is None:
        idx = torch.empty((N, k), dtype=torch.int32, device=x.device)
    if w is None:
        w = torch.empty((N, k), dtype=torch.float32, device=x.device)
    if workspace is None:
        nbytes = int(load().molora_route_mlp_workspace_bytes(N, H))
        workspace = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=x.device)
    bf = torch.bfloat16
    ws, ws_bytes = _flat_bytes(workspace, "workspace")
    _call("molora_route_mlp", _dev(x, bf, "x"), _dev(W1, bf, "W1", (d_in, H)),
                                 _dev(b1, torch.float32, "b1", (H,)), _dev(W2, bf, "W2"),
                                 _dev(b2, torch.float32, "b2", (K,)), _dev(idx, torch.int32, "idx", (N, k)),
                                 _dev(w, torch.float32, "w", (N, k)), N, d_in, H, K, k, ws, ws_bytes,
                                 _stream(stream))
    return idx, w


def molora_route_compose(v, adapter, breaks, n_adapters, r=None, stream=None):
    """r[i] = adapter[i] * M + modality(v[i]), -1 when either part is out of range."""
    N = int(v.shape[0])
    arr, M = _breaks(breaks)
    if r is None:
        r = torch.empty(N, dtype=torch.int32, device=v.device)
    _call("molora_route_compose", _dev(v, torch.int32, "v", (N,)), _dev(adapter, torch.int32, "adapter", (N,)),
                                     arr, M, n_adapters, _dev(r, torch.int32, "r", (N,)), N, _stream(stream))
    return r


def molora_gate_dispatch(v, breaks, adapter=None, n_adapters=1, r=None, offsets=None, perm=None,
                         err_flag=None, stream=None):
    """Vocabulary / compositional gating and bucketing in one launch: (r, offsets, perm)."""
    N = int(v.shape[0])
    arr, M = _breaks(breaks)
    C = n_adapters * M
    if r is None:
        r = torch.empty(N, dtype=torch.int32, device=v.device)
    if offsets is None:
        offsets = torch.empty(C + 1, dtype=torch.int32, device=v.device)
    if perm is None:
        perm = torch.empty(max(N, 1), dtype=torch.int32, device=v.device)[:N]
    _call("molora_gate_dispatch", 
        _dev(v, torch.int32, "v", (N,)), _opt(adapter, torch.int32, "adapter", (N,)),
        arr, M, n_adapters, _dev(r, torch.int32, "r", (N,)), _dev(offsets, torch.int32, "offsets", (C + 1,)),
        _dev(perm, torch.int32, "perm", (N,)), N,
        _opt(err_flag, torch.int32, "err_flag"), _stream(stream))
    return r, offsets, perm


def molora_apply_mix(x, W, A, B, idx, w=None, slots=None, C=None, h=None, workspace=None, stream=None):
    """h[i] = x[i] W + sum_j w[i][j] (x[i] A_s) B_s, s = slots[idx[i][j]] (slots None: idx)."""
    N, d_in, d_out, S, rank = _shapes(x, W, A, B)
    if idx.dim() == 1:
        idx = idx.reshape(N, 1)
    k = int(idx.shape[1])
    if C is None:
        C = S if slots is None else int(slots.shape[0])
    if slots is None and C > S:
        raise ValueError("without a slot table the adapter indices address the pool: C <= pool size")
    if h is None:
        h = torch.empty((N, d_out), dtype=torch.float32, device=x.device)
    if workspace is None:
        nbytes = int(load().molora_apply_mix_workspace_bytes(N, d_in, d_out, C, rank, k))
        workspace = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=x.device)
    bf = torch.bfloat16
    ws, ws_bytes = _flat_bytes(workspace, "workspace")
    _call("molora_apply_mix", 
        _dev(x, bf, "x"), _dev(W, bf, "W"), _dev(A, bf, "A"), _dev(B, bf, "B"),
        _dev(idx, torch.int32, "idx", (N, k)), _opt(w, torch.float32, "w", (N, k)),
        _opt(slots, torch.int32, "slots", (C,)), _dev(h, torch.float32, "h", (N, d_out)),
        N, d_in, d_out, C, rank, k, ws, ws_bytes, _stream(stream))
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
                _check(load().molora_graph_begin(_stream_now(graph.stream)), "molora_graph_begin")

            def __exit__(self, et, ev, tb):
                h = ctypes.c_void_p()
                st = load().molora_graph_end(_stream_now(graph.stream), ctypes.byref(h))
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
        _check(load().molora_graph_launch(self._handle, _stream_now(stream or self.stream)),
               "molora_graph_launch")

    def destroy(self):
        if self._handle is not None:
            load().molora_graph_destroy(self._handle)
            self._handle = None


class LaunchTimer:
    """Device-side duration of one base-projection launch (what a kernel trace reports):

        t = LaunchTimer()
        t.arm(); molora_base_expand(...)     # the call's GEMM launch records its own start and end
        us = t.elapsed_us()                  # waits for that launch
    """

    def __init__(self):
        h = ctypes.c_void_p()
        _check(load().molora_launch_timer_create(ctypes.byref(h)), "molora_launch_timer_create")
        self._handle = h

    def arm(self):
        _check(load().molora_launch_timer_arm(self._handle), "molora_launch_timer_arm")

    def elapsed_us(self):
        us = ctypes.c_double()
        _check(load().molora_launch_timer_elapsed_us(self._handle, ctypes.byref(us)), "molora_launch_timer_elapsed_us")
        return float(us.value)

    def destroy(self):
        if self._handle is not None:
            load().molora_launch_timer_destroy(self._handle)
            self._handle = None
