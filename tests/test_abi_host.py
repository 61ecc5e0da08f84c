"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol
the header declares, and rejects bad arguments before anything is enqueued."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2603_15965_amd import binding, build
    if not os.path.exists(binding.LIB_PATH):
        build.build()
    return binding.load()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "molora.h")).read()
    body = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(molora_[a-z_]+)\s*\(", body))
    assert {"molora_route", "molora_route_vocab", "molora_bucket", "molora_apply",
            "molora_apply_bucketed", "molora_apply_workspace_bytes",
            "molora_status_string", "molora_version"} <= declared
    for name in declared:
        assert hasattr(lib, name), f"{name} declared in molora.h but not exported"
    from paper_2603_15965_amd import binding
    assert set(binding.EXPORTS) <= declared


def test_status_strings(lib):
    from paper_2603_15965_amd import binding
    assert binding.status_string(0) == "ok"
    assert "workspace" in binding.status_string(-3)
    assert binding.version().startswith("molora-gfx950")


def test_workspace_size_formula(lib):
    f = lib.molora_apply_workspace_bytes
    # offsets + perm + t as [hi | lo] bf16 (+ the scratch of a K-split shrink), each rounded up
    # to 256 bytes
    r256 = lambda b: (b + 255) // 256 * 256
    g = lib.molora_shrink_workspace_bytes
    for (N, di, do, C, rk) in [(256, 256, 256, 4, 8), (16384, 4096, 12288, 32, 32), (64, 4096, 12288, 16, 64)]:
        assert f(N, di, do, C, rk) == r256(4 * (C + 1)) + r256(4 * N) + r256(N * 2 * rk * 2) + g(N, di, C, rk)
    # a few dozen tokens, long K, wide intermediate: four K slices of fp32 partial sums
    assert g(64, 4096, 16, 64) == 4 * 64 * 64 * 4
    assert g(16384, 4096, 32, 32) == 0 and g(256, 256, 4, 8) == 0 and g(0, 4096, 16, 64) == 0
    assert g(64, 4096, 16, 60) == 0          # rank not a multiple of 8
    assert f(16, 10, 64, 4, 8) == 0          # d_in not a multiple of 8
    assert f(16, 64, 64, 4, 12) == 0         # rank not a multiple of 8
    assert f(16, 64, 64, 4, 256) == 0        # rank above the limit
    assert f(16, 64, 64, 0, 8) == 0
    assert f(-1, 64, 64, 4, 8) == 0


def test_bad_arguments_are_rejected_before_launch(lib):
    EINVAL, EALIGN, EWORKSPACE = -1, -2, -3
    p = ctypes.c_void_p
    buf = (ctypes.c_char * 4096)()
    a = ctypes.addressof(buf)
    a += (-a) % 256                                       # a 256-byte aligned fake pointer
    assert lib.molora_route(None, p(a), p(a), 16, 64, 4, None) == EINVAL
    assert lib.molora_route(p(a), p(a), p(a), 16, 60, 4, None) == EINVAL     # d_in % 8
    assert lib.molora_route(p(a), p(a), p(a), 16, 64, 2000, None) == EINVAL  # C too large
    assert lib.molora_route(p(a + 2), p(a), p(a), 16, 64, 4, None) == EALIGN
    assert lib.molora_route(None, None, None, 0, 64, 4, None) == 0           # N = 0 is a no-op
    br = (ctypes.c_int32 * 3)(0, 10, 10)
    assert lib.molora_route_vocab(p(a), br, 2, p(a), 16, None) == EINVAL     # not increasing
    assert lib.molora_route_vocab(p(a), None, 2, p(a), 16, None) == EINVAL
    assert lib.molora_bucket(p(a), None, p(a), 16, 4, None, None) == EINVAL
    assert lib.molora_bucket(p(a), p(a), p(a), 16, 0, None, None) == EINVAL
    assert lib.molora_bucket(p(a), p(a + 4), p(a), 16, 4, None, None) == EALIGN
    args = lambda ws, nbytes, rank=8, x=a: (p(x), p(a), p(a), p(a), p(a), p(a), 16, 64, 64, 4, rank, p(ws), nbytes, None)
    assert lib.molora_apply(*args(a, 10)) == EWORKSPACE
    assert lib.molora_apply(*args(a + 16, 1 << 20)) == EALIGN
    assert lib.molora_apply(*args(a, 1 << 20, rank=12)) == EINVAL
    assert lib.molora_apply(*args(a, 1 << 20, x=0)) == EINVAL
    assert lib.molora_apply_bucketed(p(a), p(a), p(a), p(a), None, p(a), p(a), 16, 64, 64, 4, 8, p(a), 1 << 20, None) == EINVAL


def test_widened_entry_points_reject_bad_arguments(lib):
    EINVAL, EALIGN, EWORKSPACE = -1, -2, -3
    p = ctypes.c_void_p
    buf = (ctypes.c_char * 8192)()
    a = ctypes.addressof(buf)
    a += (-a) % 256
    r256 = lambda b: (b + 255) // 256 * 256
    # router MLP: hidden pre-activations are the only scratch
    f = lib.molora_route_mlp_workspace_bytes
    assert f(100, 64) == r256(100 * 64 * 4)
    assert f(100, 60) == 0 and f(100, 512) == 0 and f(-1, 64) == 0
    mlp = lambda k=2, H=64, K=8, ws=a, nb=1 << 20, x=a: lib.molora_route_mlp(
        p(x), p(a), p(a), p(a), p(a), p(a), p(a), 16, 64, H, K, k, p(ws), nb, None)
    assert mlp(k=0) == EINVAL and mlp(k=5) == EINVAL and mlp(k=3, K=2) == EINVAL
    assert mlp(H=12) == EINVAL and mlp(K=2000) == EINVAL
    assert mlp(x=0) == EINVAL
    assert mlp(ws=a + 16) == EALIGN
    assert mlp(nb=100) == EWORKSPACE
    # compositional gating
    br = (ctypes.c_int32 * 3)(0, 10, 20)
    bad = (ctypes.c_int32 * 3)(0, 10, 5)
    assert lib.molora_route_compose(p(a), p(a), bad, 2, 3, p(a), 16, None) == EINVAL
    assert lib.molora_route_compose(p(a), p(a), br, 2, 0, p(a), 16, None) == EINVAL
    assert lib.molora_route_compose(p(a), p(a), br, 2, 600, p(a), 16, None) == EINVAL   # 1200 targets
    assert lib.molora_route_compose(p(a), None, br, 2, 3, p(a), 16, None) == EINVAL
    assert lib.molora_route_compose(p(a + 4), p(a), br, 2, 3, p(a), 16, None) == EALIGN
    assert lib.molora_route_compose(None, None, br, 2, 3, None, 0, None) == 0
    assert lib.molora_gate_dispatch(p(a), None, bad, 2, 1, p(a), p(a), p(a), 16, None, None) == EINVAL
    assert lib.molora_gate_dispatch(p(a), None, br, 2, 1, p(a), None, p(a), 16, None, None) == EINVAL
    assert lib.molora_gate_dispatch(p(a), None, br, 2, 1, p(a), p(a + 4), p(a), 16, None, None) == EALIGN
    # mixture: tuples must fit the bucket limit, the stacked rank the rank limit
    g = lib.molora_apply_mix_workspace_bytes
    N, C, rk, k = 300, 8, 16, 2
    assert g(N, 64, 64, C, rk, k) == (r256(4 * N) + r256(4 * N * k) + r256(4 * (C ** k + 1)) + r256(4 * N)
                                      + r256(N * 2 * k * rk * 2))   # no K split at these sizes
    assert g(N, 64, 64, 40, rk, 2) == 0          # 1600 tuples
    assert g(N, 64, 64, 4, 64, 4) == 0           # stacked rank 256
    assert g(N, 64, 64, 4, 8, 5) == 0            # k above the limit
    assert g(N, 64, 64, C, rk, 1) == r256(4 * N) + r256(4 * N) + r256(4 * (C + 1)) + r256(4 * N) + r256(N * 2 * rk * 2)
    mix = lambda k=2, C=8, ws=a, nb=1 << 20, idx=a: lib.molora_apply_mix(
        p(a), p(a), p(a), p(a), p(idx), None, None, p(a), 16, 64, 64, C, 8, k, p(ws), nb, None)
    assert mix(k=0) == EINVAL and mix(C=40) == EINVAL and mix(idx=0) == EINVAL
    assert mix(ws=a + 16) == EALIGN
    assert mix(nb=64) == EWORKSPACE
    # recorded sequences: the null stream cannot be captured, NULL handles are rejected
    h = ctypes.c_void_p()
    assert lib.molora_graph_begin(None) == EINVAL
    assert lib.molora_graph_end(None, ctypes.byref(h)) == EINVAL
    assert lib.molora_graph_launch(None, None) == EINVAL
    lib.molora_graph_destroy(None)


def test_one_launch_dispatch_and_shrink_reject_bad_arguments(lib):
    EINVAL, EALIGN = -1, -2
    p = ctypes.c_void_p
    buf = (ctypes.c_char * 4096)()
    a = ctypes.addressof(buf)
    a += (-a) % 256
    small, dense = lib.molora_bucket_shrink_small_supported, lib.molora_dense_shrink_supported
    assert small(64, 4096, 16, 64) == 1 and small(1, 64, 4, 40) == 1
    assert small(65, 4096, 16, 64) == 0      # more than one wavefront of targets
    assert small(64, 4096, 16, 32) == 0      # narrow ranks take another shrink kernel
    assert small(0, 4096, 16, 64) == 0 and small(64, 4096, 16, 60) == 0
    assert dense(4096, 2048, 2, 16) == 1 and dense(4096, 2048, 4, 16) == 1
    assert dense(512, 2048, 2, 16) == 0 and dense(4096, 2048, 8, 16) == 0
    f = lib.molora_bucket_shrink_small
    call = lambda N=64, rank=64, r=a, t=a, ws=None: f(p(r), p(a), p(a), p(a), p(a), p(t), N, 4096, 16, rank,
                                                      ws, 0, None, None)
    assert call(N=65) == EINVAL and call(rank=32) == EINVAL and call(r=0) == EINVAL
    assert call(t=a + 8) == EALIGN
    k1 = lambda N=64, rank=64, W=a, h=a: lib.molora_shrink_base_small(p(a), p(a), p(W), p(a), p(a), p(a), p(a), p(h),
                                                                     N, 4096, 256, 16, rank, None, None)
    assert k1(N=65) == EINVAL and k1(rank=32) == EINVAL and k1(W=0) == EINVAL and k1(h=a + 4) == EALIGN
    k2 = lambda N=64, B=a, h=a: lib.molora_expand_small(p(B), p(a), p(a), p(a), p(h), N, 256, 16, 64, None)
    assert k2(N=65) == EINVAL and k2(B=0) == EINVAL and k2(h=a + 4) == EALIGN and k2(N=0) == 0
    g = lib.molora_bucket_shrink
    assert g(p(a), p(a), p(a), p(a), p(a), p(a), 64, 4096, 2, 16, None, None) == EINVAL   # N <= 512
    assert g(p(a), p(a), p(a), p(a), p(a), p(a), 4096, 2048, 8, 16, None, None) == EINVAL  # C * rank > 64
    assert g(None, p(a), p(a), p(a), p(a), p(a), 4096, 2048, 2, 16, None, None) == EINVAL


def test_packed_base_weight_entry_points_reject_bad_arguments(lib):
    """The packed form of a base weight exists for whole column groups only (64 columns, 32 up
    to d_out = 8192); everything else is an error before any launch."""
    EINVAL, EALIGN = -1, -2
    p = ctypes.c_void_p
    buf = (ctypes.c_char * 8192)()
    a = ctypes.addressof(buf)
    a += (-a) % 256
    b = a + 4096
    cols = lib.molora_pack_w_cols
    assert cols(64) == 32 and cols(8192) == 32 and cols(8256) == 64 and cols(12288) == 64
    assert cols(72) == 0 and cols(8200) == 0 and cols(8224) == 0 and cols(16) == 0 and cols(0) == 0 and cols(-64) == 0
    pack = lambda W=a, Wp=b, d_in=64, d_out=64: lib.molora_pack_w(p(W), p(Wp), d_in, d_out, None)
    assert pack(d_out=72) == EINVAL and pack(d_in=4) == EINVAL and pack(d_in=12) == EINVAL
    assert pack(W=0) == EINVAL and pack(Wp=0) == EINVAL and pack(Wp=a) == EINVAL   # in place: not supported
    assert pack(Wp=b + 8) == EALIGN
    k1 = lambda N=64, d_out=256, W=a: lib.molora_shrink_base_small_packed(
        p(a), p(a), p(W), p(a), p(a), p(a), p(a), p(a), N, 4096, d_out, 16, 64, None, None)
    assert k1(d_out=264) == EINVAL and k1(N=65) == EINVAL and k1(W=0) == EINVAL and k1(W=a + 8) == EALIGN
    k2 = lambda N=64, d_out=256, rank=64, B=a: lib.molora_expand_small_packed(p(B), p(a), p(a), p(a), p(a), N, d_out,
                                                                              16, rank, None)
    assert k2(rank=40) == EINVAL and k2(d_out=264) == EINVAL and k2(N=65) == EINVAL and k2(B=0) == EINVAL
    assert k2(B=a + 8) == EALIGN and k2(N=0) == 0


def test_operands_of_4_gib_are_rejected_for_the_tiled_kernel(lib):
    """The tiled GEMM (N > 512) keeps per-lane byte offsets into x and W in 32 bits; sizes
    beyond that are an error before launch, not silently wrapped addresses."""
    EINVAL, EWORKSPACE = -1, -3
    p = ctypes.c_void_p
    buf = (ctypes.c_char * 4096)()
    a = ctypes.addressof(buf)
    a += (-a) % 256
    f = lib.molora_apply
    call = lambda N, di, do: f(p(a), p(a), p(a), p(a), p(a), p(a), N, di, do, 4, 8, p(a), 16, None)
    assert call(1 << 20, 4096, 64) == EINVAL          # x = 8 GiB
    assert call(1 << 19, 4096, 64) == EINVAL          # x = 4 GiB exactly
    assert call((1 << 19) - 8, 4096, 64) == EWORKSPACE  # just below: passes the size check
    assert call(1024, 65536, 32768) == EINVAL         # W = 4 GiB
    assert call(1024, 65536, 32760) == EWORKSPACE
    assert call(512, 65536, 32768) == EWORKSPACE      # the small-batch kernel has no such limit
    be = lib.molora_base_expand
    assert be(p(a), p(a), p(a), p(a), p(a), p(a), p(a), 1 << 20, 4096, 64, 4, 8, None) == EINVAL
    fx = lib.molora_base_expand_fixed
    assert fx(p(a), p(a), p(a), p(a), p(a), p(a), p(a), 64, 65536, 32768, 4, 8, 256, None) == EINVAL
    assert fx(p(a), p(a), p(a), p(a), p(a), p(a), p(a), 64, 64, 64, 4, 8, 100, None) == EINVAL  # no such tile
    assert fx(None, None, None, None, None, None, None, 0, 64, 64, 4, 8, 128, None) == 0
