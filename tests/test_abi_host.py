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
    # offsets + perm + t as [hi | lo] bf16, each rounded up to 256 bytes
    r256 = lambda b: (b + 255) // 256 * 256
    for (N, di, do, C, rk) in [(256, 256, 256, 4, 8), (16384, 4096, 12288, 32, 32), (64, 4096, 12288, 16, 64)]:
        assert f(N, di, do, C, rk) == r256(4 * (C + 1)) + r256(4 * N) + r256(N * 2 * rk * 2)
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
