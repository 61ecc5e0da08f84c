"""The Python binding checks every tensor against the sizes it passes to the C ABI before
anything is launched (no GPU needed: shape and type errors are raised for host tensors too,
ahead of the complaint that a tensor is not on the device).  A kernel given sizes larger than
an allocation reads or writes past its end, which on a GPU is a memory fault, not an error
code."""
import numpy as np
import pytest
import torch

from paper_2603_15965_amd import binding as mb

bf, i32, f32 = torch.bfloat16, torch.int32, torch.float32
N, d_in, d_out, C, rank = 16, 64, 32, 2, 8


def tens(shape, dtype=bf):
    return torch.zeros(shape, dtype=dtype)


@pytest.fixture(scope="module", autouse=True)
def _lib():
    from paper_2603_15965_amd import build
    import os
    if not os.path.exists(mb.LIB_PATH):
        build.build()
    mb.load()


def good():
    return dict(x=tens((N, d_in)), W=tens((d_in, d_out)), A=tens((C, d_in, rank)), B=tens((C, rank, d_out)),
                r=tens((N,), i32), offsets=tens((C + 1,), i32), perm=tens((N,), i32),
                t=tens((N, 2 * rank)), td=tens((N, 2 * C * rank)), h=tens((N, d_out), f32),
                ws=tens((1 << 16,), torch.uint8))


def test_bf16_tensor_takes_bit_patterns_only():
    """Reinterpreting a float32 array as 16-bit patterns would double its last dimension: the
    tensor would then claim a d_in twice that of the other operands."""
    with pytest.raises(TypeError):
        mb.bf16_tensor(np.zeros((4, 8), np.float32), device="cpu")
    with pytest.raises(TypeError):
        mb.bf16_tensor(np.zeros((4, 8), np.int32), device="cpu")
    t = mb.bf16_tensor(np.full((4, 8), 0x3F80, np.uint16), device="cpu")
    assert t.shape == (4, 8) and t.dtype == bf and float(t[0, 0]) == 1.0


def test_right_shapes_pass_the_checks_and_stop_at_the_device_test():
    g = good()
    calls = [
        lambda: mb.molora_apply(g["x"], g["W"], g["A"], g["B"], g["r"], g["h"], g["ws"]),
        lambda: mb.molora_apply_bucketed(g["x"], g["W"], g["A"], g["B"], g["offsets"], g["perm"], g["h"], g["ws"]),
        lambda: mb.molora_apply_static(g["x"], g["W"], g["A"], g["B"], g["r"], g["h"]),
        lambda: mb.molora_shrink(g["x"], g["A"], g["offsets"], g["perm"], g["t"], workspace=None),
        lambda: mb.molora_base_expand(g["x"], g["W"], g["B"], g["t"], g["offsets"], g["perm"], g["h"]),
        lambda: mb.molora_base_expand_dense(g["x"], g["W"], g["B"], g["td"], g["offsets"], g["perm"], g["h"]),
        lambda: mb.molora_bucket_shrink(g["r"], g["x"], g["A"], g["offsets"], g["perm"], g["td"]),
        lambda: mb.molora_bucket(g["r"], C, g["offsets"], g["perm"]),
        lambda: mb.molora_route(g["x"], tens((d_in, C)), g["r"]),
    ]
    for f in calls:
        with pytest.raises(TypeError, match="device tensor"):
            f()


@pytest.mark.parametrize("which, shape", [
    ("W", (2 * d_in, d_out)), ("W", (d_in // 2, d_out)), ("A", (C, d_in // 2, rank)), ("A", (C, d_in, 2 * rank)),
    ("B", (C, rank, 2 * d_out)), ("B", (C + 1, rank, d_out)), ("r", (N - 1,)), ("h", (N, d_out - 8)),
    ("h", (N - 1, d_out)),
])
def test_apply_rejects_mismatched_shapes(which, shape):
    g = good()
    g[which] = tens(shape, g[which].dtype)
    with pytest.raises(ValueError):
        mb.molora_apply(g["x"], g["W"], g["A"], g["B"], g["r"], g["h"], g["ws"])
    with pytest.raises(ValueError):
        mb.molora_apply_static(g["x"], g["W"], g["A"], g["B"], g["r"], g["h"])


@pytest.mark.parametrize("which, shape", [
    ("A", (C, d_in // 2, rank)), ("offsets", (C,)), ("perm", (N // 2,)), ("t", (N, rank)), ("t", (N // 2, 2 * rank)),
])
def test_shrink_rejects_mismatched_shapes(which, shape):
    g = good()
    g[which] = tens(shape, g[which].dtype)
    with pytest.raises(ValueError):
        mb.molora_shrink(g["x"], g["A"], g["offsets"], g["perm"], g["t"], workspace=None)


@pytest.mark.parametrize("which, shape", [
    ("W", (d_in // 2, d_out)), ("W", (2 * d_in, d_out)), ("B", (C, rank, d_out // 2)), ("t", (N, rank)),
    ("offsets", (C,)), ("perm", (N - 1,)), ("h", (N, d_out // 2)),
])
def test_base_expand_rejects_mismatched_shapes(which, shape):
    g = good()
    g[which] = tens(shape, g[which].dtype)
    for tile in (None, 128):
        with pytest.raises(ValueError):
            mb.molora_base_expand(g["x"], g["W"], g["B"], g["t"], g["offsets"], g["perm"], g["h"], tile_rows=tile)
    g["t"] = g["td"] if which != "t" else g["t"]
    with pytest.raises(ValueError):
        mb.molora_base_expand_dense(g["x"], g["W"], g["B"], g["t"], g["offsets"], g["perm"], g["h"])


def test_one_launch_dispatch_and_shrink_reject_mismatched_shapes():
    g = good()
    v = tens((N,), i32)
    with pytest.raises(ValueError):   # the grouped form's t is too narrow for the token-order form
        mb.molora_bucket_shrink(g["r"], g["x"], g["A"], g["offsets"], g["perm"], g["t"])
    with pytest.raises(ValueError):
        mb.molora_bucket_shrink(tens((N + 1,), i32), g["x"], g["A"], g["offsets"], g["perm"], g["td"])
    with pytest.raises(ValueError):   # two modalities x one adapter = 2 buckets, A holds 3
        mb.molora_gate_dispatch_shrink(v, [0, 10, 20], g["x"], tens((3, d_in, rank)))
    with pytest.raises(ValueError):
        mb.molora_gate_dispatch_shrink(tens((N - 1,), i32), [0, 10, 20], g["x"], g["A"], t=g["td"])
    with pytest.raises(ValueError):
        mb.molora_gate_dispatch_shrink(v, [0, 10, 20], g["x"], g["A"], adapter=tens((N - 1,), i32))
    with pytest.raises(ValueError):
        mb.molora_gate_dispatch(v, [0], None, 1)
    with pytest.raises(ValueError):   # the small-batch form writes the bucket-order t
        mb.molora_bucket_shrink_small(g["r"], g["x"], g["A"], g["offsets"], g["perm"], g["td"], workspace=None)
    with pytest.raises(ValueError):
        mb.molora_bucket_shrink_small(g["r"], g["x"], g["A"], tens((C,), i32), g["perm"], g["t"], workspace=None)
    with pytest.raises(TypeError, match="device tensor"):
        mb.molora_bucket_shrink_small(g["r"], g["x"], g["A"], g["offsets"], g["perm"], g["t"], workspace=None)


def test_packed_base_weight_rejects_mismatched_shapes():
    g = good()
    assert mb.molora_pack_w_cols(d_out) == 32 and mb.molora_pack_w_cols(d_out + 8) == 0
    with pytest.raises(ValueError, match="no packed form"):
        mb.molora_pack_w(tens((d_in, d_out + 8)))
    with pytest.raises(ValueError):   # the packed weight has W's element count and shape
        mb.molora_pack_w(g["W"], tens((d_in, d_out // 2)))
    with pytest.raises(TypeError, match="device tensor"):
        mb.molora_pack_w(g["W"], tens((d_in, d_out)))
    with pytest.raises(ValueError, match="no packed form"):
        mb.molora_shrink_base_small(g["r"], g["x"], tens((d_in, d_out + 8)), g["A"], packed=True)
    with pytest.raises(ValueError):   # W of another d_in
        mb.molora_shrink_base_small(g["r"], g["x"], tens((d_in * 2, d_out)), g["A"], g["offsets"], g["perm"],
                                    g["t"], g["h"], packed=True)
    with pytest.raises(TypeError, match="device tensor"):
        mb.molora_shrink_base_small(g["r"], g["x"], g["W"], g["A"], g["offsets"], g["perm"], g["t"], g["h"],
                                    packed=True)
    B16 = tens((C, 16, d_out))
    with pytest.raises(ValueError, match="multiple of 16"):   # rank 8: a slab would straddle two adapters
        mb.molora_pack_b(g["B"])
    with pytest.raises(ValueError):
        mb.molora_pack_b(B16, tens((C, 16, d_out // 2)))
    with pytest.raises(TypeError, match="device tensor"):
        mb.molora_pack_b(B16)
    with pytest.raises(ValueError, match="no packed form"):
        mb.molora_expand_small(g["B"], g["t"], g["offsets"], g["perm"], g["h"], packed=True)
    with pytest.raises(ValueError):   # t of another rank
        mb.molora_expand_small(B16, g["t"], g["offsets"], g["perm"], g["h"], packed=True)
    with pytest.raises(TypeError, match="device tensor"):
        mb.molora_expand_small(B16, tens((N, 32)), g["offsets"], g["perm"], g["h"], packed=True)


def test_routes_and_mixture_reject_mismatched_shapes():
    g = good()
    with pytest.raises(ValueError):
        mb.molora_route(g["x"], tens((d_in // 2, C)), g["r"])
    with pytest.raises(ValueError):
        mb.molora_route(g["x"], tens((d_in, C)), tens((N - 1,), i32))
    with pytest.raises(ValueError):
        mb.molora_route_vocab(tens((N,), i32), [0, 5], tens((N + 1,), i32))
    with pytest.raises(ValueError):
        mb.molora_route_compose(tens((N,), i32), tens((N - 1,), i32), [0, 5], 2)
    with pytest.raises(ValueError):
        mb.molora_bucket(g["r"], C, tens((C,), i32), g["perm"])
    H, K = 16, 4
    mlp = dict(W1=tens((d_in, H)), b1=tens((H,), f32), W2=tens((H, K)), b2=tens((K,), f32))
    for which, shape in [("W1", (d_in // 2, H)), ("b1", (H - 1,)), ("b2", (K + 1,))]:
        m = dict(mlp)
        m[which] = tens(shape, mlp[which].dtype)
        with pytest.raises(ValueError):
            mb.molora_route_mlp(g["x"], m["W1"], m["b1"], m["W2"], m["b2"], 2, workspace=g["ws"])
    with pytest.raises(ValueError):
        mb.molora_route_mlp(g["x"], mlp["W1"], mlp["b1"], mlp["W2"], mlp["b2"], 2, idx=tens((N, 1), i32),
                            workspace=g["ws"])
    idx = tens((N, 2), i32)
    with pytest.raises(ValueError):
        mb.molora_apply_mix(g["x"], g["W"], g["A"], g["B"], idx, w=tens((N, 1), f32), workspace=g["ws"])
    with pytest.raises(ValueError):   # no slot table: indices address the pool of C adapters directly
        mb.molora_apply_mix(g["x"], g["W"], g["A"], g["B"], idx, C=C + 1, workspace=g["ws"])
    with pytest.raises(ValueError):
        mb.molora_apply_mix(g["x"], g["W"], g["A"], g["B"], idx, slots=tens((4,), i32), C=5, workspace=g["ws"])


def test_wrong_dtype_or_layout_is_rejected():
    g = good()
    with pytest.raises(TypeError):
        mb.molora_apply(g["x"].float(), g["W"], g["A"], g["B"], g["r"], g["h"], g["ws"])
    with pytest.raises(TypeError):
        mb.molora_apply(g["x"], g["W"], g["A"], g["B"], g["r"].long(), g["h"], g["ws"])
    with pytest.raises(ValueError):
        mb.molora_apply(g["x"], tens((d_out, d_in)).t(), g["A"], g["B"], g["r"], g["h"], g["ws"])
