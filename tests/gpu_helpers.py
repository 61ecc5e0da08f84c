"""Helpers shared by the GPU parity tests: run the HIP library (through its C ABI binding)
and the CPU oracle on the same seeded inputs and compare."""
import numpy as np
import torch

import oracle
from paper_2603_15965_amd import binding as mb

TOL_REL_RMS = 1e-2     # the build's stated bar: max|h_gpu - h_oracle| <= 1e-2 * RMS(h_oracle)


def dev_bf16(bits):
    return mb.bf16_tensor(bits, "cuda")


def dev_i32(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()


def rms(a):
    return float(np.sqrt(np.mean(np.asarray(a, dtype=np.float64) ** 2)))


def gpu_route(wl):
    if wl.G is not None:
        return mb.molora_route(dev_bf16(wl.x), dev_bf16(wl.G))
    if wl.v is not None:
        return mb.molora_route_vocab(dev_i32(wl.v), wl.breaks)
    return dev_i32(wl.r)


def oracle_route(wl):
    if wl.G is not None:
        return oracle.route_gate(wl.x, wl.G)
    if wl.v is not None:
        return oracle.route_vocab(wl.v, wl.breaks)
    return wl.r


def check_bucket(r_np, C):
    r_d = dev_i32(r_np)
    flag = torch.zeros(1, dtype=torch.int32, device="cuda")
    offsets, perm = mb.molora_bucket(r_d, C, err_flag=flag)
    torch.cuda.synchronize()
    o_ref, p_ref, bad = oracle.bucket(r_np, C)
    assert np.array_equal(offsets.cpu().numpy(), o_ref), "offsets differ"
    assert np.array_equal(perm.cpu().numpy(), p_ref), "perm differs"
    assert int(flag.item()) == (1 if bad else 0)
    return offsets, perm


def gpu_apply(wl, r_np, bucketed=False):
    x, W, A, B = dev_bf16(wl.x), dev_bf16(wl.W), dev_bf16(wl.A), dev_bf16(wl.B)
    r_d = dev_i32(r_np)
    if bucketed:
        offsets, perm = mb.molora_bucket(r_d, wl.shape.C)
        h = mb.molora_apply_bucketed(x, W, A, B, offsets, perm)
    else:
        h = mb.molora_apply(x, W, A, B, r_d)
    torch.cuda.synchronize()
    return h


def assert_h_close(h_gpu_rows, h_ref_rows, what=""):
    h_gpu_rows = np.asarray(h_gpu_rows)
    assert h_gpu_rows.shape == h_ref_rows.shape
    assert np.all(np.isfinite(h_gpu_rows)), f"{what}: non-finite output"
    scale = rms(h_ref_rows)
    err = float(np.max(np.abs(h_gpu_rows.astype(np.float64) - h_ref_rows.astype(np.float64)))) if h_ref_rows.size else 0.0
    assert err <= TOL_REL_RMS * scale, f"{what}: max err {err:.3e} > {TOL_REL_RMS} * rms {scale:.3e}"
    return err / scale if scale else 0.0
