"""Helpers shared by the GPU parity tests: run the HIP library (through its C ABI binding)
and the CPU oracle on the same seeded inputs and compare."""
import numpy as np
import torch

import oracle
from paper_2603_15965_amd import binding as mb

TOL_REL_RMS = 1e-2     # the build's stated bar: max|h_gpu - h_oracle| <= 1e-2 * RMS(h_oracle)
# Regression bound, asserted beside the bar.  Both sides accumulate exact bf16 x bf16 products in
# fp32 and differ only in the order of the additions; the rounding errors of a K-term sum add
# like a random walk, ~sqrt(K) * 2^-24 * |partial sums|, i.e. a few 1e-6 of the RMS per element
# and ~2e-5 at the maximum over 1e8 outputs with K up to 12288 (observed: 1.5e-5).  Ten times
# that still lies ten times below the smallest structural mistake the path can make (losing
# the low half of t costs 2e-3 of the RMS, one dropped k element of 12288 about 6e-3).
REGRESSION_REL_RMS = 2e-4


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
    assert err <= REGRESSION_REL_RMS * scale, \
        f"{what}: max err {err:.3e} is within the bar but above the regression bound " \
        f"{REGRESSION_REL_RMS} * rms {scale:.3e}"
    return err / scale if scale else 0.0


def bucket_column_sums_ref(wl, r):
    """sum over the tokens of every bucket of h, from the definition in float64:
    sum_{i in c} h_i = (sum_{i in c} x_i) (W + A_c B_c); row C holds the tokens without
    adapter, (sum x_i) W.  A linear functional of h that touches every element, cheap at any
    size."""
    from paper_2603_15965_amd import workloads as wlm
    C = wl.shape.C
    N, d_in = wl.x.shape
    key = np.where((r >= 0) & (r < C), r, C).astype(np.int64)
    xs = np.zeros((C + 1, d_in), dtype=np.float64)
    for lo in range(0, N, 2048):
        blk = wlm.bf16_bits_to_f32(wl.x[lo:lo + 2048]).astype(np.float64)
        onehot = np.zeros((C + 1, blk.shape[0]), dtype=np.float64)
        onehot[key[lo:lo + 2048], np.arange(blk.shape[0])] = 1.0
        xs += onehot @ blk
    out = xs @ wlm.bf16_bits_to_f32(wl.W).astype(np.float64)
    for c in range(C):
        if np.any(key == c):
            t = xs[c] @ wlm.bf16_bits_to_f32(wl.A[c]).astype(np.float64)
            out[c] += t @ wlm.bf16_bits_to_f32(wl.B[c]).astype(np.float64)
    return out, np.bincount(key, minlength=C + 1)


def check_bucket_column_sums(h, wl, r, what=""):
    """Whole-tensor check: per-bucket column sums of the GPU's h (accumulated in float64 on the
    device) against the float64 definition.  An element that is wrong by e moves one sum by e;
    the legitimate difference is the fp32 rounding of n independent elements, ~sqrt(n) * 1e-5
    of the RMS, so the bound sqrt(n) * 1e-4 * RMS(h) catches any tile of wrong values."""
    C = wl.shape.C
    ref, cnt = bucket_column_sums_ref(wl, r)
    key = torch.from_numpy(np.where((r >= 0) & (r < C), r, C).astype(np.int64)).cuda()
    got = torch.zeros((C + 1, h.shape[1]), dtype=torch.float64, device="cuda")
    for lo in range(0, h.shape[0], 4096):
        got.index_add_(0, key[lo:lo + 4096], h[lo:lo + 4096].double())
    got = got.cpu().numpy()
    scale = float(h.double().pow(2).mean().sqrt())
    worst = 0.0
    for c in range(C + 1):
        if cnt[c] == 0:
            assert not np.any(got[c]), f"{what}: bucket {c} is empty but has a non-zero sum"
            continue
        err = float(np.max(np.abs(got[c] - ref[c])))
        bound = 1e-4 * scale * np.sqrt(cnt[c]) + 1e-9
        assert err <= bound, f"{what}: column sums of bucket {c} off by {err:.3e} > {bound:.3e}"
        worst = max(worst, err / bound)
    return worst
