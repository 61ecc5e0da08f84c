"""Seeded random shapes through molora_apply / molora_apply_mix against the oracle: every
kernel path (32- and 64-column small-batch, three-stage and two-stage tiles, row-item and
streaming shrink), ragged sizes, random slot tables, invalid entries."""
import sys

import numpy as np
import pytest

from paper_2603_15965_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _cases():
    rng = np.random.default_rng(20260315)
    out = []
    ranks = [8, 16, 24, 32, 64, 128]
    for i in range(36):
        N = int(rng.choice([1, 3, 17, 40, 64, 65, 130, 300, 513, 700]))
        d_in = int(rng.integers(1, 80)) * 8
        d_out = int(rng.integers(1, 80)) * 8
        if i % 6 == 0:
            d_in, d_out = int(rng.integers(100, 160)) * 8, int(rng.integers(1, 20)) * 8   # long K
        k = int(rng.choice([1, 1, 2, 3]))
        rank = int(rng.choice([r for r in ranks if r * k <= 128]))
        cmax = {1: 40, 2: 31, 3: 10}[k]
        C = int(rng.integers(max(k, 1), cmax + 1))
        S = None if rng.random() < 0.5 else C + int(rng.integers(0, 5))
        bad = bool(rng.random() < 0.3)
        out.append((i, N, d_in, d_out, C, rank, k, S, bad))
    # small batches (one row tile in token order, and a few tiles of sorted rows): the expand
    # phase with every rank / tuple width, many and few buckets per tile
    for i in range(36, 64):
        N = int(rng.integers(1, 65)) if i % 2 == 0 else int(rng.integers(65, 513))
        d_in = int(rng.integers(1, 70)) * 8
        d_out = int(rng.integers(1, 70)) * 8
        k = int(rng.choice([1, 1, 2, 3, 4]))
        rank = int(rng.choice([r for r in ranks if r * k <= 128]))
        cmax = {1: 64, 2: 31, 3: 10, 4: 5}[k]
        C = int(rng.integers(max(k, 1), cmax + 1))
        S = None if rng.random() < 0.5 else C + int(rng.integers(0, 5))
        bad = bool(rng.random() < 0.3)
        out.append((i, N, d_in, d_out, C, rank, k, S, bad))
    # both sides of the choice between the streaming kernel and the tiled one (129 .. 4096 rows:
    # decided by a cost of both, not by a fixed number of rows), many adapters included
    for i in range(64, 88):
        N = int([rng.integers(129, 600), rng.integers(600, 1500), rng.integers(1500, 4300)][i % 3])
        d_in = int(rng.integers(1, 160)) * 8
        d_out = int(rng.integers(1, 200)) * 8 if i % 4 else int(rng.integers(8, 100)) * 64
        while N * d_in * d_out > 2e9:
            d_in = max(8, d_in // 16 * 8)
        k = int(rng.choice([1, 1, 1, 2, 3, 4]))
        rank = int(rng.choice([r for r in ranks if r * k <= 128]))
        cmax = {1: 200, 2: 31, 3: 10, 4: 5}[k]
        C = int(rng.integers(max(k, 1), cmax + 1))
        S = None if rng.random() < 0.5 else C + int(rng.integers(0, 5))
        bad = bool(rng.random() < 0.3)
        out.append((i, N, d_in, d_out, C, rank, k, S, bad))
    return out


@pytest.mark.parametrize("i,N,d_in,d_out,C,rank,k,S,bad", _cases())
def test_random_shape(i, N, d_in, d_out, C, rank, k, S, bad):
    import oracle
    import torch
    import gpu_helpers as gpu
    from paper_2603_15965_amd import binding as mb
    print(f"random shape {i}: N={N} {d_in}->{d_out} C={C} rank={rank} k={k} S={S} bad={bad}", flush=True)
    sys.stdout.flush()
    w = wl.custom("rnd", N, d_in, d_out, S or C, rank, wl.BASE_SEED + 31000 + i)
    rng = np.random.default_rng(7000 + i)
    idx = np.stack([rng.permutation(C)[:k] for _ in range(N)]).astype(np.int32)
    wts = rng.random((N, k)).astype(np.float32) + 0.05
    wts /= wts.sum(axis=1, keepdims=True)
    if bad:
        idx[rng.random((N, k)) < 0.15] = -1
    slots = None if S is None else rng.permutation(S)[:C].astype(np.int32)
    x, W, A, B = (gpu.dev_bf16(t) for t in (w.x, w.W, w.A, w.B))
    h = mb.molora_apply_mix(x, W, A, B, gpu.dev_i32(idx), torch.from_numpy(wts).cuda(),
                            None if slots is None else gpu.dev_i32(slots), C=C)
    torch.cuda.synchronize()
    ref = oracle.apply_mix(w.x, w.W, w.A, w.B, idx, wts, slots, C=C)
    gpu.assert_h_close(h.cpu().numpy(), ref, f"random shape {i}")
    if k == 1 and S is None and not bad:   # the plain entry point on the same routing: same bits
        h1 = mb.molora_apply(x, W, A, B, gpu.dev_i32(idx[:, 0]))
        torch.cuda.synchronize()
        gpu.assert_h_close(h1.cpu().numpy(), oracle.apply(w.x, w.W, w.A, w.B, idx[:, 0]), f"apply {i}")


def _plain_cases():
    """Shapes that take molora_apply's special routes: a few narrow adapters (dispatch and
    token-order shrink in one launch) and decode-sized batches (dispatch, shrink and x W in one
    launch, then the expand), with targets out of range in half of them."""
    rng = np.random.default_rng(20260316)
    out = []
    for i in range(12):   # C * rank <= 64, N > 512
        C, rank = [(1, 8), (2, 8), (4, 8), (8, 8), (1, 16), (2, 16), (4, 16), (3, 16), (1, 32), (2, 32), (1, 64),
                   (5, 8)][i]
        N = int(rng.integers(513, 6000))
        out.append((i, N, int(rng.integers(2, 90)) * 8, int(rng.integers(2, 90)) * 8, C, rank, i % 2 == 1))
    for i in range(12, 24):   # N <= 64, rank above 32
        rank = int(rng.choice([40, 48, 64, 96, 128]))
        out.append((i, int(rng.integers(1, 65)), int(rng.integers(2, 160)) * 8, int(rng.integers(2, 90)) * 8,
                    int(rng.integers(1, 40)), rank, i % 2 == 1))
    return out


@pytest.mark.parametrize("i,N,d_in,d_out,C,rank,bad", _plain_cases())
def test_random_shape_plain_routes(i, N, d_in, d_out, C, rank, bad):
    import oracle
    import torch
    import gpu_helpers as gpu
    from paper_2603_15965_amd import binding as mb
    print(f"random plain shape {i}: N={N} {d_in}->{d_out} C={C} rank={rank} bad={bad}", flush=True)
    assert mb.molora_dense_shrink_supported(N, d_in, C, rank) or mb.molora_bucket_shrink_small_supported(N, d_in, C, rank)
    w = wl.custom("rndp", N, d_in, d_out, C, rank, wl.BASE_SEED + 32000 + i, structure="zipf" if i % 3 else "uniform")
    r = w.r.copy()
    if bad:
        rng = np.random.default_rng(7100 + i)
        r[rng.random(N) < 0.2] = int(rng.choice([-1, C, C + 5, -1000]))
    x, W, A, B = (gpu.dev_bf16(t) for t in (w.x, w.W, w.A, w.B))
    h = mb.molora_apply(x, W, A, B, gpu.dev_i32(r))
    torch.cuda.synchronize()
    gpu.assert_h_close(h.cpu().numpy(), oracle.apply(w.x, w.W, w.A, w.B, r), f"random plain shape {i}")
    if N <= 64 and mb.molora_pack_w_cols(d_out):   # the packed base weight: the two launches, same bits as apply
        rd = gpu.dev_i32(r)
        o, p, t, h2 = mb.molora_shrink_base_small(rd, x, mb.molora_pack_w(W), A, packed=True)
        if rank % 16 == 0:
            mb.molora_expand_small(mb.molora_pack_b(B), t, o, p, h2, packed=True)
        else:
            mb.molora_expand_small(B, t, o, p, h2)
        torch.cuda.synchronize()
        assert torch.equal(h, h2), f"random plain shape {i}: packed base weight (and B)"
