"""Pins of the oracle's learned-router / weighted-mixture / compositional-gating part
(Sec. "Router Architecture", Alg. "Compositional Gating Kernel", Def. "Hot-Set Layout")
against things other than itself: float64 math, numpy's sort, the single-adapter oracle."""
import math

import numpy as np
import pytest

import oracle
from oracle import build as obuild
from paper_2603_15965_amd import workloads as wl


@pytest.fixture(scope="module", autouse=True)
def _built():
    obuild.build(force=False)


def bf16(a):
    return wl.to_bf16_bits(np.asarray(a, dtype=np.float32))


def f32(bits):
    return wl.bf16_bits_to_f32(bits).astype(np.float64)


def test_exp_matches_float64():
    assert oracle.expf(0.0) == 1.0
    ys = np.concatenate([np.linspace(-87, 5, 4001), -np.logspace(-8, 1.9, 500)])
    for y in ys:
        y32 = float(np.float32(y))
        ref = math.exp(y32)
        assert abs(oracle.expf(y32) - ref) <= 4e-7 * ref, y
    assert oracle.expf(-100.0) == 0.0
    assert oracle.expf(float("-inf")) == 0.0


def test_gelu_matches_erf_form():
    for u in np.concatenate([np.linspace(-8, 8, 3201), [0.0, -0.0, 1e-6, -1e-6, 20.0, -20.0]]):
        u32 = float(np.float32(u))
        ref = 0.5 * u32 * (1.0 + math.erf(u32 / math.sqrt(2.0)))
        assert abs(oracle.gelu(u32) - ref) <= 2.5e-7 * max(1.0, abs(u32)), u
    assert oracle.gelu(0.0) == 0.0


def _router(seed, N, d, H, K):
    rng = np.random.default_rng(seed)
    x = bf16(rng.standard_normal((N, d)))
    W1 = bf16(rng.standard_normal((d, H)) / math.sqrt(d))
    b1 = (0.1 * rng.standard_normal(H)).astype(np.float32)
    W2 = bf16(rng.standard_normal((H, K)) / math.sqrt(H))
    b2 = (0.1 * rng.standard_normal(K)).astype(np.float32)
    return x, W1, b1, W2, b2


def test_mlp_logits_match_float64():
    x, W1, b1, W2, b2 = _router(1, 37, 96, 64, 9)
    got = oracle.mlp_logits(x, W1, b1, W2, b2)
    u = f32(x) @ f32(W1) + b1.astype(np.float64)
    g = 0.5 * u * (1.0 + np.vectorize(math.erf)(u / math.sqrt(2.0)))
    ref = g @ f32(W2) + b2.astype(np.float64)
    assert got.shape == (37, 9) and got.dtype == np.float32
    assert np.max(np.abs(got - ref)) <= 2e-5
    # a transposed W1 or W2, a dropped bias or a missing activation would be far off
    assert np.max(np.abs(got - (u @ f32(W2) + b2))) > 1e-2


def test_topk_is_a_stable_descending_sort_prefix():
    rng = np.random.default_rng(2)
    l = rng.standard_normal((200, 12)).astype(np.float32)
    l[5, :] = 0.25                      # all equal: indices 0, 1, 2
    l[6, [3, 7, 9]] = 4.0               # three-way tie at the top
    for k in (1, 2, 4, 12):
        idx, w = oracle.topk_softmax(l, k)
        order = np.argsort(-l.astype(np.float64), axis=1, kind="stable")[:, :k]
        assert np.array_equal(idx, order)
        sel = np.take_along_axis(l.astype(np.float64), order, axis=1)
        e = np.exp(sel - sel[:, :1])
        ref = e / e.sum(axis=1, keepdims=True)
        assert np.max(np.abs(w - ref)) <= 1e-6
        assert np.max(np.abs(w.sum(axis=1) - 1.0)) <= 1e-6
        assert np.all(w[:, :-1] >= w[:, 1:])
    idx, w = oracle.topk_softmax(l, 3)
    assert list(idx[5]) == [0, 1, 2] and list(idx[6]) == [3, 7, 9]
    assert np.all(w[5] == w[5, 0])
    idx1, w1 = oracle.topk_softmax(l, 1)
    assert np.all(w1 == 1.0)           # softmax over a single selected logit


def test_mix_with_k1_is_the_single_adapter_oracle_bit_for_bit():
    w = wl.make(wl.shapes()["tiny"])
    ref = oracle.apply(w.x, w.W, w.A, w.B, w.r)
    got = oracle.apply_mix(w.x, w.W, w.A, w.B, w.r.reshape(-1, 1))
    assert np.array_equal(got, ref)
    ones = np.ones((w.shape.N, 1), dtype=np.float32)
    assert np.array_equal(oracle.apply_mix(w.x, w.W, w.A, w.B, w.r.reshape(-1, 1), ones), ref)


def test_mix_is_the_weighted_sum_of_single_adapter_deltas():
    sh = wl.shapes()["tiny"]
    w = wl.make(sh)
    N, C = sh.N, sh.C
    rng = np.random.default_rng(3)
    idx = np.stack([rng.permutation(C)[:2] for _ in range(N)]).astype(np.int32)
    wts = rng.random((N, 2)).astype(np.float32)
    wts /= wts.sum(axis=1, keepdims=True)
    got = oracle.apply_mix(w.x, w.W, w.A, w.B, idx, wts).astype(np.float64)
    base = f32(w.x) @ f32(w.W)
    single = [oracle.apply(w.x, w.W, w.A, w.B, np.full(N, c, dtype=np.int32)).astype(np.float64) - base
              for c in range(C)]
    ref = base.copy()
    for j in range(2):
        ref += wts[:, j:j + 1].astype(np.float64) * np.stack([single[idx[i, j]][i] for i in range(N)])
    scale = np.sqrt(np.mean(ref ** 2))
    assert np.max(np.abs(got - ref)) <= 2e-5 * scale
    # equal logits over all adapters: the plain average of the C single-adapter deltas
    idx_all = np.tile(np.arange(C, dtype=np.int32), (N, 1))
    w_all = np.full((N, C), 1.0 / C, dtype=np.float32)
    avg = base + sum(single) / C
    got_all = oracle.apply_mix(w.x, w.W, w.A, w.B, idx_all, w_all).astype(np.float64)
    assert np.max(np.abs(got_all - avg)) <= 2e-5 * scale
    # an index outside [0, C) contributes nothing
    idx_bad = idx.copy()
    idx_bad[:, 1] = -1
    only0 = oracle.apply_mix(w.x, w.W, w.A, w.B, idx_bad, wts).astype(np.float64)
    ref0 = base + wts[:, :1].astype(np.float64) * np.stack([single[idx[i, 0]][i] for i in range(N)])
    assert np.max(np.abs(only0 - ref0)) <= 2e-5 * scale


def test_mix_scales_exactly_with_powers_of_two():
    w = wl.make(wl.shapes()["tiny"])
    N, C = w.shape.N, w.shape.C
    W0 = np.zeros_like(w.W)
    rng = np.random.default_rng(4)
    idx = np.stack([rng.permutation(C)[:2] for _ in range(N)]).astype(np.int32)
    wts = np.full((N, 2), 0.5, dtype=np.float32)
    B2 = bf16(2.0 * wl.bf16_bits_to_f32(w.B))
    h1 = oracle.apply_mix(w.x, W0, w.A, w.B, idx, wts)
    h2 = oracle.apply_mix(w.x, W0, w.A, B2, idx, wts)
    assert np.array_equal(h2, 2.0 * h1)


def test_slot_table_indirection():
    w = wl.make(wl.shapes()["tiny"])
    N, C = w.shape.N, w.shape.C
    ref = oracle.apply(w.x, w.W, w.A, w.B, w.r)
    ident = np.arange(C, dtype=np.int32)
    assert np.array_equal(oracle.apply_mix(w.x, w.W, w.A, w.B, w.r.reshape(-1, 1), None, ident), ref)
    # pools with S = C + 2 slots; adapter c lives in slot sigma[c]
    sigma = np.array([5, 0, 3, 2], dtype=np.int32)[:C]
    S = 6
    A_pool = np.zeros((S,) + w.A.shape[1:], dtype=np.uint16)
    B_pool = np.zeros((S,) + w.B.shape[1:], dtype=np.uint16)
    rng = np.random.default_rng(5)
    A_pool[:] = bf16(rng.standard_normal(A_pool.shape))   # unused slots hold garbage
    B_pool[:] = bf16(rng.standard_normal(B_pool.shape))
    for c in range(C):
        A_pool[sigma[c]] = w.A[c]
        B_pool[sigma[c]] = w.B[c]
    got = oracle.apply_mix(w.x, w.W, A_pool, B_pool, w.r.reshape(-1, 1), None, sigma)
    assert np.array_equal(got, ref)


def test_compose_is_adapter_times_modalities_plus_modality():
    rng = np.random.default_rng(6)
    breaks = np.array([0, 1000, 1500, 4000], dtype=np.int32)
    M, n_ad = 3, 5
    v = rng.integers(-50, 4100, size=5000).astype(np.int32)
    a = rng.integers(-1, n_ad + 1, size=5000).astype(np.int32)
    got = oracle.route_compose(v, a, breaks, n_ad)
    m = np.searchsorted(breaks, v, side="right") - 1
    ok = (v >= breaks[0]) & (v < breaks[-1]) & (a >= 0) & (a < n_ad)
    ref = np.where(ok, a * M + m, -1)
    assert np.array_equal(got, ref)
    assert got.max() == n_ad * M - 1 and (got == -1).any()
    # with one adapter the composite target is the vocabulary route
    one = oracle.route_compose(v, np.zeros_like(v), breaks, 1)
    assert np.array_equal(one, oracle.route_vocab(v, breaks))
