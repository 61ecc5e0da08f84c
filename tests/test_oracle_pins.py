"""Pins for the CPU oracle: each test checks the oracle against something the paper or
the mathematics fixes independently of the oracle's own code (float64 numpy products,
numpy's stable sort / bincount / searchsorted, hand-worked integers, fp32 rounding
facts).  CPU only."""
import json
import os

import numpy as np
import pytest

from paper_2603_15965_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def f64(bits):
    return wl.bf16_bits_to_f32(bits).astype(np.float64)


def rms(a):
    return float(np.sqrt(np.mean(np.asarray(a, dtype=np.float64) ** 2)))


def dense_reference(w, r):
    """float64: brute force over ALL adapters, then select the routed one per token
    (work K*N instead of N, Thm. 'Computational Optimality')."""
    x, W, A, B = f64(w.x), f64(w.W), f64(w.A), f64(w.B)
    base = x @ W
    all_delta = np.stack([(x @ A[c]) @ B[c] for c in range(A.shape[0])])  # [C][N][d_out]
    out = base.copy()
    for i, c in enumerate(r):
        if 0 <= c < A.shape[0]:
            out[i] += all_delta[c, i]
    return out


# non-square on purpose: a transposed operand or a swapped d_in/d_out/rank index
# cannot survive these shapes
def small(seed=7, N=97, d_in=80, d_out=48, C=5, rank=8):
    return wl.custom("pin", N, d_in, d_out, C, rank, seed)


def test_hand_worked_example(oracle_lib):
    g = json.load(open(os.path.join(GOLDEN, "hand_worked_pertok.json")))
    bits = lambda a: wl.to_bf16_bits(np.array(a, dtype=np.float32))
    h = oracle_lib.apply(bits(g["x"]), bits(g["W"]), bits(g["A"]), bits(g["B"]),
                         np.array(g["r"], dtype=np.int32))
    assert np.array_equal(h, np.array(g["h"], dtype=np.float32))


def test_all_tokens_one_adapter_is_per_sequence_formula(oracle_lib):
    # Eq. (perseq): with r(i) = c for every i, h = x W + (x A_c) B_c as dense products
    w = small()
    for c in (0, 3):
        r = np.full(w.shape.N, c, dtype=np.int32)
        h = oracle_lib.apply(w.x, w.W, w.A, w.B, r)
        ref = f64(w.x) @ f64(w.W) + (f64(w.x) @ f64(w.A[c])) @ f64(w.B[c])
        assert np.max(np.abs(h - ref)) <= 2e-5 * rms(ref)


def test_brute_force_all_adapters_then_select(oracle_lib):
    w = small(seed=11)
    h = oracle_lib.apply(w.x, w.W, w.A, w.B, w.r)
    ref = dense_reference(w, w.r)
    assert np.max(np.abs(h - ref)) <= 2e-5 * rms(ref)
    # and the selection matters: a shifted routing must NOT match
    wrong = dense_reference(w, (w.r + 1) % w.shape.C)
    assert np.max(np.abs(h - wrong)) > 0.1 * rms(ref)


def test_zero_B_adapter_reduces_to_base(oracle_lib):
    w = small(seed=13)
    B = w.B.copy()
    B[2] = 0
    h = oracle_lib.apply(w.x, w.W, w.A, B, w.r)
    base = f64(w.x) @ f64(w.W)
    sel = w.r == 2
    assert sel.any() and (~sel).any()
    assert np.max(np.abs(h[sel] - base[sel])) <= 2e-5 * rms(base)
    # x W + 0 is exact: identical bits to the no-adapter result
    h_none = oracle_lib.apply(w.x, w.W, w.A, B, np.full_like(w.r, -1))
    assert np.array_equal(h[sel], h_none[sel])
    assert np.max(np.abs(h[~sel] - base[~sel])) > 0.1 * rms(base)


def test_single_adapter_is_dense_lora(oracle_lib):
    # Sec. 2.1: h = xW + xAB
    w = small(seed=17, C=1)
    h = oracle_lib.apply(w.x, w.W, w.A, w.B, np.zeros(w.shape.N, dtype=np.int32))
    ref = f64(w.x) @ f64(w.W) + f64(w.x) @ f64(w.A[0]) @ f64(w.B[0])
    assert np.max(np.abs(h - ref)) <= 2e-5 * rms(ref)


def test_tiny_config_against_float64(oracle_lib):
    w = wl.make(wl.shapes()["tiny"])
    h = oracle_lib.apply(w.x, w.W, w.A, w.B, w.r)
    ref = dense_reference(w, w.r)
    assert np.max(np.abs(h - ref)) <= 2e-5 * rms(ref)
    # statistics implied by the stated distributions: Var(xW) ~ 1, Var(xAB) ~ 1
    assert abs(rms(h) - np.sqrt(2.0)) < 0.05
    assert abs(rms(f64(w.x) @ f64(w.W)) - 1.0) < 0.05


def test_apply_rows_subset_matches_full(oracle_lib):
    w = small(seed=19)
    rows = np.array([96, 0, 5, 5, 42], dtype=np.int64)
    ref = dense_reference(w, w.r)[rows]
    sub = oracle_lib.apply_rows(w.x, w.W, w.A, w.B, w.r, rows)
    assert np.max(np.abs(sub - ref)) <= 2e-5 * rms(ref)


def test_power_of_two_scaling_is_exact(oracle_lib):
    # doubling B doubles the low-rank term bit-exactly (scaling by 2 commutes with rounding)
    w = small(seed=23)
    none = np.full_like(w.r, -1)
    base = oracle_lib.apply(w.x, w.W, w.A, w.B, none)
    zeroW = np.zeros_like(w.W)
    d1 = oracle_lib.apply(w.x, zeroW, w.A, w.B, w.r)
    B2 = wl.to_bf16_bits(2.0 * wl.bf16_bits_to_f32(w.B))
    d2 = oracle_lib.apply(w.x, zeroW, w.A, B2, w.r)
    assert np.array_equal(d2, 2.0 * d1)
    ref_delta = dense_reference(w, w.r) - f64(w.x) @ f64(w.W)
    assert np.max(np.abs(d1 - ref_delta)) <= 2e-5 * rms(ref_delta)
    assert base.shape == d1.shape


def test_token_permutation_equivariance(oracle_lib):
    w = small(seed=29)
    rng = np.random.default_rng(1)
    p = rng.permutation(w.shape.N)
    h = oracle_lib.apply(w.x, w.W, w.A, w.B, w.r)
    hp = oracle_lib.apply(w.x[p], w.W, w.A, w.B, w.r[p])
    assert np.array_equal(hp, h[p])


def test_fp32_ascending_order_of_the_gate_sum(oracle_lib):
    # terms (1, 2^30, -2^30): ascending fp32 accumulation gives 0 (1 is absorbed), a
    # descending or a wider accumulation gives 1.  Column 1 holds the terms in the
    # opposite order and must give 1.  Both facts follow from fp32 rounding alone.
    x = wl.to_bf16_bits(np.array([[1.0, 1.0, 1.0]], dtype=np.float32))
    G = wl.to_bf16_bits(np.array([[1.0, -2.0 ** 30], [2.0 ** 30, 2.0 ** 30], [-2.0 ** 30, 1.0]],
                                 dtype=np.float32))
    logits = oracle_lib.gate_logits(x, G)
    assert logits.tolist() == [[0.0, 1.0]]
    assert oracle_lib.route_gate(x, G).tolist() == [1]


def test_gate_on_exact_integer_inputs_and_ties(oracle_lib):
    # small integers: every partial sum is exact, so the argmax is order-independent
    rng = np.random.default_rng(5)
    N, d, C = 300, 64, 7
    xi = rng.integers(-4, 5, size=(N, d))
    Gi = rng.integers(-3, 4, size=(d, C))
    Gi[:, 5] = Gi[:, 2]                      # columns 2 and 5 always tie exactly
    x, G = wl.to_bf16_bits(xi.astype(np.float32)), wl.to_bf16_bits(Gi.astype(np.float32))
    logits = xi @ Gi
    expect = np.argmax(logits, axis=1)       # numpy argmax returns the first maximum
    r = oracle_lib.route_gate(x, G)
    assert np.array_equal(r, expect)
    assert not np.any(r == 5)                # the lower index of a tie always wins
    assert np.array_equal(oracle_lib.gate_logits(x, G), logits.astype(np.float32))


def test_gate_one_hot_columns_select_a_coordinate(oracle_lib):
    w = small(seed=31, d_in=40, C=6)
    ks = [3, 39, 0, 17, 8, 21]
    G = np.zeros((40, 6), dtype=np.float32)
    for c, k in enumerate(ks):
        G[k, c] = 1.0
    r = oracle_lib.route_gate(w.x, wl.to_bf16_bits(G))
    xv = wl.bf16_bits_to_f32(w.x)[:, ks]
    assert np.array_equal(r, np.argmax(xv, axis=1))


def test_gate_matches_float64_argmax_away_from_ties(oracle_lib):
    w = wl.custom("g", 512, 256, 16, 8, 8, 37, route="gate")
    r = oracle_lib.route_gate(w.x, w.G)
    logits = f64(w.x) @ f64(w.G)
    srt = np.sort(logits, axis=1)
    clear = (srt[:, -1] - srt[:, -2]) > 1e-4
    assert clear.sum() > 480
    assert np.array_equal(r[clear], np.argmax(logits, axis=1)[clear])
    assert np.max(np.abs(oracle_lib.gate_logits(w.x, w.G) - logits)) < 1e-4


def test_vocab_routing_is_searchsorted(oracle_lib):
    breaks = np.array([0, 100, 250, 251, 1000], dtype=np.int32)
    rng = np.random.default_rng(3)
    v = np.concatenate([rng.integers(0, 1000, size=500), [0, 99, 100, 249, 250, 251, 999]]).astype(np.int32)
    r = oracle_lib.route_vocab(v, breaks)
    assert np.array_equal(r, np.searchsorted(breaks, v, side="right") - 1)
    # ids outside [b_0, b_M) route nowhere
    assert oracle_lib.route_vocab(np.array([-1, 1000, 5000], dtype=np.int32), breaks).tolist() == [-1, -1, -1]


@pytest.mark.parametrize("N,C", [(0, 3), (1, 1), (257, 4), (5000, 32), (64, 16)])
def test_bucket_is_stable_counting_sort(oracle_lib, N, C):
    rng = np.random.default_rng(N + C)
    r = rng.integers(0, C, size=N).astype(np.int32)
    offsets, perm, bad = oracle_lib.bucket(r, C)
    assert bad == 0
    cnt = np.bincount(r, minlength=C)               # histogram h[k] = |{t : r(t) = k}|
    assert np.array_equal(offsets, np.concatenate([[0], np.cumsum(cnt)]))
    assert np.array_equal(perm, np.argsort(r, kind="stable"))


def test_bucket_out_of_range_targets_go_last(oracle_lib):
    r = np.array([2, -1, 0, 7, 2, 3, 0, -5], dtype=np.int32)
    offsets, perm, bad = oracle_lib.bucket(r, 3)
    assert bad == 4
    assert offsets.tolist() == [0, 2, 2, 4]
    assert perm.tolist() == [2, 6, 0, 4, 1, 3, 5, 7]


def test_bucket_invariants_with_empty_buckets(oracle_lib):
    r = wl.zipf_targets(9, 64, 16, 1.1)
    offsets, perm, bad = oracle_lib.bucket(r, 16)
    assert bad == 0 and offsets[0] == 0 and offsets[-1] == 64
    assert np.all(np.diff(offsets) >= 0)
    assert sorted(perm.tolist()) == list(range(64))
    for c in range(16):
        seg = perm[offsets[c]:offsets[c + 1]]
        assert np.all(r[seg] == c) and np.all(np.diff(seg) > 0)
