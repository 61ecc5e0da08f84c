"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle on the same
seeded inputs.  Routing, offsets and permutation are compared bit for bit; h within
max|h_gpu - h_oracle| <= 1e-2 * RMS(h_oracle)."""
import sys

import numpy as np
import pytest

from paper_2603_15965_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2603_15965_amd import binding
    binding.load()          # fails loudly if libmolora.so is not built
    import gpu_helpers
    return gpu_helpers


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


# ------------------------------------------------------------------ dispatch
@pytest.mark.parametrize("N,C,kind", [
    (0, 3, "uniform"), (1, 1, "uniform"), (63, 2, "uniform"), (64, 16, "zipf"), (257, 4, "uniform"),
    (4096, 2, "uniform"), (8192, 8, "uniform"), (16384, 32, "uniform"), (16384, 32, "all0"),
    (5000, 33, "skew"), (20001, 100, "uniform"), (3000, 1024, "uniform"), (70000, 7, "uniform"),
])
def test_bucket_bit_exact(gpu, N, C, kind):
    say(f"bucket N={N} C={C} {kind}")
    if kind == "uniform":
        r = wl.uniform_targets(N + C, N, C)
    elif kind == "zipf":
        r = wl.zipf_targets(N + C, N, C, 1.1)
    elif kind == "all0":
        r = np.zeros(N, dtype=np.int32)
    else:
        p = np.ones(C); p[0] = 20 * C; p[5] = 0
        r = wl.skewed_targets(N + C, N, p)
    gpu.check_bucket(r, C)


def test_bucket_out_of_range_targets(gpu):
    say("bucket with out-of-range targets")
    r = wl.uniform_targets(5, 3000, 12) - 2      # values -2..9 with C = 8
    gpu.check_bucket(r, 8)


def test_route_vocab_bit_exact(gpu):
    import oracle
    w = wl.make(wl.shapes()["vocab_q17"], want=("route",))
    say("route_vocab config 1")
    r = gpu.gpu_route(w).cpu().numpy()
    assert np.array_equal(r, oracle.route_vocab(w.v, w.breaks))
    v = np.array([-5, 0, 99, 100, 250, 251, 999, 1000, 7], dtype=np.int32)
    br = np.array([0, 100, 250, 251, 1000], dtype=np.int32)
    from paper_2603_15965_amd import binding as mb
    got = mb.molora_route_vocab(gpu.dev_i32(v), br).cpu().numpy()
    assert np.array_equal(got, oracle.route_vocab(v, br))


# ------------------------------------------------------------------ learned gate
@pytest.mark.parametrize("N,d_in,C", [
    (1, 8, 1), (77, 136, 3), (300, 256, 4), (300, 264, 8), (129, 1000, 16), (513, 520, 32),
    (200, 320, 64), (100, 200, 100), (64, 64, 300), (40, 72, 1024),
    # four token groups per workgroup, ragged token counts
    (8200, 264, 8), (16390, 136, 24), (20000, 72, 33), (33000, 40, 64),
])
def test_route_gate_bit_exact_small(gpu, N, d_in, C):
    import oracle
    say(f"route N={N} d_in={d_in} C={C}")
    w = wl.custom("g", N, d_in, 16, C, 8, 9000 + N + C, route="gate")
    r = gpu.gpu_route(w).cpu().numpy()
    assert np.array_equal(r, oracle.route_gate(w.x, w.G))


def test_route_gate_exact_ties_pick_lowest_index(gpu):
    import oracle
    say("route ties")
    rng = np.random.default_rng(5)
    N, d, C = 256, 64, 12
    xi = rng.integers(-4, 5, size=(N, d)).astype(np.float32)
    Gi = rng.integers(-3, 4, size=(d, C)).astype(np.float32)
    Gi[:, 7] = Gi[:, 2]
    Gi[:, 11] = Gi[:, 0]
    w = wl.custom("t", N, d, 16, C, 8, 1, route="gate")
    w.x, w.G = wl.to_bf16_bits(xi), wl.to_bf16_bits(Gi)
    r = gpu.gpu_route(w).cpu().numpy()
    assert np.array_equal(r, oracle.route_gate(w.x, w.G))
    assert not np.any((r == 7) | (r == 11))


@pytest.mark.parametrize("nan_col", [0, 3])
def test_route_gate_nan_logits_follow_the_scan(gpu, nan_col):
    """Unsupported input with a defined result: a NaN logit above target 0 is never selected,
    a NaN at target 0 (the scan's starting point) yields 0."""
    import oracle
    say(f"route with NaN logits in column {nan_col}")
    w = wl.custom("nan", 300, 128, 16, 9, 8, 9100, route="gate")
    G = w.G.copy()
    G[5, nan_col] = 0x7FC0  # bf16 quiet NaN: every token's logit for this target is NaN
    w.G = G
    r = gpu.gpu_route(w).cpu().numpy()
    ref = oracle.route_gate(w.x, w.G)
    assert np.array_equal(r, ref)
    assert np.all(r == 0) if nan_col == 0 else not np.any(r == nan_col)


@pytest.mark.parametrize("name", ["gate_up17", "prefill8_q", "prefill8_down"])
def test_route_gate_bit_exact_full_configs(gpu, name):
    import oracle
    say(f"route full {name}")
    w = wl.make(wl.shapes()[name], want=("x", "route"))
    r = gpu.gpu_route(w).cpu().numpy()
    ref = oracle.route_gate(w.x, w.G)
    assert np.array_equal(r, ref), f"{int((r != ref).sum())} routing mismatches"
    gpu.check_bucket(ref, w.shape.C)


# ------------------------------------------------------------------ the projection
@pytest.mark.parametrize("N,d_in,d_out,C,rank,structure", [
    (1, 64, 64, 1, 8, "uniform"),
    (97, 80, 48, 5, 8, "uniform"),          # nothing a multiple of a tile
    (300, 200, 328, 3, 16, "uniform"),      # ragged K tail and N tail, 3 column tiles
    (515, 520, 264, 7, 24, "uniform"),      # rank not a multiple of 16
    (700, 256, 512, 40, 32, "zipf"),        # many small and empty buckets inside one tile
    (64, 512, 1024, 16, 64, "zipf"),
    (50, 1024, 520, 5, 16, "uniform"),      # small-batch path with the K range split, ragged
    (64, 2048, 1024, 16, 64, "zipf"),       # small-batch path, many buckets in the one row tile
    (7, 1096, 264, 3, 8, "uniform"),        # small-batch path, K tail
    (64, 640, 200, 11, 8, "uniform"),       # small-batch path, four buckets per expand item (2R = 16), 3 items
    (61, 512, 136, 37, 16, "uniform"),      # two buckets per expand item, more items than wavefronts
    (33, 128, 72, 9, 24, "uniform"),        # fewer pieces of W than wavefronts; 2R = 48, one bucket per item
    (64, 256, 328, 6, 128, "zipf"),         # four 64-row pieces of [B; B] per bucket
    (16, 64, 64, 16, 40, "uniform"),        # one piece of W, 2R = 80: a full and a short piece per bucket
    (200, 520, 328, 9, 24, "zipf"),         # small-batch path, four row tiles, ragged everywhere
    (700, 2048, 136, 3, 64, "zipf"),        # buckets of several 64-row tiles in the small-batch shrink
    (600, 328, 1000, 7, 24, "zipf"),        # 128 x 128 tiles with three stages, K shorter than the ring
    (1500, 1096, 392, 5, 16, "uniform"),    # same, K tail tile
    (1000, 128, 136, 4, 128, "uniform"),    # maximum rank
    (2304, 192, 2560, 6, 16, "all0"),       # large-tile path (>= 512 tiles), one bucket
    (2500, 128, 4000, 9, 8, "uniform"),     # large-tile path, ragged everything
    (4000, 3080, 1992, 5, 24, "zipf"),      # 128 x 256 tiles with three stages (K >= 3072), ragged everything, K tail
    (1100, 3072, 3800, 12, 16, "uniform"),  # the same tiles, two narrow buckets per expand tile
    (4090, 4096, 2048, 3, 8, "zipf"),       # the same tiles with the token-order intermediate (C * rank <= 64)
])
def test_apply_small_shapes(gpu, N, d_in, d_out, C, rank, structure):
    import oracle
    say(f"apply N={N} {d_in}->{d_out} C={C} rank={rank} {structure}")
    w = wl.custom("a", N, d_in, d_out, C, rank, 7000 + N, structure=structure)
    h = gpu.gpu_apply(w, w.r).cpu().numpy()
    gpu.assert_h_close(h, oracle.apply(w.x, w.W, w.A, w.B, w.r), "apply")


@pytest.mark.parametrize("N,d_in,d_out,C,rank,structure", [
    (1500, 520, 392, 4, 16, "uniform"),     # C * rank = 64, ragged K tail, 128 x 128 tiles
    (700, 256, 264, 2, 32, "zipf"),         # two wide adapters, three-stage tiles
    (3000, 264, 520, 8, 8, "uniform"),      # eight rank-8 adapters
    (600, 1096, 136, 1, 64, "uniform"),     # one adapter of rank 64
    (2500, 128, 4000, 3, 8, "zipf"),        # 256 x 256 tiles, C * rank = 24 (padded to 32 columns)
    (5000, 328, 264, 5, 8, "uniform"),      # five dispatch workgroups, 40 columns
    (20000, 136, 136, 2, 16, "uniform"),    # sixteen dispatch workgroups, 32-row shrink items
])
def test_apply_few_narrow_adapters_one_launch_dispatch_and_shrink(gpu, N, d_in, d_out, C, rank, structure):
    """C * rank <= 64 and N > 512: molora_apply runs dispatch and token-order shrink in one
    launch.  The pieces are checked one by one (offsets and perm bit for bit, also with targets
    out of range; t against the float64 product) and the whole against the oracle."""
    import oracle
    import torch
    from paper_2603_15965_amd import binding as mb
    say(f"dense shrink path N={N} {d_in}->{d_out} C={C} rank={rank} {structure}")
    assert mb.molora_dense_shrink_supported(N, d_in, C, rank)
    w = wl.custom("d", N, d_in, d_out, C, rank, 7300 + N, structure=structure)
    r = w.r.copy()
    r[5::23] = -1
    r[7::31] = C
    x, W, A, B = (gpu.dev_bf16(t) for t in (w.x, w.W, w.A, w.B))
    flag = torch.zeros(1, dtype=torch.int32, device="cuda")
    offsets, perm, t = mb.molora_bucket_shrink(gpu.dev_i32(r), x, A, err_flag=flag)
    torch.cuda.synchronize()
    o_ref, p_ref, bad = oracle.bucket(r, C)
    assert np.array_equal(offsets.cpu().numpy(), o_ref) and np.array_equal(perm.cpu().numpy(), p_ref)
    assert int(flag.item()) == 1 and bad > 0
    # t = hi + lo against x A_c in float64, every token and every adapter (two bf16 halves carry
    # 16 significant bits: 2^-17 |t| = 3e-5 at |t| = 4, plus the fp32 sum's ~1e-6)
    tt = t.float().cpu().numpy().astype(np.float64).reshape(N, 2, C, rank)
    x64 = wl.bf16_bits_to_f32(w.x).astype(np.float64)
    for c in range(C):
        ref_t = x64 @ wl.bf16_bits_to_f32(w.A[c]).astype(np.float64)
        got_t = tt[:, 0, c, :] + tt[:, 1, c, :]
        assert np.max(np.abs(got_t - ref_t) / np.maximum(1.0, np.abs(ref_t))) <= 2e-5, f"t of adapter {c}"
    h = mb.molora_base_expand_dense(x, W, B, t, offsets, perm)
    torch.cuda.synchronize()
    ref = oracle.apply(w.x, w.W, w.A, w.B, r)
    gpu.assert_h_close(h.cpu().numpy(), ref, "dispatch+shrink, then expand")
    h2 = gpu.gpu_apply(w, r)
    assert torch.equal(h, h2), "molora_apply takes the same path"
    h3 = gpu.gpu_apply(w, r, bucketed=True)
    assert torch.equal(h, h3), "molora_apply_bucketed: the token-order shrink alone, same bits"


@pytest.mark.parametrize("N,d_in,d_out,C,rank,structure", [
    (384, 1024, 8192, 6, 16, "uniform"),    # at most 512 rows, wide output: the choice is 128 x 128 tiles
    (200, 4096, 12288, 16, 64, "zipf"),     # the same with a long K and many column tiles
    (576, 4096, 1024, 8, 32, "uniform"),    # more than 512 rows, narrow output: the choice is the streaming kernel
    (1500, 4104, 520, 5, 24, "zipf"),       # the same, ragged, K tail, 24 row tiles of 64
    (130, 264, 328, 9, 8, "uniform"),       # just above the rows that always stream
    (4096, 512, 72, 3, 8, "uniform"),       # the largest batch the rule looks at
])
def test_kernel_choice_and_forced_tile_heights(gpu, N, d_in, d_out, C, rank, structure):
    """The fused base + expand through the kernel the shape-driven choice picks and through every
    forced row-tile height (64: the streaming kernel at any N; 128 and 256: the tiled kernel,
    also below 512 rows): h against the oracle each time, targets out of range included."""
    import oracle
    import torch
    from paper_2603_15965_amd import binding as mb
    say(f"kernel choice N={N} {d_in}->{d_out} C={C} rank={rank} {structure}")
    w = wl.custom("s", N, d_in, d_out, C, rank, 9700 + N + C, structure=structure)
    r = w.r.copy()
    r[1::19] = -1
    ref = oracle.apply(w.x, w.W, w.A, w.B, r)
    gpu.assert_h_close(gpu.gpu_apply(w, r).cpu().numpy(), ref, "the choice, through molora_apply")
    x, W, A, B = (gpu.dev_bf16(q) for q in (w.x, w.W, w.A, w.B))
    o, p = mb.molora_bucket(gpu.dev_i32(r), C)
    t = mb.molora_shrink(x, A, o, p, workspace="auto")
    for tile_rows in (None, 64, 128, 256):
        h = mb.molora_base_expand(x, W, B, t, o, p, tile_rows=tile_rows)
        torch.cuda.synchronize()
        gpu.assert_h_close(h.cpu().numpy(), ref, f"tile_rows={tile_rows}")


@pytest.mark.parametrize("N,d_in,d_out,C,rank,structure,invalid", [
    (64, 4096, 1024, 16, 64, "zipf", False),    # configuration 3's shape class: K split over 4 slices
    (64, 1024, 264, 16, 64, "uniform", True),   # K split over 2 slices, targets out of range
    (1, 256, 72, 4, 64, "uniform", False),      # one token
    (37, 520, 136, 8, 40, "zipf", True),        # ragged everything, rank not a multiple of 16
    (33, 2048, 64, 3, 128, "uniform", True),    # the widest intermediate
    (50, 264, 64, 1024, 64, "uniform", False),  # as many adapters as the dispatch step allows: most buckets empty
    (64, 512, 128, 2, 48, "all0", False),       # every token in one bucket
])
def test_bucket_shrink_small_one_launch(gpu, N, d_in, d_out, C, rank, structure, invalid):
    """A batch of at most 64 tokens: the dispatch step inside the shrink launch.  offsets and
    perm bit for bit as the oracle's, t bit for bit as molora_bucket followed by molora_shrink
    (with and without the K-split workspace), h as the oracle's and as molora_apply's."""
    import oracle
    import torch
    from paper_2603_15965_amd import binding as mb
    say(f"dispatch inside the shrink N={N} {d_in}->{d_out} C={C} rank={rank} {structure}")
    assert mb.molora_bucket_shrink_small_supported(N, d_in, C, rank)
    w = wl.custom("s", N, d_in, d_out, C, rank, 7500 + N + C, structure=structure)
    r = w.r.copy()
    if invalid:
        r[3::7] = -1
        r[5::11] = C
    x, W, A, B = (gpu.dev_bf16(q) for q in (w.x, w.W, w.A, w.B))
    rd = gpu.dev_i32(r)
    o_ref, p_ref, bad = oracle.bucket(r, C)
    o2, p2 = mb.molora_bucket(rd, C)
    for workspace in (None, "auto"):  # the last t is the one molora_apply computes too
        flag = torch.zeros(1, dtype=torch.int32, device="cuda")
        offsets, perm, t = mb.molora_bucket_shrink_small(rd, x, A, workspace=workspace, err_flag=flag)
        torch.cuda.synchronize()
        assert np.array_equal(offsets.cpu().numpy(), o_ref) and np.array_equal(perm.cpu().numpy(), p_ref)
        assert int(flag.item()) == (1 if bad else 0)
        t2 = mb.molora_shrink(x, A, o2, p2, workspace=workspace)
        torch.cuda.synchronize()
        n_routed = int(o_ref[C])
        assert torch.equal(t[:n_routed], t2[:n_routed]), f"t, workspace={workspace}"
    # t against its definition (reading: two bf16 halves carry 16 significant bits)
    tt = t.float().cpu().numpy().astype(np.float64)
    x64 = wl.bf16_bits_to_f32(w.x).astype(np.float64)
    for p in range(n_routed):
        c = int(np.searchsorted(o_ref, p, side="right") - 1)
        ref_t = x64[p_ref[p]] @ wl.bf16_bits_to_f32(w.A[c]).astype(np.float64)
        got = tt[p, :rank] + tt[p, rank:]
        assert np.max(np.abs(got - ref_t) / np.maximum(1.0, np.abs(ref_t))) <= 2e-5, f"t of sorted position {p}"
    h = mb.molora_base_expand(x, W, B, t, offsets, perm)
    torch.cuda.synchronize()
    ref = oracle.apply(w.x, w.W, w.A, w.B, r)
    gpu.assert_h_close(h.cpu().numpy(), ref, "dispatch inside the shrink, then expand")
    # the two-launch form: dispatch + shrink + h = x W in one launch, then the expand added to h
    o3, p3, t3, h3 = mb.molora_shrink_base_small(rd, x, W, A)
    torch.cuda.synchronize()
    assert np.array_equal(o3.cpu().numpy(), o_ref) and np.array_equal(p3.cpu().numpy(), p_ref)
    t_unsplit = mb.molora_bucket_shrink_small(rd, x, A, workspace=None)[2]
    assert torch.equal(t3[:n_routed], t_unsplit[:n_routed]), "t of the combined launch"
    base = oracle.apply(w.x, w.W, w.A, w.B, np.full(N, -1, dtype=np.int32))   # no adapter anywhere: x W
    gpu.assert_h_close(h3.cpu().numpy(), base, "base projection of the combined launch")
    mb.molora_expand_small(B, t3, o3, p3, h3)
    torch.cuda.synchronize()
    gpu.assert_h_close(h3.cpu().numpy(), ref, "combined launch, then the expand added")
    assert torch.equal(h3, gpu.gpu_apply(w, r)), "molora_apply takes the two-launch path"


@pytest.mark.parametrize("N,d_in,d_out,C,rank,structure", [
    (64, 4096, 1024, 16, 64, "zipf"),      # groups of 32 columns (d_out <= 8192)
    (64, 1024, 14336, 16, 64, "zipf"),     # configuration 3's width: groups of 64 columns
    (37, 520, 8256, 8, 40, "uniform"),     # groups of 64, a K tail (the last piece of W is short)
    (1, 256, 64, 4, 64, "uniform"),        # one token, two groups of 32
    (33, 72, 8320, 3, 128, "uniform"),     # K of one short piece
])
def test_packed_base_weight_small_batch(gpu, N, d_in, d_out, C, rank, structure):
    """The base weight stored column group by column group: molora_pack_w against the
    rearrangement written out in numpy (bit for bit), molora_shrink_base_small on the packed
    weight bit for bit as on the row-major one, and h after the expand as the oracle's."""
    import oracle
    import torch
    from paper_2603_15965_amd import binding as mb
    say(f"packed W N={N} {d_in}->{d_out} C={C} rank={rank}")
    gc = mb.molora_pack_w_cols(d_out)
    assert gc == (32 if d_out <= 8192 else 64)
    w = wl.custom("s", N, d_in, d_out, C, rank, 9100 + N + C, structure=structure)
    r = w.r.copy()
    r[2::9] = -1
    x, W, A, B = (gpu.dev_bf16(q) for q in (w.x, w.W, w.A, w.B))
    rd = gpu.dev_i32(r)
    Wp = mb.molora_pack_w(W)
    torch.cuda.synchronize()
    want = np.concatenate([w.W[k0:k0 + 16].reshape(-1, d_out // gc, gc).transpose(1, 0, 2).ravel()
                           for k0 in range(0, d_in, 16)])   # slab by slab, group after group
    assert np.array_equal(Wp.view(torch.int16).cpu().numpy().view(np.uint16).ravel(), want), "molora_pack_w"
    o1, p1, t1, h1 = mb.molora_shrink_base_small(rd, x, W, A)
    o2, p2, t2, h2 = mb.molora_shrink_base_small(rd, x, Wp, A, packed=True)
    torch.cuda.synchronize()
    n_routed = int(o1[C].item())
    assert torch.equal(o1, o2) and torch.equal(p1, p2) and torch.equal(t1[:n_routed], t2[:n_routed])
    assert torch.equal(h1, h2), "h = x W from the packed weight, same bits"
    h3 = h2.clone()
    mb.molora_expand_small(B, t2, o2, p2, h2)
    torch.cuda.synchronize()
    gpu.assert_h_close(h2.cpu().numpy(), oracle.apply(w.x, w.W, w.A, w.B, r), "packed W, then the expand")
    if rank % 16 == 0:   # the adapters' B packed the same way (a slab of 16 rows lies inside one adapter)
        Bp = mb.molora_pack_b(B)
        torch.cuda.synchronize()
        stacked = w.B.reshape(C * rank, d_out)
        want_b = np.concatenate([stacked[k0:k0 + 16].reshape(-1, d_out // gc, gc).transpose(1, 0, 2).ravel()
                                 for k0 in range(0, C * rank, 16)])
        assert np.array_equal(Bp.view(torch.int16).cpu().numpy().view(np.uint16).ravel(), want_b), "molora_pack_b"
        mb.molora_expand_small(Bp, t2, o2, p2, h3, packed=True)
        torch.cuda.synchronize()
        assert torch.equal(h2, h3), "expand from the packed B, same bits"
    else:
        with pytest.raises(ValueError):
            mb.molora_pack_b(B)


@pytest.mark.parametrize("N,d_in,d_out,C,rank,structure", [
    (1500, 256, 320, 200, 8, "zipf"),       # four buckets of rank 8 per expand tile, a long tail of small buckets
    (1500, 264, 320, 200, 16, "uniform"),   # two of rank 16; ~7 tokens per bucket, a K tail
    (2100, 128, 512, 37, 8, "zipf"),        # the 256-row tile (2100 x 512 gives enough of them)
    (700, 128, 136, 90, 16, "uniform"),     # ragged everything
    (1300, 128, 256, 60, 24, "uniform"),    # 2R = 48: no sharing (not a power of two)
])
def test_many_small_buckets_share_expand_tiles(gpu, N, d_in, d_out, C, rank, structure):
    """Row tiles crossed by many small buckets: buckets of rank 8 / 16 lie side by side in the
    k range of one expand tile.  h against the oracle, targets out of range included."""
    import oracle
    import torch
    say(f"many small buckets N={N} {d_in}->{d_out} C={C} rank={rank} {structure}")
    w = wl.custom("s", N, d_in, d_out, C, rank, 9300 + N + C, structure=structure)
    r = w.r.copy()
    r[4::13] = -1
    r[6::17] = C + 3
    h = gpu.gpu_apply(w, r)
    gpu.assert_h_close(h.cpu().numpy(), oracle.apply(w.x, w.W, w.A, w.B, r), "many small buckets")


@pytest.mark.parametrize("N,d_in,C,rank,structure", [
    (16500, 1024, 12, 32, "zipf"),      # more tiles than compute units: workgroups of four wavefronts
    (16500, 1024, 12, 32, "one"),       # every token on one adapter: its tiles spread over the XCDs
    (9000, 2048, 70, 16, "zipf"),       # more than 64 buckets: two groups in the search; eight wavefronts
    (20000, 1024, 5, 64, "runs"),       # two column groups of the rank
])
def test_streaming_shrink_finds_its_tiles_under_skew(gpu, N, d_in, C, rank, structure):
    """The streaming shrink numbers the 64-row tiles that are in use and every workgroup finds
    its bucket and tile from offsets: skewed, single-target and run-structured routing, some
    targets out of range; h against the oracle."""
    import oracle
    say(f"streaming shrink N={N} d_in={d_in} C={C} rank={rank} {structure}")
    d_out = 64
    w = wl.custom("ss", N, d_in, d_out, C, rank, 9700 + N + C, structure="zipf" if structure == "zipf" else "uniform")
    r = w.r.copy()
    if structure == "one":
        r[:] = C // 2
    elif structure == "runs":
        r = np.repeat(np.random.default_rng(N).integers(0, C, N // 90 + 1), 90)[:N].astype(np.int32)
    r[5::19] = -1
    r[7::23] = C + 1
    h = gpu.gpu_apply(w, r)
    gpu.assert_h_close(h.cpu().numpy(), oracle.apply(w.x, w.W, w.A, w.B, r), "streaming shrink under skew")


def test_gate_dispatch_shrink_matches_separate_calls(gpu):
    """Gating + dispatch + shrink in one launch on configuration 1's shape and on composite
    targets: r, offsets, perm bit for bit as the oracle's, h as the oracle's."""
    import oracle
    import torch
    from paper_2603_15965_amd import binding as mb
    say("gate_dispatch_shrink")
    w = wl.make(wl.shapes()["vocab_q17"])
    x, W, A, B = (gpu.dev_bf16(t) for t in (w.x, w.W, w.A, w.B))
    r, offsets, perm, t = mb.molora_gate_dispatch_shrink(gpu.dev_i32(w.v), w.breaks, x, A)
    h = mb.molora_base_expand_dense(x, W, B, t, offsets, perm)
    torch.cuda.synchronize()
    r_ref = oracle.route_vocab(w.v, w.breaks)
    o_ref, p_ref, _ = oracle.bucket(r_ref, 2)
    assert np.array_equal(r.cpu().numpy(), r_ref)
    assert np.array_equal(offsets.cpu().numpy(), o_ref) and np.array_equal(perm.cpu().numpy(), p_ref)
    gpu.assert_h_close(h.cpu().numpy(), oracle.apply(w.x, w.W, w.A, w.B, r_ref), "config 1, one-launch dispatch")
    # composite targets a * M + m, some invalid
    rng = np.random.default_rng(77)
    N, n_ad, breaks = 3001, 3, (0, 1000, 5000)
    wc = wl.custom("dc", N, 264, 200, n_ad * 2, 8, 7400)
    v = rng.integers(-50, 5100, size=N).astype(np.int32)
    a = rng.integers(-1, n_ad + 1, size=N).astype(np.int32)
    xc, Wc, Ac, Bc = (gpu.dev_bf16(q) for q in (wc.x, wc.W, wc.A, wc.B))
    flag = torch.zeros(1, dtype=torch.int32, device="cuda")
    r, offsets, perm, t = mb.molora_gate_dispatch_shrink(gpu.dev_i32(v), breaks, xc, Ac, adapter=gpu.dev_i32(a),
                                                         n_adapters=n_ad, err_flag=flag)
    h = mb.molora_base_expand_dense(xc, Wc, Bc, t, offsets, perm)
    torch.cuda.synchronize()
    r_ref = oracle.route_compose(v, a, np.array(breaks, dtype=np.int32), n_ad)
    o_ref, p_ref, bad = oracle.bucket(r_ref, n_ad * 2)
    assert np.array_equal(r.cpu().numpy(), r_ref)
    assert np.array_equal(offsets.cpu().numpy(), o_ref) and np.array_equal(perm.cpu().numpy(), p_ref)
    assert int(flag.item()) == (1 if bad else 0)
    gpu.assert_h_close(h.cpu().numpy(), oracle.apply(wc.x, wc.W, wc.A, wc.B, r_ref), "composite targets")


def test_apply_tokens_without_adapter_get_base_only(gpu):
    import oracle
    say("apply with out-of-range targets")
    w = wl.custom("a", 400, 128, 256, 6, 16, 7700)
    r = w.r.copy()
    r[::7] = -1
    r[3::11] = 6
    h = gpu.gpu_apply(w, r).cpu().numpy()
    gpu.assert_h_close(h, oracle.apply(w.x, w.W, w.A, w.B, r), "apply")


def test_apply_bucketed_equals_apply(gpu):
    say("apply_bucketed == apply")
    w = wl.custom("a", 777, 256, 384, 5, 16, 7800)
    h1 = gpu.gpu_apply(w, w.r).cpu().numpy()
    h2 = gpu.gpu_apply(w, w.r, bucketed=True).cpu().numpy()
    assert np.array_equal(h1, h2)


def test_apply_zero_B_and_doubling(gpu):
    # zero-B adapters reduce to the base output; doubling B doubles the low-rank term
    say("apply invariants")
    w = wl.custom("a", 512, 256, 256, 4, 16, 7900)
    none = np.full_like(w.r, -1)
    base = gpu.gpu_apply(w, none).cpu().numpy()
    B0 = w.B.copy(); B0[1] = 0
    w0 = wl.custom("a", 512, 256, 256, 4, 16, 7900); w0.B = B0
    h0 = gpu.gpu_apply(w0, w.r).cpu().numpy()
    sel = w.r == 1
    assert np.array_equal(h0[sel], base[sel])
    assert not np.array_equal(h0[~sel], base[~sel])
    # B -> 2B doubles every product of the expand exactly, so the low-rank term doubles up to
    # the fp32 rounding of the sums it is added into (a few 1e-7 of |h| per element)
    h1 = gpu.gpu_apply(w, w.r).cpu().numpy().astype(np.float64)
    w2 = wl.custom("a", 512, 256, 256, 4, 16, 7900)
    w2.B = wl.to_bf16_bits(2.0 * wl.bf16_bits_to_f32(w.B))
    h2 = gpu.gpu_apply(w2, w.r).cpu().numpy().astype(np.float64)
    b64 = base.astype(np.float64)
    assert np.max(np.abs((h2 - b64) - 2.0 * (h1 - b64))) <= 2e-5 * gpu.rms(h1)
    assert gpu.rms(h1 - b64) > 0.5, "the low-rank term is not small: the check above means something"


def test_kpass_baseline_matches_oracle(gpu):
    """The K-pass per-sequence baseline of the ablation benchmark (one whole-batch pass per
    adapter, rows selected afterwards: the brute force of Thm. "Computational Optimality")
    gives the oracle's per-token result, and the single per-token pass gives the same."""
    import oracle
    import torch
    from paper_2603_15965_amd import baselines
    say("K-pass baseline")
    w = wl.custom("kpass", 1000, 256, 384, 4, 16, 7950)
    r = w.r.copy()
    r[::13] = -1
    x, W, A, B = (gpu.dev_bf16(t) for t in (w.x, w.W, w.A, w.B))
    h = baselines.kpass_apply(x, W, A, B, gpu.dev_i32(r))
    torch.cuda.synchronize()
    ref = oracle.apply(w.x, w.W, w.A, w.B, r)
    gpu.assert_h_close(h.cpu().numpy(), ref, "K passes")
    gpu.assert_h_close(gpu.gpu_apply(w, r).cpu().numpy(), ref, "one pass")


@pytest.mark.parametrize("name", ["tiny", "vocab_q17", "gate_up17", "decode_up8"])
def test_configs_0_to_3_end_to_end(gpu, name):
    import oracle
    w = wl.make(wl.shapes()[name])
    say(f"end-to-end {name}")
    r_gpu = gpu.gpu_route(w)
    r_ref = gpu.oracle_route(w)
    assert np.array_equal(r_gpu.cpu().numpy(), r_ref)
    gpu.check_bucket(r_ref, w.shape.C)
    h_dev = gpu.gpu_apply(w, r_ref)
    h = h_dev.cpu().numpy()
    rel = gpu.assert_h_close(h, oracle.apply(w.x, w.W, w.A, w.B, r_ref), name)
    say(f"  {name}: max err / rms = {rel:.2e}")
    if name == "decode_up8":   # the launch configuration the benchmark times: the two calls on packed weights
        import torch
        from paper_2603_15965_amd import binding as mb
        x, W, A, B = (gpu.dev_bf16(t) for t in (w.x, w.W, w.A, w.B))
        o, p, t, h2 = mb.molora_shrink_base_small(gpu.dev_i32(r_ref), x, mb.molora_pack_w(W), A, packed=True)
        mb.molora_expand_small(mb.molora_pack_b(B), t, o, p, h2, packed=True)
        torch.cuda.synchronize()
        assert torch.equal(h_dev, h2), "decode step on packed weights: same bits as molora_apply"


@pytest.mark.parametrize("proj", ["q", "k", "v", "o", "gate", "up", "down"])
@pytest.mark.parametrize("degenerate", [False, True])
def test_config_4_full_size(gpu, proj, degenerate):
    """All seven full-size projections of the Qwen3-8B-shaped layer, with learned routing and
    with every token on adapter 0, in the launch configuration the benchmark times.  Routing
    and bucketing are compared on all tokens.  h is compared with the oracle on every 16th
    token, every 32nd sorted position and each bucket's first and last row (rows the oracle
    computes one by one; no 256 x 256 output tile is without a sampled row), and as a whole
    through its per-bucket column sums against the float64 definition."""
    import oracle
    import torch
    name = f"prefill8_{proj}" + ("_deg" if degenerate else "")
    w = wl.make(wl.shapes()[name])
    say(f"config 4 {name}")
    r_ref = gpu.oracle_route(w)
    if w.G is not None:
        assert np.array_equal(gpu.gpu_route(w).cpu().numpy(), r_ref)
    offsets, perm = gpu.check_bucket(r_ref, w.shape.C)
    h = gpu.gpu_apply(w, r_ref)
    o, p, _ = oracle.bucket(r_ref, w.shape.C)
    rows = set(range(0, w.shape.N, 16)) | {w.shape.N - 1} | {int(t) for t in p[::32]}
    for c in range(w.shape.C):
        if o[c + 1] > o[c]:
            rows |= {int(p[o[c]]), int(p[o[c + 1] - 1])}
    rows = np.array(sorted(rows), dtype=np.int64)
    pos = np.empty(w.shape.N, dtype=np.int64)
    pos[p] = np.arange(w.shape.N)
    assert len(set((pos[rows] // 128).tolist())) == (w.shape.N + 127) // 128, "a row tile has no sampled row"
    ref = oracle.apply_rows(w.x, w.W, w.A, w.B, r_ref, rows)
    got = h[torch.from_numpy(rows).cuda()].cpu().numpy()
    rel = gpu.assert_h_close(got, ref, name)
    assert bool(torch.isfinite(h).all())
    worst = gpu.check_bucket_column_sums(h, w, r_ref, name)
    say(f"  {name}: {len(rows)} rows, max err / rms = {rel:.2e}, column sums at {worst:.2f} of their bound, "
        f"rms(h) = {float(h.pow(2).mean().sqrt()):.3f}")
