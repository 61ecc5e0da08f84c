"""Recorded launch sequences (Sec. "CUDA Graph Compatibility"): a captured route -> bucket ->
apply step must give, on every replay and with refreshed inputs, what the eager calls give,
and what the oracle gives."""
import numpy as np
import pytest

from paper_2603_15965_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _setup(w):
    import torch
    from paper_2603_15965_amd import binding as mb
    shape = w.shape
    d = dict(x=mb.bf16_tensor(w.x), W=mb.bf16_tensor(w.W), A=mb.bf16_tensor(w.A), B=mb.bf16_tensor(w.B),
             G=mb.bf16_tensor(w.G))
    N, C = shape.N, shape.C
    d["r"] = torch.empty(N, dtype=torch.int32, device="cuda")
    d["offsets"] = torch.empty(C + 1, dtype=torch.int32, device="cuda")
    d["perm"] = torch.empty(N, dtype=torch.int32, device="cuda")
    d["h"] = torch.empty((N, shape.d_out), dtype=torch.float32, device="cuda")
    d["ws"] = mb.new_workspace(N, shape.d_in, shape.d_out, C, shape.rank)
    return d


@pytest.mark.parametrize("N", [300, 48])
def test_captured_step_replays(N):
    import torch
    import oracle
    from paper_2603_15965_amd import binding as mb
    import gpu_helpers as gpu
    print(f"graph replay N={N}", flush=True)
    w = wl.custom("graph_step", N, 512, 384, 5, 16, wl.BASE_SEED + 7700 + N, route="gate")
    shape = w.shape
    d = _setup(w)
    side = torch.cuda.Stream()

    def step(stream):
        mb.molora_route(d["x"], d["G"], d["r"], stream=stream)
        mb.molora_bucket(d["r"], shape.C, d["offsets"], d["perm"], stream=stream)
        mb.molora_apply_bucketed(d["x"], d["W"], d["A"], d["B"], d["offsets"], d["perm"], d["h"],
                                 workspace=d["ws"], stream=stream)

    torch.cuda.synchronize()
    g = mb.Graph(side)
    with g.capture():
        step(side)
    rng = np.random.default_rng(5)
    x_bits = w.x
    for replay in range(4):
        # eager work and a synchronisation between replays; inputs refreshed in place
        if replay > 0:
            x_bits = w.x[rng.permutation(N)]
            d["x"].copy_(mb.bf16_tensor(x_bits))
        d["h"].zero_()
        d["r"].fill_(-7)
        torch.cuda.synchronize()
        g.launch()
        side.synchronize()
        r_gpu = d["r"].cpu().numpy()
        h_gpu = d["h"].cpu().numpy()
        r_ref = oracle.route_gate(x_bits, w.G)
        assert np.array_equal(r_gpu, r_ref), f"replay {replay}"
        gpu.assert_h_close(h_gpu, oracle.apply(x_bits, w.W, w.A, w.B, r_ref), f"replay {replay}")
        # the eager path on the same inputs gives the same bits
        d["h"].zero_()
        step(None)
        torch.cuda.synchronize()
        assert np.array_equal(d["h"].cpu().numpy(), h_gpu), f"replay {replay} vs eager"
    g.destroy()


def test_captured_decode_step_replays():
    """A decode-sized batch (64 tokens, rank 64) through molora_apply: the dispatch runs inside
    the shrink launch, K is split over workgroups with a second pass, then the streaming GEMM.
    Recorded once, replayed with targets and inputs refreshed in place: every replay as the
    oracle's and bit for bit as the eager call."""
    import torch
    import oracle
    from paper_2603_15965_amd import binding as mb
    import gpu_helpers as gpu
    N, d_in, d_out, C, rank = 64, 1024, 392, 16, 64
    print("graph replay, decode-sized batch", flush=True)
    assert mb.molora_bucket_shrink_small_supported(N, d_in, C, rank)
    w = wl.custom("graph_decode", N, d_in, d_out, C, rank, wl.BASE_SEED + 7800, structure="zipf")
    x, W, A, B = (mb.bf16_tensor(q) for q in (w.x, w.W, w.A, w.B))
    r = gpu.dev_i32(w.r)
    h = torch.empty((N, d_out), dtype=torch.float32, device="cuda")
    ws = mb.new_workspace(N, d_in, d_out, C, rank)
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    g = mb.Graph(side)
    with g.capture():
        mb.molora_apply(x, W, A, B, r, h, ws, stream=side)
    rng = np.random.default_rng(9)
    x_bits, r_np = w.x, w.r
    for replay in range(4):
        if replay > 0:
            x_bits = w.x[rng.permutation(N)]
            r_np = rng.integers(-1, C + 1, size=N).astype(np.int32)  # some tokens without adapter
            x.copy_(mb.bf16_tensor(x_bits))
            r.copy_(gpu.dev_i32(r_np))
        h.zero_()
        torch.cuda.synchronize()
        g.launch()
        side.synchronize()
        h_gpu = h.cpu().numpy()
        gpu.assert_h_close(h_gpu, oracle.apply(x_bits, w.W, w.A, w.B, r_np), f"replay {replay}")
        h.zero_()
        mb.molora_apply(x, W, A, B, r, h, ws)
        torch.cuda.synchronize()
        assert np.array_equal(h.cpu().numpy(), h_gpu), f"replay {replay} vs eager"
    g.destroy()


def test_captured_seven_projection_layer():
    """The whole Qwen3-8B-shaped layer of configuration 4 at full size (seven projections,
    N = 16384, each route -> bucket -> apply) recorded as ONE launch sequence, the form the
    benchmark replays with --graph.  Every replay (inputs refreshed in place, eager work and a
    synchronisation in between) must reproduce the eager calls bit for bit (r, offsets, perm, h
    of every projection), and h is compared with the oracle on every 64th token."""
    import torch
    import oracle
    from paper_2603_15965_amd import binding as mb
    import gpu_helpers as gpu
    names = [f"prefill8_{p}" for p in ("q", "k", "v", "o", "gate", "up", "down")]
    side = torch.cuda.Stream()
    P = []
    for name in names:
        print(f"layer graph: inputs of {name}", flush=True)
        w = wl.make(wl.shapes()[name])
        d = _setup(w)
        d["w"] = w
        P.append(d)

    def step(stream):
        for d in P:
            sh = d["w"].shape
            mb.molora_route(d["x"], d["G"], d["r"], stream=stream)
            mb.molora_bucket(d["r"], sh.C, d["offsets"], d["perm"], stream=stream)
            mb.molora_apply_bucketed(d["x"], d["W"], d["A"], d["B"], d["offsets"], d["perm"], d["h"],
                                     workspace=d["ws"], stream=stream)

    step(None)  # eager reference of the first inputs (also: first launches outside capture)
    torch.cuda.synchronize()
    g = mb.Graph(side)
    with g.capture():
        step(side)
    rows = np.arange(0, P[0]["w"].shape.N, 64, dtype=np.int64)
    rows_d = torch.from_numpy(rows).cuda()
    for replay in range(3):
        print(f"layer graph: replay {replay}", flush=True)
        if replay > 0:  # refresh every projection's x in place: rows rolled by a fixed amount
            for d in P:
                d["x"].copy_(torch.roll(d["x"], 1000 * replay + 1, dims=0))
        step(None)
        torch.cuda.synchronize()
        eager = [{k: d[k].clone() for k in ("r", "offsets", "perm", "h")} for d in P]
        for d in P:
            d["h"].zero_()
            d["r"].fill_(-7)
            d["perm"].fill_(-1)
        torch.cuda.synchronize()
        g.launch()
        side.synchronize()
        for d, e, name in zip(P, eager, names):
            for k in ("r", "offsets", "perm", "h"):
                assert torch.equal(d[k], e[k]), f"replay {replay}: {k} of {name} differs from the eager call"
        if replay != 1:
            continue
        for d, name in zip(P, names):  # one replay against the oracle, on sampled rows
            w = d["w"]
            x_bits = np.roll(w.x, 1001, axis=0)
            r_gpu = d["r"].cpu().numpy()
            ref = oracle.apply_rows(x_bits, w.W, w.A, w.B, r_gpu, rows)
            gpu.assert_h_close(d["h"][rows_d].cpu().numpy(), ref, f"replayed {name}")
            sample = rows[::8]
            assert np.array_equal(r_gpu[sample], oracle.route_gate(x_bits[sample], w.G)), name
    g.destroy()
