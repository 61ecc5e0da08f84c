#!/usr/bin/env python3
"""Benchmark of the routed-LoRA hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic input that is already
resident in HBM:  route (vocabulary or learned gate; skipped when r is given) -> bucket ->
shrink -> fused base GEMM + expand, every call through the C ABI of libmolora.so.  The
default workload is configuration 1 (N = 4096 tokens, Qwen3-1.7B q_proj 2048 -> 2048, two
adapters of rank 16, vocabulary-routed interleaved text/image runs).

Prints ONE JSON line: whole-step throughput in tokens/s, the roofline of the dominant kernel
(the fused GEMM) from HIP-event timing of that kernel inside the timed region, and the CPU
oracle timed on the host cores.  Inputs rotate through several independent copies so that
consecutive steps do not find their operands in the 256 MB Infinity Cache.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="vocab_q17",
                    help="a shape name from paper_2603_15965_amd.workloads.shapes()")
    ap.add_argument("--sets", type=int, default=0,
                    help="independent input copies to rotate through (0 = enough for > 600 MB)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-events", action="store_true",
                    help="leave the per-kernel HIP events out of the timed region")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one 256 MiB device copy (reference for rocprofv3 --pmc FETCH_SIZE/WRITE_SIZE)")
    return ap.parse_args()


def algorithmic_work(shape, n_routed, touched):
    """Flops and bytes the method itself needs (x, W, touched A/B, h once; no extra passes)."""
    N, di, do, C, rk = shape.N, shape.d_in, shape.d_out, shape.C, shape.rank
    gemm_flops = 2.0 * N * di * do + 2.0 * n_routed * rk * do
    shrink_flops = 2.0 * n_routed * di * rk
    gate_flops = 2.0 * N * di * C if shape.route == "gate" else 0.0
    gemm_bytes = 2.0 * N * di + 2.0 * di * do + 2.0 * touched * rk * do + 4.0 * n_routed * rk + 4.0 * N * do
    layer_bytes = 2.0 * N * di + 2.0 * di * do + 2.0 * touched * rk * (di + do) + 4.0 * N * do
    if shape.route == "gate":
        layer_bytes += 2.0 * di * C
    return {"gemm_flops": gemm_flops, "shrink_flops": shrink_flops, "gate_flops": gate_flops,
            "gemm_bytes": gemm_bytes, "layer_bytes": layer_bytes,
            "layer_flops": gemm_flops + shrink_flops + gate_flops}


def cpu_baseline(wl_mod, shape):
    """The oracle, as it stands, on the host cores: route + bucket + apply on a bounded
    sample of the same workload."""
    import numpy as np
    import oracle
    w = wl_mod.make(shape)
    N = shape.N
    # bound the CPU work to roughly 10-30 s: ~1e11 flops per second of 8-core work
    flops_per_token = 2.0 * shape.d_in * shape.d_out + 2.0 * shape.rank * (shape.d_in + shape.d_out)
    n_sample = int(min(N, max(64, 1.5e12 // flops_per_token)))
    rows = np.arange(n_sample, dtype=np.int64)
    reps = 3 if n_sample == N and N * flops_per_token < 2e11 else 1
    best = None
    for _ in range(reps):
        t0 = time.perf_counter()
        if w.G is not None:
            r = oracle.route_gate(w.x[:n_sample], w.G)
        elif w.v is not None:
            r = oracle.route_vocab(w.v[:n_sample], w.breaks)
        else:
            r = w.r[:n_sample]
        oracle.bucket(r, shape.C)
        r_full = np.zeros(N, dtype=np.int32)
        r_full[:n_sample] = r
        oracle.apply_rows(w.x, w.W, w.A, w.B, r_full, rows)
        dt = time.perf_counter() - t0
        best = dt if best is None else min(best, dt)
    return {"value": n_sample / best, "unit": "tokens/s", "cores": oracle.num_threads(),
            "kind": "oracle", "seconds": best,
            "sample": f"first {n_sample} of {N} tokens of the same workload, route+bucket+apply, "
                      f"best of {reps}"}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the path needs no exchange between "
              "GPUs: token ranges are independent); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2603_15965_amd import binding as mb
    from paper_2603_15965_amd import workloads as wl_mod

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    mb.load()
    shape = wl_mod.shapes()[args.workload]
    N, di, do, C, rk = shape.N, shape.d_in, shape.d_out, shape.C, shape.rank

    # ---- resident inputs: `sets` independent copies (different seeds for x), rotated ----
    per_set = 2.0 * N * di + 2.0 * di * do + 2.0 * C * rk * (di + do) + 4.0 * N * do
    sets = args.sets if args.sets > 0 else int(max(2, min(64, -(-600e6 // per_set))))
    base = wl_mod.make(shape)
    rng = np.random.default_rng(123)
    S = []
    for s in range(sets):
        d = {}
        # every copy holds the same distributions; copies > 0 are row/element shuffles of copy 0
        x_bits = base.x if s == 0 else base.x[rng.permutation(N)]
        d["x"] = mb.bf16_tensor(x_bits)
        d["W"] = mb.bf16_tensor(base.W if s == 0 else np.roll(base.W, s, axis=0))
        d["A"] = mb.bf16_tensor(base.A if s == 0 else np.roll(base.A, s, axis=1))
        d["B"] = mb.bf16_tensor(base.B if s == 0 else np.roll(base.B, s, axis=1))
        if base.G is not None:
            d["G"] = mb.bf16_tensor(base.G)
        if base.v is not None:
            d["v"] = torch.from_numpy(base.v if s == 0 else np.roll(base.v, 17 * s)).cuda()
        if base.r is not None:
            d["r_given"] = torch.from_numpy(base.r if s == 0 else np.roll(base.r, 17 * s)).cuda()
        d["r"] = torch.empty(N, dtype=torch.int32, device="cuda")
        d["offsets"] = torch.empty(C + 1, dtype=torch.int32, device="cuda")
        d["perm"] = torch.empty(N, dtype=torch.int32, device="cuda")
        d["t"] = torch.empty((N, 2 * rk), dtype=torch.bfloat16, device="cuda")
        d["h"] = torch.empty((N, do), dtype=torch.float32, device="cuda")
        S.append(d)
    breaks = base.breaks

    def step(d, ev=None):
        if "G" in d:
            r = mb.molora_route(d["x"], d["G"], d["r"])
        elif "v" in d:
            r = mb.molora_route_vocab(d["v"], breaks, d["r"])
        else:
            r = d["r_given"]
        mb.molora_bucket(r, C, d["offsets"], d["perm"])
        mb.molora_shrink(d["x"], d["A"], d["offsets"], d["perm"], d["t"])
        if ev is not None:
            ev[0].record()
        mb.molora_base_expand(d["x"], d["W"], d["B"], d["t"], d["offsets"], d["perm"], d["h"])
        if ev is not None:
            ev[1].record()

    if args.copy_calibration:
        a = torch.empty(256 << 20, dtype=torch.uint8, device="cuda")
        b = torch.empty_like(a)
        b.copy_(a)
        torch.cuda.synchronize()

    for i in range(args.warmup):
        step(S[i % sets])
    torch.cuda.synchronize()

    use_ev = not args.no_kernel_events
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
           for _ in range(args.steps)] if use_ev else None
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(S[i % sets], evs[i] if use_ev else None)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = 1e3 * elapsed / args.steps
    gemm_us = (sum(a.elapsed_time(b) for a, b in evs) / args.steps * 1e3) if use_ev else None

    # ---- untimed breakdown of the other kernels (events around each call) ----
    def timed_calls(fn, reps=50):
        es = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for i in range(reps):
            d = S[i % sets]
            es[i][0].record()
            fn(d)
            es[i][1].record()
        torch.cuda.synchronize()
        return sum(a.elapsed_time(b) for a, b in es) / reps * 1e3

    breakdown = {}
    if "G" in S[0]:
        breakdown["route_us"] = timed_calls(lambda d: mb.molora_route(d["x"], d["G"], d["r"]))
    elif "v" in S[0]:
        breakdown["route_us"] = timed_calls(lambda d: mb.molora_route_vocab(d["v"], breaks, d["r"]))
    rsrc = (lambda d: d["r"]) if ("G" in S[0] or "v" in S[0]) else (lambda d: d["r_given"])
    breakdown["bucket_us"] = timed_calls(lambda d: mb.molora_bucket(rsrc(d), C, d["offsets"], d["perm"]))
    breakdown["shrink_us"] = timed_calls(lambda d: mb.molora_shrink(d["x"], d["A"], d["offsets"], d["perm"], d["t"]))
    breakdown["gemm_us"] = timed_calls(lambda d: mb.molora_base_expand(d["x"], d["W"], d["B"], d["t"], d["offsets"], d["perm"], d["h"]))

    offs = S[0]["offsets"].cpu().numpy()
    n_routed = int(offs[C])
    touched = int((np.diff(offs) > 0).sum())
    work = algorithmic_work(shape, n_routed, touched)

    t_gemm = (gemm_us if gemm_us is not None else breakdown["gemm_us"]) * 1e-6
    ai = work["gemm_flops"] / work["gemm_bytes"]
    if ai >= PEAK_BF16_TFLOPS * 1e12 / (PEAK_HBM_GBS * 1e9):
        ach = work["gemm_flops"] / t_gemm / 1e12
        roof = {"bound": "mfma", "achieved": ach, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                "frac": ach / PEAK_BF16_TFLOPS}
    else:
        ach = work["gemm_bytes"] / t_gemm / 1e9
        roof = {"bound": "hbm", "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": ach / PEAK_HBM_GBS}
    traffic = None
    try:  # measured with rocprofv3 --pmc in a separate run (see profiles/)
        with open(os.path.join(ROOT, "profiles", "traffic.json")) as f:
            tj = json.load(f).get(shape.name)
        if tj:
            traffic = tj["read_bytes"] + tj["write_bytes"]
    except (OSError, ValueError, KeyError):
        traffic = None
    roof.update({"kernel": "fused_gemm_kernel (base x.W + grouped expand, unpermuting fp32 store)",
                 "kernel_us": t_gemm * 1e6, "traffic": traffic,
                 "algorithmic_flops": work["gemm_flops"], "algorithmic_bytes": work["gemm_bytes"]})

    out = {
        "metric": "routed-LoRA layer tokens/s",
        "value": N * args.steps / elapsed,
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{shape.name}: N={N} tokens, {di}->{do}, C={C} adapters of rank {rk}, "
                               f"route={shape.route}", "rotating_sets": sets,
                   "kernel_events_in_timed_region": use_ev},
        "roofline": roof,
        "layer": {"tflops": work["layer_flops"] / (elapsed / args.steps) / 1e12,
                  "gbs": work["layer_bytes"] / (elapsed / args.steps) / 1e9,
                  "routed_tokens": n_routed, "touched_adapters": touched},
        "breakdown_us": breakdown,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl_mod, shape)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
