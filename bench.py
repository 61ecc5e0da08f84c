#!/usr/bin/env python3
"""Benchmark of the routed-LoRA hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic input that is already
resident in HBM:  route (vocabulary or learned gate; skipped when r is given) -> bucket ->
shrink -> fused base GEMM + expand, every call through the C ABI of libmolora.so (vocabulary
routing and bucketing share one launch, as in the paper's gating kernel; with a few narrow
adapters, C * rank <= 64, the shrink shares that launch too: molora_gate_dispatch_shrink; a
batch of at most 64 tokens is dispatched inside its shrink launch: molora_bucket_shrink_small).  The
default workload is configuration 1 (N = 4096 tokens, Qwen3-1.7B q_proj 2048 -> 2048, two
adapters of rank 16, vocabulary-routed interleaved text/image runs).

Prints ONE JSON line: whole-step throughput in tokens/s, the roofline of the dominant kernel
(the fused GEMM) from HIP-event timing of that kernel inside the timed region, the per-step
latency distribution (median, P99, coefficient of variation) and the CPU oracle timed on the
host cores.  Inputs rotate through several independent copies so that consecutive steps do
not find their operands in the 256 MB Infinity Cache.

The default run (configuration 1 as `value`) also times the other configurations briefly
(gate_up17, decode_up8 and the seven-projection layer of configuration 4) and reports them
in a `configs` object of the same JSON line: step time, tokens/s, roofline fraction of the
dominant kernel and of the whole step.

--workload prefill8_layer runs all seven projections of configuration 4 in one step;
--graph replays the step from a recorded launch sequence (one per input copy) instead of
launching the kernels one by one.
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
PREWARM_S = 0.15            # untimed steps before the warm-up steps, until the clocks have settled


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="vocab_q17",
                    help="a shape name from paper_2603_15965_amd.workloads.shapes(), or "
                         "prefill8_layer / prefill8_layer_deg (the seven projections of one layer)")
    ap.add_argument("--streams", type=int, default=1,
                    help="launch consecutive steps round-robin on this many streams (independent "
                         "batches overlap; 1 = every step after the previous one)")
    ap.add_argument("--graph", action="store_true",
                    help="replay each step from a recorded launch sequence (HIP graph)")
    ap.add_argument("--sets", type=int, default=0,
                    help="independent input copies to rotate through (0 = enough for > 600 MB)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--timed-only", action="store_true",
                    help="stop after the timed region: no latency pass, no two-stream pass, no per-kernel "
                         "breakdown (for profiler runs, whose per-kernel averages then cover the "
                         "warm-up and the timed region only)")
    ap.add_argument("--no-kernel-events", action="store_true",
                    help="leave the per-kernel HIP events out of the timed region")
    ap.add_argument("--row-major-w", action="store_true",
                    help="decode-sized batches: give the kernel the row-major base weight, not the packed one")
    ap.add_argument("--no-other-configs", action="store_true",
                    help="leave out the short runs of the other configurations (the `configs` object)")
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
    # dispatch + shrink + h = x W in one launch (decode-sized batches): x, W, touched A, t and h once
    first_bytes = 2.0 * N * di + 2.0 * di * do + 2.0 * touched * rk * di + 4.0 * n_routed * rk + 4.0 * N * do
    layer_bytes = 2.0 * N * di + 2.0 * di * do + 2.0 * touched * rk * (di + do) + 4.0 * N * do
    if shape.route == "gate":
        layer_bytes += 2.0 * di * C
    return {"gemm_flops": gemm_flops, "shrink_flops": shrink_flops, "gate_flops": gate_flops,
            "gemm_bytes": gemm_bytes, "first_bytes": first_bytes, "layer_bytes": layer_bytes,
            "layer_flops": gemm_flops + shrink_flops + gate_flops}


LAYER = ["q", "k", "v", "o", "gate", "up", "down"]


def cpu_baseline(wl_mod, shape, budget_flops=1.5e12):
    """The oracle, as it stands, on the host cores: route + bucket + apply on a bounded
    sample of the same workload."""
    import numpy as np
    import oracle
    w = wl_mod.make(shape)
    N = shape.N
    # bound the CPU work to roughly 10-30 s: ~1e11 flops per second of 8-core work
    flops_per_token = 2.0 * shape.d_in * shape.d_out + 2.0 * shape.rank * (shape.d_in + shape.d_out)
    n_sample = int(min(N, max(64, budget_flops // flops_per_token)))
    rows = np.arange(n_sample, dtype=np.int64)
    # a small workload finishes in a fraction of a second: repeat it for about 3 s and quote the
    # median, so that the figure is not one noisy sample
    times = []
    t_all = time.perf_counter()
    while True:
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
        times.append(time.perf_counter() - t0)
        if time.perf_counter() - t_all > 3.0 or len(times) >= 25:
            break
    reps = len(times)
    best = float(np.median(times))
    return {"value": n_sample / best, "unit": "tokens/s", "cores": oracle.num_threads(),
            "kind": "oracle", "seconds": best,
            "sample": f"first {n_sample} of {N} tokens of the same workload, route+bucket+apply, "
                      f"median of {reps} run(s)"}


def run_workload(args, workload, steps, warmup, full):
    """One workload: resident inputs, warm-up, the timed region, and (full=True) the latency,
    two-stream and per-kernel passes plus the CPU baseline.  Returns the JSON object."""
    import numpy as np
    import torch
    from paper_2603_15965_amd import binding as mb
    from paper_2603_15965_amd import workloads as wl_mod

    all_shapes = wl_mod.shapes()
    if workload in ("prefill8_layer", "prefill8_layer_deg"):
        suffix = "_deg" if workload.endswith("_deg") else ""
        shapes = [all_shapes[f"prefill8_{p}{suffix}"] for p in LAYER]
    else:
        shapes = [all_shapes[workload]]
    N = shapes[0].N

    # ---- resident inputs: `sets` independent copies (different seeds for x), rotated ----
    per_set = sum(2.0 * sh.N * sh.d_in + 2.0 * sh.d_in * sh.d_out
                  + 2.0 * sh.C * sh.rank * (sh.d_in + sh.d_out) + 4.0 * sh.N * sh.d_out for sh in shapes)
    sets = args.sets if args.sets > 0 else int(max(2, min(64, -(-600e6 // per_set))))
    if args.sets <= 0 and sets % 2:
        sets += 1  # even: the two-stream pass below gives every copy to one stream
    rng = np.random.default_rng(123)
    S = [[] for _ in range(sets)]
    for sh in shapes:
        base = wl_mod.make(sh)
        C, rk = sh.C, sh.rank
        for s in range(sets):
            d = {"shape": sh, "breaks": base.breaks}
            # every copy holds the same distributions; copies > 0 are row/element shuffles of copy 0
            x_bits = base.x if s == 0 else base.x[rng.permutation(sh.N)]
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
            d["r"] = torch.empty(sh.N, dtype=torch.int32, device="cuda")
            d["offsets"] = torch.empty(C + 1, dtype=torch.int32, device="cuda")
            d["perm"] = torch.empty(sh.N, dtype=torch.int32, device="cuda")
            # a few narrow adapters: dispatch and shrink share one launch and the intermediate is
            # in token order, all adapters side by side
            d["dense"] = mb.molora_dense_shrink_supported(sh.N, sh.d_in, C, rk)
            # a batch of at most 64 tokens: the dispatch runs inside the shrink launch
            d["small"] = mb.molora_bucket_shrink_small_supported(sh.N, sh.d_in, C, rk)
            d["t"] = torch.empty((sh.N, 2 * rk * (C if d["dense"] else 1)), dtype=torch.bfloat16, device="cuda")
            d["sws"] = mb.molora_shrink_workspace(sh.N, sh.d_in, C, rk)  # None for most sizes
            d["h"] = torch.empty((sh.N, sh.d_out), dtype=torch.float32, device="cuda")
            # a decode-sized batch streams the base weight and the touched B_c once: they are given
            # in the layout that stream reads best (slabs of 16 rows, column group after column
            # group: made once per weight by molora_pack_w / molora_pack_b, outside every timed
            # region); same bits out
            d["Wp"], d["Bp"] = None, None
            if d["small"] and base.v is None and not args.row_major_w and mb.molora_pack_w_cols(sh.d_out):
                d["Wp"] = mb.molora_pack_w(d["W"])
                if rk % 16 == 0:
                    d["Bp"] = mb.molora_pack_b(d["B"])
            S[s].append(d)
        del base

    use_packed = [True]  # False: the row-major weight although a packed one is there (second region)

    def route(d, stream=None):
        if "G" in d:
            return mb.molora_route(d["x"], d["G"], d["r"], stream=stream)
        if "v" in d:
            return mb.molora_route_vocab(d["v"], d["breaks"], d["r"], stream=stream)
        return d["r_given"]

    def dispatch_and_shrink(d, stream=None):
        if d["dense"]:  # gating / dispatch and the token-order shrink in ONE launch
            if "v" in d:
                mb.molora_gate_dispatch_shrink(d["v"], d["breaks"], d["x"], d["A"], None, 1, d["r"], d["offsets"],
                                               d["perm"], d["t"], stream=stream)
            else:
                mb.molora_bucket_shrink(route(d, stream), d["x"], d["A"], d["offsets"], d["perm"], d["t"],
                                        stream=stream)
            return
        if d["small"] and "v" not in d:
            # a decode-sized batch: dispatch + shrink + h = x W in ONE launch (the latency-bound
            # shrink hides behind the stream of W); gemm() below then adds the expand
            packed = d["Wp"] is not None and use_packed[0]
            mb.molora_shrink_base_small(route(d, stream), d["x"], d["Wp"] if packed else d["W"], d["A"],
                                        d["offsets"], d["perm"], d["t"], d["h"], stream=stream, packed=packed)
            return
        if "v" in d:  # integer routing: gating inside the dispatch kernel (one launch)
            mb.molora_gate_dispatch(d["v"], d["breaks"], None, 1, d["r"], d["offsets"], d["perm"], stream=stream)
        else:
            mb.molora_bucket(route(d, stream), d["shape"].C, d["offsets"], d["perm"], stream=stream)
        mb.molora_shrink(d["x"], d["A"], d["offsets"], d["perm"], d["t"], workspace=d["sws"], stream=stream)

    def gemm(d, stream=None):
        if d["small"] and "v" not in d:
            packed = d["Bp"] is not None and use_packed[0]
            return mb.molora_expand_small(d["Bp"] if packed else d["B"], d["t"], d["offsets"], d["perm"], d["h"],
                                          stream=stream, packed=packed)
        f = mb.molora_base_expand_dense if d["dense"] else mb.molora_base_expand
        f(d["x"], d["W"], d["B"], d["t"], d["offsets"], d["perm"], d["h"], stream=stream)

    def two_launch(d):  # a decode-sized batch: its dominant kernel is the first launch
        return d["small"] and "v" not in d

    def step(projs, ev=None, stream=None):
        # ev: one launch timer per projection; armed right before the call whose launch holds the
        # base projection, which then records its own start and end on it
        for j, d in enumerate(projs):
            if two_launch(d):
                if ev is not None:
                    ev[j].arm()
                dispatch_and_shrink(d, stream)   # dispatch + shrink + h = x W
                gemm(d, stream)                  # h += t B
                continue
            dispatch_and_shrink(d, stream)
            if ev is not None:
                ev[j].arm()
            gemm(d, stream)

    if args.copy_calibration and full:
        a = torch.empty(256 << 20, dtype=torch.uint8, device="cuda")
        b = torch.empty_like(a)
        b.copy_(a)
        torch.cuda.synchronize()

    # ---- how a step is launched: kernel by kernel, or one recorded sequence per input copy ----
    run_stream = torch.cuda.current_stream()
    graphs = None
    if args.graph:
        run_stream = torch.cuda.Stream()
        step(S[0], stream=run_stream)  # module load and first-touch costs outside the recorded region
        run_stream.synchronize()
        graphs = []
        for s in range(sets):
            g = mb.Graph(run_stream)
            with g.capture():
                step(S[s], stream=run_stream)
            graphs.append(g)

    # several streams: step i runs on stream i % streams with input copy i % sets; the number
    # of copies is a multiple of the number of streams, so a copy is always used by one stream
    extra = []
    if args.streams > 1:
        if graphs is not None or sets % args.streams != 0:
            print("bench.py: --streams needs eager launches and --sets a multiple of it", file=sys.stderr)
            sys.exit(2)
        extra = [torch.cuda.Stream() for _ in range(args.streams)]

    def run_step(i, ev=None):
        if graphs is not None:
            graphs[i % sets].launch()
        elif extra:
            step(S[i % sets], None, stream=extra[i % args.streams])
        else:
            step(S[i % sets], ev)

    # Untimed pre-warm: the chip takes 30-50 ms of sustained work to reach the clocks it then
    # holds (kernel-trace durations fall by 20-25 % over that time), whatever --warmup says; a
    # serving loop runs in that state, so the W warm-up steps and the timed region start there.
    t_pre = time.perf_counter()
    n_pre = 0
    while time.perf_counter() - t_pre < PREWARM_S:
        for _ in range(8):
            run_step(n_pre)
            n_pre += 1
        torch.cuda.synchronize()

    # The dominant kernel is timed inside the timed region by HIP events that the launch itself
    # records at its start and at its end (molora_launch_timer: hipExtLaunchKernelGGL), i.e. the
    # interval a kernel trace reports.  Events recorded around the call are marker packets of
    # their own: they read 5 us more at config 1 (46.0 against 40.7 us, kernel trace 40.1) and
    # cost the stream ~3 us each; a timed launch costs the step ~0.3 us, and every 4th step is
    # timed.  The per-step latency distribution is taken in a second pass after the timed region.
    use_ev = not args.no_kernel_events and graphs is None and not extra
    P = len(shapes)
    EV_EVERY = 4 if steps >= 16 else 1
    ev_steps = [i for i in range(steps) if i % EV_EVERY == EV_EVERY - 1] or [steps - 1]
    evs = {i: [mb.LaunchTimer() for _ in range(P)] for i in ev_steps} if use_ev else {}
    # One untimed burst enqueued exactly as the timed region is (same depth, same events).  The
    # first time a process has this many launches outstanding, the HIP runtime holds the host
    # for ~30 ms once (measured: 30 steps of 4 launches take 33 ms to enqueue the first time and
    # 1.5 ms every time after; what the runtime does in that time was not looked into); the GPU
    # drains and idles meanwhile.  The pre-warm above syncs every 8 steps and never gets that deep, so
    # without this burst the one-off stall landed in the timed region of the workloads whose
    # steps are long enough for the queue to fill.  A serving process pays it once per process.
    for i in range(steps):
        run_step(i, evs.get(i))
    torch.cuda.synchronize()
    for i in range(warmup):
        run_step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        run_step(i, evs.get(i))
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = 1e3 * elapsed / steps
    gemm_us = None
    if use_ev:
        gemm_us = sum(t.elapsed_us() for e in evs.values() for t in e) / len(evs)
        for e in evs.values():
            for t in e:
                t.destroy()

    # the same K steps on the row-major weight, where the step above used the packed one
    row_major = None
    if any(d["Wp"] is not None for d in S[0]) and not args.timed_only and graphs is None:
        use_packed[0] = False
        for i in range(warmup):
            run_step(i)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for i in range(steps):
            run_step(i)
        torch.cuda.synchronize()
        el = time.perf_counter() - t1
        use_packed[0] = True
        row_major = {"ms_per_step": 1e3 * el / steps, "value": N * steps / el, "unit": "tokens/s",
                     "what": "the same steps with W [d_in][d_out] and B [C][rank][d_out] row-major "
                             "(molora_shrink_base_small, molora_expand_small)"}

    skip_passes = bool(extra) or args.timed_only or not full
    latency = None
    if not skip_passes:
        ticks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
        for i in range(steps):
            ticks[i].record(run_stream)
            run_step(i)
        ticks[steps].record(run_stream)
        torch.cuda.synchronize()
        lat = np.array([ticks[i].elapsed_time(ticks[i + 1]) * 1e3 for i in range(steps)])
        latency = {"p50_us": float(np.percentile(lat, 50)), "p99_us": float(np.percentile(lat, 99)),
               "mean_us": float(lat.mean()), "cv": float(lat.std() / lat.mean()),
               "how": "HIP events between consecutive steps on the launch stream, in a second pass "
                      "after the timed region (one event per step adds ~3 us to each)"}

    # ---- same K steps with independent batches overlapping (reported beside `value`) ----
    pipelined = None
    if graphs is None and not skip_passes and sets % 2 == 0:
        two = [torch.cuda.Stream(), torch.cuda.Stream()]
        for i in range(min(warmup, 4)):
            step(S[i % sets], None, stream=two[i % 2])
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for i in range(steps):
            step(S[i % sets], None, stream=two[i % 2])
        torch.cuda.synchronize()
        el2 = time.perf_counter() - t1
        pipelined = {"streams": 2, "value": N * steps / el2, "unit": "tokens/s",
                     "ms_per_step": 1e3 * el2 / steps,
                     "what": "the same steps launched round-robin on two streams, so that the "
                             "latency-bound dispatch and shrink of one batch overlap the GEMM of "
                             "the previous one (every input copy belongs to one stream)"}

    # ---- untimed breakdown of the kernels (events around each call), summed over projections ----
    def timed_calls(fn, reps=30):
        total = 0.0
        for j in range(P):
            es = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
            for i in range(reps):
                d = S[i % sets][j]
                es[i][0].record()
                fn(d)
                es[i][1].record()
            torch.cuda.synchronize()
            total += sum(a.elapsed_time(b) for a, b in es) / reps * 1e3
        return total

    breakdown = {}
    if full and not (args.timed_only and gemm_us is not None):
        if S[0][0]["dense"] or (S[0][0]["small"] and "v" not in S[0][0]):
            breakdown["dispatch_and_shrink_us"] = timed_calls(lambda d: dispatch_and_shrink(d))
        else:
            if "G" in S[0][0] or "v" in S[0][0]:
                breakdown["route_us"] = timed_calls(lambda d: route(d))
            rsrc = (lambda d: d["r"]) if ("G" in S[0][0] or "v" in S[0][0]) else (lambda d: d["r_given"])
            breakdown["bucket_us"] = timed_calls(lambda d: mb.molora_bucket(rsrc(d), d["shape"].C, d["offsets"], d["perm"]))
            breakdown["shrink_us"] = timed_calls(lambda d: mb.molora_shrink(d["x"], d["A"], d["offsets"], d["perm"], d["t"], workspace=d["sws"]))
        breakdown["expand_us" if two_launch(S[0][0]) else "gemm_us"] = timed_calls(lambda d: gemm(d))

    work = None
    n_routed_all, touched_all = [], []
    for d in S[0]:
        offs = d["offsets"].cpu().numpy()
        n_routed, touched = int(offs[d["shape"].C]), int((np.diff(offs) > 0).sum())
        n_routed_all.append(n_routed)
        touched_all.append(touched)
        w1 = algorithmic_work(d["shape"], n_routed, touched)
        work = w1 if work is None else {k: work[k] + w1[k] for k in work}

    first = two_launch(S[0][0])  # the dominant kernel is the first launch (dispatch + shrink + x W)
    dom_key = "dispatch_and_shrink_us" if first else "gemm_us"
    t_gemm = (gemm_us if gemm_us is not None else breakdown[dom_key]) * 1e-6
    dom_bytes = work["first_bytes"] if first else work["gemm_bytes"]
    dom_flops = (work["gemm_flops"] + work["shrink_flops"]) if first else work["gemm_flops"]
    ai = dom_flops / dom_bytes
    if ai >= PEAK_BF16_TFLOPS * 1e12 / (PEAK_HBM_GBS * 1e9):
        ach = dom_flops / t_gemm / 1e12
        roof = {"bound": "mfma", "achieved": ach, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                "frac": ach / PEAK_BF16_TFLOPS}
    else:
        ach = dom_bytes / t_gemm / 1e9
        roof = {"bound": "hbm", "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": ach / PEAK_HBM_GBS}
    # HBM-side bytes per launch are counter readings of separate rocprofv3 --pmc runs of this
    # command, kept under profiles/; they are quoted here (never measured by this run) and only
    # for the library version they were taken on
    traffic, traffic_from = None, None
    try:
        with open(os.path.join(ROOT, "profiles", "traffic.json")) as f:
            tj_all = json.load(f)
        tj = tj_all.get(workload)
        if tj and tj_all.get("_library_version") == mb.version():
            traffic = tj["read_bytes"] + tj["write_bytes"]
            traffic_from = (f"profiles/traffic.json: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of {tj['kernel']} "
                            f"on {tj_all['_library_version']} (a constant of that profile, not of this run)")
    except (OSError, ValueError, KeyError):
        traffic, traffic_from = None, None
    kname = ("small_batch_kernel" if N <= 64 else "fused_gemm_kernel") + \
        " (base x.W + grouped expand, unpermuting fp32 store)"
    if first:
        kname = "shrink_base_small_kernel (dispatch + shrink + base x.W in one launch; the expand follows)"
    if P > 1:
        kname += f", {P} launches per step summed"
    roof.update({"kernel": kname, "kernel_us": t_gemm * 1e6, "traffic": traffic, "traffic_from": traffic_from,
                 "kernel_event_samples": len(evs) if gemm_us is not None else 0,
                 "kernel_us_from": f"HIP events recorded by the launch itself at its start and end "
                                   f"(molora_launch_timer, hipExtLaunchKernelGGL) on every {EV_EVERY}th step of "
                                   f"the timed region"
                 if gemm_us is not None
                 else "HIP events around the call, outside the timed region",
                 "algorithmic_flops": dom_flops, "algorithmic_bytes": dom_bytes})

    # the whole step against the roofline that binds the whole step's algorithmic work
    step_s = elapsed / steps
    if work["layer_flops"] / work["layer_bytes"] >= PEAK_BF16_TFLOPS * 1e12 / (PEAK_HBM_GBS * 1e9):
        step_roof = {"bound": "mfma", "achieved": work["layer_flops"] / step_s / 1e12, "peak": PEAK_BF16_TFLOPS,
                     "unit": "TFLOP/s"}
    else:
        step_roof = {"bound": "hbm", "achieved": work["layer_bytes"] / step_s / 1e9, "peak": PEAK_HBM_GBS,
                     "unit": "GB/s"}
    step_roof["frac"] = step_roof["achieved"] / step_roof["peak"]
    step_roof["what"] = ("algorithmic flops (bytes) of route + shrink + base + expand of one step over the "
                         "wall time of a step, launch gaps included")

    if P == 1:
        sh = shapes[0]
        wname = (f"{sh.name}: N={sh.N} tokens, {sh.d_in}->{sh.d_out}, C={sh.C} adapters of rank {sh.rank}, "
                 f"route={sh.route}")
    else:
        wname = (f"{workload}: N={N} tokens through the seven projections of a Qwen3-8B-shaped layer "
                 f"(q, o 4096->4096; k, v 4096->1024; gate, up 4096->12288; down 12288->4096), "
                 f"C={shapes[0].C} adapters of rank {shapes[0].rank}, route={shapes[0].route} per projection")
    out = {
        "metric": "routed-LoRA layer tokens/s",
        "value": N * steps / elapsed,
        "unit": "tokens/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": wname, "rotating_sets": sets, "prewarm_ms": PREWARM_S * 1e3,
                   "launch": "recorded sequence (HIP graph) per step" if graphs is not None
                   else "kernel by kernel" + (f", steps round-robin on {args.streams} streams" if extra else ""),
                   "kernel_events_in_timed_region": (f"every {EV_EVERY}th step" if use_ev else False),
                   "w_layout": "W and B packed once by molora_pack_w / molora_pack_b (slabs of 16 rows, column "
                               "group after column group); row-major figure under row_major_w"
                   if any(d["Wp"] is not None for d in S[0]) else "row-major [d_in][d_out]"},
        "roofline": roof,
        "step_roofline": step_roof,
        "latency": latency,
        "pipelined": pipelined,
        "row_major_w": row_major,
        "layer": {"tflops": work["layer_flops"] / (elapsed / steps) / 1e12,
                  "gbs": work["layer_bytes"] / (elapsed / steps) / 1e9,
                  "routed_tokens": n_routed_all if P > 1 else n_routed_all[0],
                  "touched_adapters": touched_all if P > 1 else touched_all[0]},
        "breakdown_us": breakdown,
        "breakdown_how": "HIP events recorded around single calls, outside the timed region: every figure "
                         "includes 5-10 us of launch gap and event overhead (the kernels' own durations are "
                         "in profiles/step_<workload>.md; roofline.kernel_us is the launch's own duration)",
    }
    if full and not args.no_cpu_baseline:
        if P == 1:
            out["cpu_baseline"] = cpu_baseline(wl_mod, shapes[0])
        else:  # the same bounded sample of tokens through every projection
            parts = [cpu_baseline(wl_mod, sh, budget_flops=2.5e11) for sh in shapes]
            n_s = min(int(p["value"] * p["seconds"] + 0.5) for p in parts)
            secs = sum(n_s / p["value"] for p in parts)
            out["cpu_baseline"] = {"value": n_s / secs, "unit": "tokens/s", "cores": parts[0]["cores"],
                                   "kind": "oracle", "seconds": secs,
                                   "sample": f"{n_s} tokens per projection (rates of the per-projection "
                                             f"samples combined), route+bucket+apply, seven projections"}
    del S
    torch.cuda.empty_cache()
    return out



OTHER_CONFIGS = [  # (workload, steps, warm-up) of the short runs reported under `configs`
    ("gate_up17", 50, 5), ("decode_up8", 100, 10), ("prefill8_layer", 10, 2)]


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the path needs no exchange between "
              "GPUs: token ranges are independent); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2603_15965_amd import binding as mb

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    mb.load()
    out = run_workload(args, args.workload, args.steps, args.warmup, full=True)
    if args.workload == "vocab_q17" and not (args.timed_only or args.no_other_configs or args.graph
                                             or args.streams > 1):
        others = {}
        for name, st, wu in OTHER_CONFIGS:
            o = run_workload(args, name, min(st, args.steps), min(wu, args.warmup), full=False)
            others[name] = {"workload": o["config"]["workload"], "steps": o["steps"], "warmup": o["warmup"],
                            "ms_per_step": o["ms_per_step"], "tokens_per_s": o["value"],
                            "w_layout": o["config"]["w_layout"], "row_major_w": o["row_major_w"],
                            "kernel": {k: o["roofline"][k] for k in ("kernel", "bound", "achieved", "peak",
                                                                      "unit", "frac", "kernel_us")},
                            "step": o["step_roofline"]}
        out["configs"] = others
    print(json.dumps(out))


if __name__ == "__main__":
    main()
