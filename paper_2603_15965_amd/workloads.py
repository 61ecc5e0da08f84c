"""Seeded synthetic inputs for the routed-LoRA hot path.

This module holds data preparation only -- random draws, scaling, rounding to bf16
bit patterns and the structure of the routing inputs (run lengths, Zipf draws).  It
contains none of the method's arithmetic (no gate logits, no projections, no
bucketing) so that the CPU oracle and the HIP library can both be fed from it
without sharing code.  bf16 tensors are returned as numpy uint16 bit patterns.

Shapes follow the build's five configurations: Qwen3-1.7B / Qwen3-8B projection
shapes with value distributions x ~ N(0,1), W ~ N(0,1/d_in), A ~ N(0,1/d_in),
B ~ N(0,1/rank), G ~ N(0,1/d_in).  They stand in for the paper's own synthetic
latency workloads (interleaved-modality batches, learned-gate batches, skewed
adapter popularity); no model weights or benchmark data are involved.
"""
from dataclasses import dataclass, field
from typing import Dict, Optional

import numpy as np

BASE_SEED = 20260315
# tensor indices inside a workload's seed block
_T_X, _T_W, _T_A, _T_B, _T_G, _T_R = range(6)


def to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round fp32 values to bf16 (round-to-nearest-even) and return the uint16 bits."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    rounded = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return rounded.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to fp32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def normal_bf16(seed: int, shape, std: float) -> np.ndarray:
    rng = np.random.Generator(np.random.PCG64(seed))
    a = rng.standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    return to_bf16_bits(a)


@dataclass
class Shape:
    """One adapted projection: N tokens, d_in -> d_out, C adapters of rank `rank`."""
    name: str
    N: int
    d_in: int
    d_out: int
    C: int
    rank: int
    route: str            # "given" | "vocab" | "gate"
    seed_block: int       # added to BASE_SEED
    structure: str = ""   # how the given r / token ids are drawn


@dataclass
class Workload:
    shape: Shape
    x: np.ndarray                       # bf16 bits [N][d_in]
    W: np.ndarray                       # bf16 bits [d_in][d_out]
    A: np.ndarray                       # bf16 bits [C][d_in][rank]
    B: np.ndarray                       # bf16 bits [C][rank][d_out]
    G: Optional[np.ndarray] = None      # bf16 bits [d_in][C]      (route == "gate")
    r: Optional[np.ndarray] = None      # int32 [N]                (route == "given")
    v: Optional[np.ndarray] = None      # int32 [N] token ids      (route == "vocab")
    breaks: Optional[np.ndarray] = None  # int32 [M+1]             (route == "vocab")
    extra: Dict = field(default_factory=dict)


QWEN3_8B_LAYER = [  # (projection, d_in, d_out)
    ("q", 4096, 4096), ("k", 4096, 1024), ("v", 4096, 1024), ("o", 4096, 4096),
    ("gate", 4096, 12288), ("up", 4096, 12288), ("down", 12288, 4096),
]


def shapes() -> Dict[str, Shape]:
    s = {}
    s["tiny"] = Shape("tiny", 256, 256, 256, 4, 8, "given", 0, "uniform")
    s["vocab_q17"] = Shape("vocab_q17", 4096, 2048, 2048, 2, 16, "vocab", 1000, "runs")
    s["gate_up17"] = Shape("gate_up17", 8192, 2048, 6144, 8, 16, "gate", 2000)
    s["decode_up8"] = Shape("decode_up8", 64, 4096, 12288, 16, 64, "given", 3000, "zipf")
    for j, (p, di, do) in enumerate(QWEN3_8B_LAYER):
        s[f"prefill8_{p}"] = Shape(f"prefill8_{p}", 16384, di, do, 32, 32, "gate", 4000 + 100 * j)
        s[f"prefill8_{p}_deg"] = Shape(f"prefill8_{p}_deg", 16384, di, do, 32, 32, "given",
                                       4000 + 100 * j, "all0")
    return s


CONFIGS = {  # the five configurations -> their projections
    0: ["tiny"],
    1: ["vocab_q17"],
    2: ["gate_up17"],
    3: ["decode_up8"],
    4: [f"prefill8_{p}" for p, _, _ in QWEN3_8B_LAYER],
}

# vocabulary layout of the interleaved text/image stand-in: text ids [0, 32768),
# image ids [32768, 40960)
VOCAB_BREAKS = np.array([0, 32768, 40960], dtype=np.int32)


def interleaved_token_ids(seed: int, n_seq: int, seq_len: int, mean_run: float,
                          breaks: np.ndarray) -> np.ndarray:
    """Token ids of n_seq sequences made of alternating modality runs.

    Every sequence starts in modality 0; run lengths are geometric on {1, 2, ...}
    with mean `mean_run` (P(L = l) = p (1-p)^(l-1), p = 1/mean_run); the modality
    advances cyclically after each run; the last run is cut at seq_len; ids are
    uniform inside the run's vocabulary range.
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    M = len(breaks) - 1
    p = 1.0 / mean_run
    ids = np.empty(n_seq * seq_len, dtype=np.int32)
    for s in range(n_seq):
        pos, m = 0, 0
        while pos < seq_len:
            run = min(int(rng.geometric(p)), seq_len - pos)
            lo, hi = int(breaks[m]), int(breaks[m + 1])
            ids[s * seq_len + pos: s * seq_len + pos + run] = rng.integers(lo, hi, size=run)
            pos += run
            m = (m + 1) % M
    return ids


def zipf_targets(seed: int, n: int, C: int, s: float) -> np.ndarray:
    """n draws from P(c) proportional to (c+1)^-s on {0..C-1}, by inverse CDF."""
    rng = np.random.Generator(np.random.PCG64(seed))
    w = (np.arange(1, C + 1, dtype=np.float64)) ** (-s)
    cdf = np.cumsum(w / w.sum())
    u = rng.random(n)
    return np.minimum(np.searchsorted(cdf, u, side="right"), C - 1).astype(np.int32)


def uniform_targets(seed: int, n: int, C: int) -> np.ndarray:
    rng = np.random.Generator(np.random.PCG64(seed))
    return rng.integers(0, C, size=n).astype(np.int32)


def skewed_targets(seed: int, n: int, probs) -> np.ndarray:
    """n draws with the given per-target probabilities (e.g. 0.8/0.1/0.05/0.05)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    probs = np.asarray(probs, dtype=np.float64)
    return rng.choice(len(probs), size=n, p=probs / probs.sum()).astype(np.int32)


def make(shape: Shape, want=("x", "W", "A", "B", "route")) -> Workload:
    """Draw the tensors of one projection.  `want` limits what is generated."""
    sd = BASE_SEED + shape.seed_block
    N, di, do, C, rk = shape.N, shape.d_in, shape.d_out, shape.C, shape.rank
    empty = np.empty(0, dtype=np.uint16)
    x = normal_bf16(sd + _T_X, (N, di), 1.0) if "x" in want else empty
    W = normal_bf16(sd + _T_W, (di, do), di ** -0.5) if "W" in want else empty
    A = normal_bf16(sd + _T_A, (C, di, rk), di ** -0.5) if "A" in want else empty
    B = normal_bf16(sd + _T_B, (C, rk, do), rk ** -0.5) if "B" in want else empty
    wl = Workload(shape, x, W, A, B)
    if "route" in want:
        if shape.route == "gate":
            wl.G = normal_bf16(sd + _T_G, (di, C), di ** -0.5)
        elif shape.route == "vocab":
            wl.breaks = VOCAB_BREAKS.copy()
            wl.v = interleaved_token_ids(sd + _T_R, N // 512, 512, 32.0, wl.breaks)
        elif shape.structure == "uniform":
            wl.r = uniform_targets(sd + _T_R, N, C)
        elif shape.structure == "zipf":
            wl.r = zipf_targets(sd + _T_R, N, C, 1.1)
        elif shape.structure == "all0":
            wl.r = np.zeros(N, dtype=np.int32)
        else:
            raise ValueError(f"unknown structure {shape.structure!r}")
    return wl


def custom(name: str, N: int, d_in: int, d_out: int, C: int, rank: int, seed: int,
           route: str = "given", structure: str = "uniform") -> Workload:
    """A free-form workload with the standard distributions (used by the tests)."""
    return make(Shape(name, N, d_in, d_out, C, rank, route, seed - BASE_SEED, structure))
