"""The synthetic input recipes: shapes, distributions and structure."""
import numpy as np

from paper_2603_15965_amd import workloads as wl


def test_bf16_rounding_is_nearest_even():
    vals = np.array([1.0, 1.00390625, 1.01171875, -2.5, 0.0, 3.0e-5], dtype=np.float32)
    # 1 + 2^-8 is a tie between 1.0 and 1 + 2^-7 -> even mantissa (1.0);
    # 1 + 3*2^-8 is a tie between 1+2^-7 and 1+2^-6 -> even mantissa (1+2^-6)
    back = wl.bf16_bits_to_f32(wl.to_bf16_bits(vals))
    assert back[0] == 1.0 and back[1] == 1.0 and back[2] == 1.015625 and back[3] == -2.5
    assert abs(back[5] - vals[5]) <= abs(vals[5]) * 2.0 ** -8


def test_shapes_cover_the_five_configs():
    s = wl.shapes()
    assert (s["tiny"].N, s["tiny"].d_in, s["tiny"].C, s["tiny"].rank) == (256, 256, 4, 8)
    q = s["vocab_q17"]
    assert (q.N, q.d_in, q.d_out, q.C, q.rank, q.route) == (4096, 2048, 2048, 2, 16, "vocab")
    u = s["gate_up17"]
    assert (u.N, u.d_in, u.d_out, u.C, u.rank, u.route) == (8192, 2048, 6144, 8, 16, "gate")
    d = s["decode_up8"]
    assert (d.N, d.d_in, d.d_out, d.C, d.rank) == (64, 4096, 12288, 16, 64)
    assert len(wl.CONFIGS[4]) == 7
    dn = s["prefill8_down"]
    assert (dn.N, dn.d_in, dn.d_out, dn.C, dn.rank, dn.route) == (16384, 12288, 4096, 32, 32, "gate")


def test_tiny_is_deterministic_and_distributed_as_stated():
    a, b = wl.make(wl.shapes()["tiny"]), wl.make(wl.shapes()["tiny"])
    assert np.array_equal(a.x, b.x) and np.array_equal(a.r, b.r) and np.array_equal(a.B, b.B)
    assert abs(wl.bf16_bits_to_f32(a.x).std() - 1.0) < 0.02
    assert abs(wl.bf16_bits_to_f32(a.W).std() - 256 ** -0.5) < 0.002
    assert abs(wl.bf16_bits_to_f32(a.B).std() - 8 ** -0.5) < 0.02
    assert a.r.min() == 0 and a.r.max() == 3


def test_interleaved_runs_alternate_and_have_the_stated_mean():
    ids = wl.interleaved_token_ids(5, 64, 512, 32.0, wl.VOCAB_BREAKS)
    assert ids.shape == (64 * 512,)
    m = (ids >= 32768).astype(np.int8).reshape(64, 512)
    assert np.all(m[:, 0] == 0)                       # every sequence starts with text
    runs = []
    for row in m:
        edges = np.flatnonzero(np.diff(row)) + 1
        lens = np.diff(np.concatenate([[0], edges, [512]]))
        runs.extend(lens[:-1])                         # the last run is truncated
    assert 26.0 < np.mean(runs) < 38.0
    assert ids.min() >= 0 and ids.max() < 40960


def test_zipf_is_skewed_toward_low_indices():
    r = wl.zipf_targets(1, 20000, 16, 1.1)
    cnt = np.bincount(r, minlength=16)
    w = np.arange(1, 17.0) ** -1.1
    assert np.all(np.abs(cnt / 20000 - w / w.sum()) < 0.015)


def test_bench_refuses_more_than_one_gpu():
    """The benchmark measures one GPU; asked for more it says so and exits without touching a GPU."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    p = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True,
                       text=True, timeout=120)
    assert p.returncode != 0
    assert "one GPU" in (p.stderr + p.stdout)
