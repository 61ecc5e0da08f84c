"""The launch timer: the device-side duration of a base-projection launch, taken from the
launch's own dispatch.  It must not change the result, must lie inside the interval that a
pair of recorded events around the call measures, and must say so when no launch took it."""
import numpy as np
import pytest

from paper_2603_15965_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("N,d_in,d_out,C,rank", [
    (1024, 512, 512, 4, 32),    # the tiled GEMM
    (200, 512, 256, 4, 32),     # the small-batch GEMM
    (48, 512, 256, 6, 64),      # a decode-sized batch: the timer goes to the first of its two launches
])
def test_launch_timer_brackets_the_base_projection(N, d_in, d_out, C, rank):
    import torch
    import gpu_helpers as gpu
    from paper_2603_15965_amd import binding as mb
    print(f"launch timer N={N} {d_in}->{d_out} C={C} rank={rank}", flush=True)
    w = wl.custom("timer", N, d_in, d_out, C, rank, 5100 + N)
    x, W, A, B = (gpu.dev_bf16(q) for q in (w.x, w.W, w.A, w.B))
    r = gpu.dev_i32(w.r)
    h0 = mb.molora_apply(x, W, A, B, r)
    torch.cuda.synchronize()
    timer = mb.LaunchTimer()
    with pytest.raises(RuntimeError):   # armed by nobody, taken by no launch
        timer.elapsed_us()
    for _ in range(2):                  # a timer can be used again after it has been read
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        timer.arm()
        h1 = mb.molora_apply(x, W, A, B, r)
        e1.record()
        torch.cuda.synchronize()
        us = timer.elapsed_us()
        around = e0.elapsed_time(e1) * 1e3
        assert 0.5 < us < around, f"kernel {us} us, events around the whole call {around} us"
        assert torch.equal(h0, h1), "the timed launch computes the same bits"
    h2 = mb.molora_apply(x, W, A, B, r)   # the pair was consumed: an ordinary launch again
    torch.cuda.synchronize()
    assert torch.equal(h0, h2)
    timer.destroy()
