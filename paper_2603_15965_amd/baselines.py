"""Comparison paths built from this library's own kernels (for the ablation benchmarks and
their parity tests); not part of the hot path."""
import torch

from . import binding as mb


def kpass_apply(x, W, A, B, r, h=None, h_pass=None, workspace=None, r_pass=None, stream=None,
                base_pass=True):
    """Per-sequence routing as the paper prices it (Table "tab:passes", Thm. "Computational
    Optimality": K * N work against N): one pass of the WHOLE batch per adapter, every token
    through adapter c in pass c, and the rows whose target is c kept from that pass.  Tokens
    without adapter keep the base output x W, which takes one more pass (base_pass=False leaves
    it out: K passes exactly, for batches in which every token has a target).  Returns h
    [N][d_out] fp32."""
    N, d_in, d_out, C, rank = mb._shapes(x, W, A, B)
    if h is None:
        h = torch.empty((N, d_out), dtype=torch.float32, device=x.device)
    if h_pass is None:
        h_pass = torch.empty_like(h)
    if workspace is None:
        workspace = mb.new_workspace(N, d_in, d_out, C, rank, x.device)
    if r_pass is None:
        r_pass = [torch.full((N,), c, dtype=torch.int32, device=x.device) for c in range(-1, C)]
    if base_pass:  # pass "-1": no adapter at all, the rows of unrouted tokens
        mb.molora_apply(x, W, A, B, r_pass[0], h=h, workspace=workspace, stream=stream)
    for c in range(C):
        first = c == 0 and not base_pass
        mb.molora_apply(x, W, A, B, r_pass[c + 1], h=h if first else h_pass, workspace=workspace,
                        stream=stream)
        if not first:
            torch.where((r == c).unsqueeze(1), h_pass, h, out=h)
    return h
