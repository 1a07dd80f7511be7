"""The entry points only enqueue kernels on the caller's stream (no allocation, no memset, no
synchronisation), so a sequence of calls can be captured in a HIP graph and replayed. Every
replay is compared with the eager result, with eager work and synchronisations in between."""
import numpy as np
import pytest
import torch

from paper_2302_02390_amd import binding as qb
from gpu_util import DEV, synth

pytestmark = pytest.mark.gpu


def test_captured_steps_replay_identically():
    n, B = 1 << 20, 1024
    xh, gh = synth(n, 1500)
    x0 = torch.from_numpy(xh).to(DEV)
    g = torch.from_numpy(gh).to(DEV)
    codes, meta = qb.alloc_packed(n, 8, B, DEV)
    meta = meta.reshape(-1)
    out = torch.empty(n, dtype=torch.bfloat16, device=DEV)

    def five_steps(x):
        for seed in range(5):
            qb.qsdp_fused_step(x, g, 1e-3, 8, 4, B, 0.0, seed, 0, codes, meta)
        qb.qsdp_dequantize(codes, meta, n, 8, B, out)

    x_eager = x0.clone()
    five_steps(x_eager)
    torch.cuda.synchronize()
    want_x, want_codes, want_out = x_eager.clone(), codes.clone(), out.clone()

    x = x0.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        five_steps(x)                       # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    x.copy_(x0)
    with torch.cuda.graph(graph):
        five_steps(x)
    for replay in range(4):
        x.copy_(x0)
        codes.fill_(-1)
        out.zero_()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(x, want_x) and torch.equal(codes, want_codes) and torch.equal(out, want_out), replay
        # eager work between replays
        tmp = x0.clone()
        qb.qsdp_fused_step(tmp, g, 1e-3, 8, 4, B, 0.0, 99)
        torch.cuda.synchronize()
