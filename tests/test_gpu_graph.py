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


@pytest.mark.parametrize("B,flags", [(1024, 0), (96, qb.QSDP_FLAG_GRAD_SHIFT)])
def test_replayed_graph_advances_its_seed_from_device_memory(B, flags):
    """One captured iteration = [step counter += 1, fused step seeded from the counter]. Every replay
    must equal the eager step with the seed the counter holds at that replay (kernel arguments are
    frozen at capture, the counter is not)."""
    n = 300 * 1024 + 77
    xh, gh = synth(n, 1600 + B)
    g = torch.from_numpy(gh).to(DEV)
    x = torch.from_numpy(xh).to(DEV)
    counter = torch.zeros(1, dtype=torch.int64, device=DEV)
    codes, meta = qb.alloc_packed(n, 8, B, DEV)
    meta = meta.reshape(-1)

    def iteration():
        counter.add_(1)
        qb.qsdp_fused_step_dseed(x, g, 1e-3, 8, 4, B, 0.0, 1000, counter, 0, flags, codes, meta)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        iteration()                          # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        iteration()
    # restart from known state
    x.copy_(torch.from_numpy(xh).to(DEV))
    counter.zero_()
    x_eager = torch.from_numpy(xh).to(DEV)
    ec, em = qb.alloc_packed(n, 8, B, DEV)
    for replay in range(1, 6):
        graph.replay()
        qb.qsdp_fused_step_ex(x_eager, g, 1e-3, 8, 4, B, 0.0, 1000 + replay, 0, flags, ec, em.reshape(-1))
        torch.cuda.synchronize()
        assert int(counter) == replay
        assert torch.equal(x, x_eager) and torch.equal(codes, ec) and torch.equal(meta, em.reshape(-1)), replay
