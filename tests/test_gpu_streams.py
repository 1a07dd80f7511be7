"""The library keeps no state and launches on the stream it is given: calls issued on two
non-default streams at once give the same results as the same calls one after the other."""
import pytest
import torch

from paper_2302_02390_amd import binding as qb
from paper_2302_02390_amd import workloads as wl
from gpu_util import DEV

pytestmark = pytest.mark.gpu


def test_two_streams_at_once_equal_sequential_calls():
    n, B = 24 * 1024 * 1024 + 300, 1024
    xs = [wl.weights(n, 50 + k, DEV) for k in range(2)]
    gs = [wl.grads_student_t3(n, 60 + k, DEV) for k in range(2)]
    want = []
    for k in range(2):
        x = xs[k].clone()
        c, m = qb.alloc_packed(n, 8, B, DEV)
        for step in range(3):
            qb.qsdp_fused_step(x, gs[k], 1e-3, 8, 4, B, 0.0, step, 0, c, m.reshape(-1))
        want.append((x, c, m))
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(device=DEV) for _ in range(2)]      # default priority
    got = []
    for k in range(2):
        got.append((xs[k].clone(), *qb.alloc_packed(n, 8, B, DEV)))
    torch.cuda.synchronize()
    for step in range(3):                                             # interleave the two streams
        for k in range(2):
            with torch.cuda.stream(streams[k]):
                x, c, m = got[k]
                qb.qsdp_fused_step(x, gs[k], 1e-3, 8, 4, B, 0.0, step, 0, c, m.reshape(-1))
    for s in streams:
        s.synchronize()
    for k in range(2):
        assert torch.equal(got[k][0], want[k][0])
        assert torch.equal(got[k][1], want[k][1]) and torch.equal(got[k][2], want[k][2])
