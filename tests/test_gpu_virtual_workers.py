"""Algorithm 2's data flow with P virtual workers on one GPU (examples/virtual_workers.py): the
entry points working together. A CPU twin built from the oracle's routines must give the same
weights bit for bit, and the quantized iteration must drive the toy objective down to the level
its grid allows."""
import os
import sys

import numpy as np
import pytest
import torch

from oracle import ref
from gpu_util import DEV, bits_equal

sys.path.insert(0, os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "examples"))
import virtual_workers as vw  # noqa: E402

pytestmark = pytest.mark.gpu


def cpu_twin(x0, targets, steps, lr, wbits, gbits, B, delta, seed0, flags=0, adamw=None):
    P, n = targets.shape
    lay = vw.layout(n, P, B, wbits, gbits)
    shard = lay["shard"]
    bounds = [(s * shard, min((s + 1) * shard, n)) for s in range(P)]
    x = x0.copy()
    mom, var = np.zeros(n, np.float32), np.zeros(n, np.float32)
    slots = []
    for a, b in bounds:
        c, m, _ = ref.quantize_weight(x[a:b], wbits, B, delta, seed0)
        slots.append((c, m))
    decoded = []
    for t in range(steps):
        w = np.concatenate([ref.dequantize(c, m, b - a, wbits, B) for (c, m), (a, b) in zip(slots, bounds)])
        decoded.append(w)
        grads = []
        for p in range(P):
            g = w - targets[p]
            grads.append(ref.quantize_grad(g, gbits, B, seed0 + 1000 * (t + 1) + p))
        for s, (a, b) in enumerate(bounds):
            nb = -(-(b - a) // B)
            gw = nb * B * gbits // 32
            cs = np.stack([c[s * lay["gwords"]: s * lay["gwords"] + gw] for c, _ in grads])
            ms = np.stack([m.reshape(-1)[s * lay["mfloats"]: s * lay["mfloats"] + 2 * nb] for _, m in grads])
            if adamw:
                b1, b2, eps, wd = adamw
                x[a:b], mom[a:b], var[a:b], wc, wm, _ = ref.recv_adamw_step(
                    x[a:b], mom[a:b], var[a:b], cs, ms, P, 1.0 / P, lr, b1, b2, eps, wd, 1.0 - b1 ** (t + 1),
                    1.0 - b2 ** (t + 1), wbits, gbits, B, delta, seed0 + t, flags=flags, emit_codes=True)
            else:
                x[a:b], wc, wm, _ = ref.recv_step(x[a:b], cs, ms, P, 1.0 / P, lr, wbits, gbits, B, delta, seed0 + t,
                                                  flags=flags, emit_codes=True)
            slots[s] = (wc, wm)
    return x, decoded


@pytest.mark.parametrize("n,P,wbits,gbits,B,delta", [
    (8 * 2048 + 300, 4, 8, 4, 1024, 0.0),
    (5 * 384 - 50, 5, 4, 8, 128, 0.0),
    (3 * 4096 + 9, 3, 8, 4, 512, 2.0 ** -9),
])
@pytest.mark.parametrize("keep_master", [False, True])
def test_virtual_workers_match_the_cpu_twin(n, P, wbits, gbits, B, delta, keep_master):
    rng = np.random.default_rng(n)
    x0 = (0.02 * rng.standard_normal(n)).astype(np.float32)
    targets = (0.02 * rng.standard_normal((P, n)) + 0.01).astype(np.float32)
    steps, lr, seed0 = 4, 0.25, 7
    seen = []
    x_gpu, losses = vw.run(torch.from_numpy(x0).to(DEV), torch.from_numpy(targets).to(DEV), steps, lr, wbits,
                           gbits, B, delta, seed0, trace=lambda t, w: seen.append(w.cpu().numpy()),
                           keep_master=keep_master)
    x_cpu, decoded = cpu_twin(x0, targets, steps, lr, wbits, gbits, B, delta, seed0,
                              ref.FLAG_KEEP_MASTER if keep_master else 0)
    for t in range(steps):
        assert bits_equal(seen[t], decoded[t]), t
    assert bits_equal(x_gpu.cpu().numpy(), x_cpu)
    assert len(losses) == steps and losses[-1] < losses[0]


def test_virtual_workers_converge_to_the_grid_floor():
    """8 workers, W8 G4: the loss falls by orders of magnitude and then stays at the floor set by
    the 8-bit weight grid (Section 4.1: convergence to a neighbourhood whose size the grid fixes)."""
    gen = torch.Generator(device=DEV).manual_seed(3)
    n, P = 1 << 18, 8
    x0 = 0.02 * torch.randn(n, device=DEV, generator=gen)
    targets = 0.02 * torch.randn((P, n), device=DEV, generator=gen) + 0.01
    x, losses = vw.run(x0, targets, steps=40, lr=0.3)
    assert losses[-1] < 5e-3 * losses[0]
    # stationary level of x <- x - lr (x - mean + e_g) + e_w: (lr^2 var(e_g) + var(e_w)) / (1 - (1 - lr)^2) per
    # element, with var(e_g) about (gradient cell)^2 / 6 / P (cell = range / 15, range about 0.2) and
    # var(e_w) = (weight cell)^2 / 12: a few 1e-7; the loss is half of that per element
    assert losses[-1] / n < 1e-6
    tail = losses[-10:]
    assert max(tail) < 1.5 * min(tail)


def test_virtual_workers_with_adamw_match_the_cpu_twin():
    """The experiments' configuration in miniature: AdamW on full-precision owner shards, W8 G4."""
    n, P, B = 6 * 1024 + 100, 3, 1024
    rng = np.random.default_rng(12)
    x0 = (0.02 * rng.standard_normal(n)).astype(np.float32)
    targets = (0.02 * rng.standard_normal((P, n)) + 0.01).astype(np.float32)
    adamw = (0.9, 0.95, 1e-8, 0.01)
    x_gpu, losses = vw.run(torch.from_numpy(x0).to(DEV), torch.from_numpy(targets).to(DEV), 5, 2e-3, 8, 4, B, 0.0, 3,
                           keep_master=True, adamw=adamw)
    x_cpu, _ = cpu_twin(x0, targets, 5, 2e-3, 8, 4, B, 0.0, 3, ref.FLAG_KEEP_MASTER, adamw)
    assert bits_equal(x_gpu.cpu().numpy(), x_cpu)
    assert losses[-1] < losses[0]
