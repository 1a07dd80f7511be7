"""Pins of the oracle's receive-side AdamW step (P workers' quantized gradients averaged, AdamW
on the owner's partition, Q^w of the result)."""
import numpy as np
import pytest
import torch

from oracle import ref

KEEP = ref.FLAG_KEEP_MASTER


def _setup(n, B, P, gbits, seed):
    rng = np.random.default_rng(seed)
    x = (0.02 * rng.standard_normal(n)).astype(np.float32)
    cs, ms = [], []
    for p in range(P):
        g = (1e-3 * rng.standard_t(3, n)).astype(np.float32)
        c, m = ref.quantize_grad(g, gbits, B, 40 + p)
        cs.append(c); ms.append(m.reshape(-1))
    return x, np.stack(cs), np.stack(ms)


@pytest.mark.parametrize("n,B,P,gbits,wbits", [(700, 128, 4, 4, 8), (500, 96, 3, 3, 5), (3000, 1024, 8, 8, 6)])
def test_follows_torch_adamw_on_the_averaged_decoded_gradient(n, B, P, gbits, wbits):
    """KEEP_MASTER: five steps against torch.optim.AdamW (float64) fed with the decode-and-average of
    the same slices; moments and weights agree to float32 rounding, codes are Q^w of the weights."""
    x, cs, ms = _setup(n, B, P, gbits, n)
    ghat = ref.dequantize_add(cs, ms, P, n, gbits, B, 1.0 / P)
    b1, b2, eps, wd, lr = 0.9, 0.95, 1e-8, 0.1, 2e-3
    xt = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.AdamW([xt], lr=lr, betas=(b1, b2), eps=eps, weight_decay=wd)
    xo, m, v = x.copy(), np.zeros(n, np.float32), np.zeros(n, np.float32)
    for t in range(1, 6):
        xt.grad = torch.tensor(ghat, dtype=torch.float64)
        opt.step()
        xo, m, v, wc, wm, _ = ref.recv_adamw_step(xo, m, v, cs, ms, P, 1.0 / P, lr, b1, b2, eps, wd, 1 - b1 ** t,
                                                  1 - b2 ** t, wbits, gbits, B, 0.0, t, flags=KEEP, emit_codes=True)
        c2, m2, _ = ref.quantize_weight(xo, wbits, B, 0.0, t)
        assert np.array_equal(wc, c2) and np.array_equal(wm.view(np.uint32), m2.view(np.uint32))
    st = opt.state[xt]
    assert np.allclose(m, st["exp_avg"].numpy(), rtol=1e-5, atol=1e-12)
    assert np.allclose(v, st["exp_avg_sq"].numpy(), rtol=1e-5, atol=1e-16)
    assert np.allclose(xo, xt.detach().numpy(), rtol=2e-5, atol=1e-8)


def test_one_peer_equals_the_single_worker_adamw_step_on_grid_gradients():
    """One peer, alpha = 1, a gradient that lies on its own 8-bit grid: the slice decodes to g and
    Q^g(g) = g in the single-worker routine too, so both routines must agree bit for bit."""
    B, n = 64, 256
    rng = np.random.default_rng(9)
    k = rng.integers(0, 256, size=n); k[::B] = 0; k[1::B] = 255
    g = (k.astype(np.float32) * np.float32(2.0 ** -12)) - np.float32(0.03125)
    x = (0.02 * rng.standard_normal(n)).astype(np.float32)
    c, mm = ref.quantize_grad(g, 8, B, 3)
    assert np.array_equal(ref.dequantize(c, mm, n, 8, B), g)
    z = np.zeros(n, np.float32)
    args = (2e-3, 0.9, 0.95, 1e-8, 0.01, 0.1, 0.05)
    a = ref.fused_adamw_step(x, g, z, z, *args, 8, 8, B, 0.0, 3, emit_codes=True)
    b = ref.recv_adamw_step(x, z, z, c[None], mm.reshape(1, -1), 1, 1.0, *args, 8, 8, B, 0.0, 3, emit_codes=True)
    for u, w in zip(a[:5], b[:5]):
        assert np.array_equal(np.ascontiguousarray(u).view(np.uint32), np.ascontiguousarray(w).view(np.uint32))


def test_without_keep_master_the_iterate_is_the_decode_of_the_codes():
    x, cs, ms = _setup(900, 128, 4, 4, 2)
    z = np.zeros(900, np.float32)
    xo, m, v, wc, wm, _ = ref.recv_adamw_step(x, z, z, cs, ms, 4, 0.25, 2e-3, 0.9, 0.95, 1e-8, 0.0, 0.1, 0.05, 8, 4, 128,
                                              0.0, 1, emit_codes=True)
    assert np.array_equal(ref.dequantize(wc, wm, 900, 8, 128).view(np.uint32), xo.view(np.uint32))
    xk, mk, vk, wck, wmk, _ = ref.recv_adamw_step(x, z, z, cs, ms, 4, 0.25, 2e-3, 0.9, 0.95, 1e-8, 0.0, 0.1, 0.05, 8,
                                                  4, 128, 0.0, 1, flags=KEEP, emit_codes=True)
    assert np.array_equal(wc, wck) and np.array_equal(m, mk) and np.array_equal(v, vk)
    cell = np.repeat(wm[:, 1], 128)[:900].astype(np.float64)
    assert np.all(np.abs(xo.astype(np.float64) - xk) <= 0.5 * cell * (1 + 1e-5) + 1e-12)


def test_rejects_bad_arguments():
    x, cs, ms = _setup(256, 128, 2, 4, 3)
    z = np.zeros(256, np.float32)
    with pytest.raises(Exception):
        ref.recv_adamw_step(x, z, z, cs, ms, 2, 0.5, 1e-3, 1.0, 0.95, 1e-8, 0.0, 0.1, 0.05, 8, 4, 128, 0.0, 0)
    with pytest.raises(Exception):
        ref.recv_adamw_step(x, z, z, cs, ms, 2, 0.5, 1e-3, 0.9, 0.95, 1e-8, 0.0, 0.1, 0.05, 8, 4, 128, 0.0, 0,
                            flags=ref.FLAG_GRAD_SHIFT)
