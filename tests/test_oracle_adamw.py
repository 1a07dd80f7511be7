"""Oracle pins, AdamW inside the quantized iteration (Appendix A: AdamW, betas 0.9/0.95, eps 1e-8)."""
import numpy as np
import pytest
import torch

from oracle import ref


def _on_grid_gradient(n, B, bits, seed):
    """Gradient whose buckets lie exactly on their own min-max grid (power-of-two spacing), so that
    the coin-flip quantizer reproduces it for every seed: Q^g(g) = g."""
    rng = np.random.default_rng(seed)
    L = 2**bits - 1
    k = rng.integers(0, L + 1, size=n)
    kb = k.reshape(-1, B)
    kb[:, 0], kb[:, 1] = 0, L
    return ((kb.astype(np.float64) - 7) * 2.0**-12).astype(np.float32).reshape(-1)


def test_moments_and_step_match_torch_adamw_when_the_gradient_is_on_its_grid():
    B, nb, gbits, wbits = 64, 6, 4, 8
    n = B * nb
    rng = np.random.default_rng(0)
    x0 = (rng.normal(size=n) * 0.02).astype(np.float32)
    lr, b1, b2, eps, wd = 2e-4, 0.9, 0.95, 1e-8, 0.1
    p = torch.nn.Parameter(torch.from_numpy(x0.copy()))
    opt = torch.optim.AdamW([p], lr=lr, betas=(b1, b2), eps=eps, weight_decay=wd)
    x, m, v = x0.copy(), np.zeros(n, np.float32), np.zeros(n, np.float32)
    for t in range(1, 5):
        g = _on_grid_gradient(n, B, gbits, t)
        # torch applies the decay to the parameter it holds; feed it the quantized iterate each step
        with torch.no_grad():
            p.copy_(torch.from_numpy(x))
        p.grad = torch.from_numpy(g.copy())
        opt.step()
        x, m, v, _, wm, _ = ref.fused_adamw_step(x, g, m, v, lr, b1, b2, eps, wd, 1 - b1**t, 1 - b2**t, wbits,
                                                 gbits, B, 0.0, seed=t, emit_codes=True)
        st = opt.state[p]
        assert np.allclose(m, st["exp_avg"].numpy(), rtol=1e-5, atol=1e-10)
        assert np.allclose(v, st["exp_avg_sq"].numpy(), rtol=1e-5, atol=1e-16)
        # the new iterate is torch's update rounded onto the bucket grid: within one cell of it
        scale = np.repeat(wm[:, 1], B)
        assert np.all(np.abs(x - p.detach().numpy()) <= scale * (1 + 1e-3) + 1e-9)
        assert np.abs(x - p.detach().numpy()).max() > 0          # and the weight quantizer did act


@pytest.mark.parametrize("flags,delta", [(0, 0.0), (1, 0.0), (4, 0.0), (0, 2.0**-10), (3, 2.0**-10)])
def test_adamw_step_is_the_composition_of_the_entry_points(flags, delta):
    B, n = 64, 64 * 5 + 9
    rng = np.random.default_rng(1)
    x = (rng.normal(size=n) * 0.02).astype(np.float32)
    g = (rng.standard_t(3, size=n) * 1e-3).astype(np.float32)
    m = (rng.normal(size=n) * 1e-3).astype(np.float32)
    v = (rng.random(size=n) * 1e-6).astype(np.float32)
    lr, b1, b2, eps, wd, bc1, bc2 = 1e-3, 0.9, 0.95, 1e-8, 0.01, 0.19, 0.0975
    gc, gm = ref.quantize_grad(g, 4, B, 3, flags=flags)
    ghat = ref.dequantize(gc, gm, n, 4, B)
    f = np.float32
    m2 = (f(b1) * m.astype(np.float64) + np.float64(f(f(1) - f(b1)) * ghat)).astype(np.float32)          # fma
    t2 = (f(f(1) - f(b2)) * ghat).astype(np.float32)
    v2 = (f(b2) * v.astype(np.float64) + np.float64((t2 * ghat).astype(np.float32))).astype(np.float32)  # fma
    upd = ((m2 / f(bc1)).astype(np.float32) / (np.sqrt((v2 / f(bc2)).astype(np.float32)).astype(np.float32) + f(eps))).astype(np.float32)
    inner = (np.float64(f(wd)) * x.astype(np.float64) + upd.astype(np.float64)).astype(np.float32)      # fma
    y = (x.astype(np.float64) - np.float64(f(lr)) * inner.astype(np.float64)).astype(np.float32)        # fma
    wc, wm, sat = ref.quantize_weight(y, 8, B, delta, 3, flags=flags)
    want = ref.dequantize(wc, wm, n, 8, B)
    xn, mn, vn, c, mm, s = ref.fused_adamw_step(x, g, m, v, lr, b1, b2, eps, wd, bc1, bc2, 8, 4, B, delta, 3,
                                                flags=flags, emit_codes=True)
    assert np.array_equal(mn, m2) and np.array_equal(vn, v2)
    assert np.array_equal(xn, want) and np.array_equal(c, wc) and np.array_equal(mm, wm) and s == sat


def test_argument_errors():
    z = np.zeros(64, np.float32)
    for kw in (dict(beta1=1.0), dict(eps=0.0), dict(bias1=0.0), dict(beta2=-0.1)):
        args = dict(lr=1e-3, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.0, bias1=0.1, bias2=0.05)
        args.update(kw)
        with pytest.raises(ValueError):
            ref.fused_adamw_step(z, z, z, z, wbits=8, gbits=4, bucket=64, delta=0.0, seed=0, **args)
