"""Pins of the KEEP_MASTER flag of the oracle's step routines (Algorithm 2: WeightUpdate acts on
the full-precision partition, QuantizeWeights only produces what is transmitted)."""
import numpy as np
import pytest

from oracle import ref

KEEP = ref.FLAG_KEEP_MASTER


def _inputs(n, seed):
    rng = np.random.default_rng(seed)
    x = (0.02 * rng.standard_normal(n)).astype(np.float32)
    g = (1e-3 * rng.standard_t(3, n)).astype(np.float32)
    return x, g


@pytest.mark.parametrize("B,n,wbits,gbits,delta", [(128, 1000, 8, 4, 0.0), (96, 500, 5, 3, 0.0), (1024, 3000, 4, 8, 2.0 ** -8)])
def test_fused_step_leaves_the_exact_sgd_update_in_x(B, n, wbits, gbits, delta):
    """x_new is x - lr*ghat itself (lr a power of two, so one binary64 expression gives the fma),
    the emitted codes are Q^w of that value and decode to within half a cell of it."""
    x, g = _inputs(n, B)
    lr = 2.0 ** -3
    gc, gm = ref.quantize_grad(g, gbits, B, 7)
    ghat = ref.dequantize(gc, gm, n, gbits, B)
    want = (x.astype(np.float64) - lr * ghat.astype(np.float64)).astype(np.float32)
    got, wc, wm, sat = ref.fused_step(x, g, lr, wbits, gbits, B, delta, 7, emit_codes=True, flags=KEEP)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    # the same call without the flag gives the same codes and the decoded iterate
    got_q, wc_q, wm_q, sat_q = ref.fused_step(x, g, lr, wbits, gbits, B, delta, 7, emit_codes=True)
    assert np.array_equal(wc, wc_q) and np.array_equal(wm.view(np.uint32), wm_q.view(np.uint32)) and sat == sat_q
    dec = ref.dequantize(wc, wm, n, wbits, B)
    assert np.array_equal(dec.view(np.uint32), got_q.view(np.uint32))
    if sat == 0:
        cell = np.repeat(wm[:, 1], B)[:n].astype(np.float64)
        assert np.all(np.abs(dec.astype(np.float64) - want) <= 0.5 * cell * (1 + 1e-5) + 1e-12)
    assert not np.array_equal(got, got_q)        # the flag does change x


def test_recv_step_leaves_the_exact_update_in_x():
    n, B, P = 700, 128, 4
    x, _ = _inputs(n, 1)
    cs, ms = [], []
    for p in range(P):
        _, g = _inputs(n, 10 + p)
        c, m = ref.quantize_grad(g, 4, B, p)
        cs.append(c); ms.append(m.reshape(-1))
    cs, ms = np.stack(cs), np.stack(ms)
    ghat = ref.dequantize_add(cs, ms, P, n, 4, B, 1.0 / P)
    want = (x.astype(np.float64) - 0.25 * ghat.astype(np.float64)).astype(np.float32)
    got, wc, wm, _ = ref.recv_step(x, cs, ms, P, 1.0 / P, 0.25, 8, 4, B, 0.0, 3, flags=KEEP, emit_codes=True)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    c2, m2, _ = ref.quantize_weight(want, 8, B, 0.0, 3)
    assert np.array_equal(wc, c2) and np.array_equal(wm.view(np.uint32), m2.view(np.uint32))


def test_adamw_step_matches_torch_adamw_exactly_in_structure():
    """With KEEP_MASTER the weights follow torch's AdamW on the decoded gradients (no weight
    quantization in the loop); the emitted codes are Q^w of those weights."""
    import torch
    n, B = 600, 96
    x, g = _inputs(n, 5)
    b1, b2, eps, wd, lr = 0.9, 0.95, 1e-8, 0.1, 2e-3
    xt = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.AdamW([xt], lr=lr, betas=(b1, b2), eps=eps, weight_decay=wd)
    xo, m, v = x.copy(), np.zeros(n, np.float32), np.zeros(n, np.float32)
    for t in range(1, 6):
        gc, gm = ref.quantize_grad(g, 4, B, t)
        ghat = ref.dequantize(gc, gm, n, 4, B)
        xt.grad = torch.tensor(ghat, dtype=torch.float64)
        opt.step()
        xo, m, v, wc, wm, _ = ref.fused_adamw_step(xo, g, m, v, lr, b1, b2, eps, wd, 1 - b1 ** t, 1 - b2 ** t,
                                                   8, 4, B, 0.0, t, flags=KEEP, emit_codes=True)
        c2, m2, _ = ref.quantize_weight(xo, 8, B, 0.0, t)
        assert np.array_equal(wc, c2) and np.array_equal(wm.view(np.uint32), m2.view(np.uint32))
    assert np.allclose(xo, xt.detach().numpy(), rtol=2e-5, atol=1e-8)


def test_flag_is_rejected_where_there_is_no_partition():
    x, g = _inputs(256, 2)
    c, m, _ = ref.quantize_weight(x, 8, 128, 0.0, 0)
    with pytest.raises(Exception):
        ref.fused_step_codes(c, m, g, 1e-3, 8, 4, 128, 0.0, 0, flags=KEEP)
    with pytest.raises(Exception):
        ref.quantize_weight(x, 8, 128, 0.0, 0, flags=KEEP)
    with pytest.raises(Exception):
        ref.quantize_grad(g, 4, 128, 0, flags=KEEP)
