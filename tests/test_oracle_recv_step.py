"""Pins of the oracle's receive-side step (Algorithm 2 with P workers: decode-and-average the
peers' quantized gradients, SGD step, Q^w): closed forms and special cases that do not re-run the
routine's own composition."""
import numpy as np
import pytest

from oracle import ref


def _peers(n, P, gbits, B, seed0, rng):
    """P workers' gradients and their quantized slices (oracle's own quantize_grad, pinned elsewhere)."""
    gs = [(1e-3 * rng.standard_normal(n)).astype(np.float32) for _ in range(P)]
    cs, ms = [], []
    for p, g in enumerate(gs):
        c, m = ref.quantize_grad(g, gbits, B, seed0 + p)
        cs.append(c); ms.append(m.reshape(-1))
    return gs, np.stack(cs), np.stack(ms)


def test_one_peer_with_exact_codes_is_plain_sgd_then_round_to_grid():
    """One peer whose gradient lies exactly on its 8-bit grid (so its codes decode to it exactly),
    alpha = 1, NO_SHIFT: the result must be the textbook affine quantizer applied to x - lr*g,
    written out here in numpy."""
    B, n = 64, 256
    rng = np.random.default_rng(1)
    k = rng.integers(0, 256, size=n)
    k[::B] = 0; k[1::B] = 255                                  # every bucket spans the full range
    g = (k.astype(np.float32) * np.float32(2.0 ** -12)) - np.float32(0.03125)   # exact in fp32
    c, m = ref.quantize_grad(g, 8, B, 0)
    assert np.array_equal(ref.dequantize(c, m, n, 8, B), g)  # precondition of this pin
    x = (0.02 * rng.standard_normal(n)).astype(np.float32)
    lr = np.float32(0.5)
    got, _, _, _ = ref.recv_step(x, c[None], m.reshape(1, -1), 1, 1.0, lr, 8, 8, B, 0.0, 3, flags=ref.FLAG_NO_SHIFT)
    y = (x.astype(np.float64) - 0.5 * g.astype(np.float64)).astype(np.float32)   # lr = 1/2: fma is exact here
    want = np.empty_like(y)
    for j in range(n // B):
        yb = y[j * B:(j + 1) * B]
        lo, hi = yb.min(), yb.max()
        scale = np.float32((hi - lo) / np.float32(255))
        inv = np.float32(np.float32(255) / (hi - lo))
        kk = np.clip(np.rint((yb - lo) * inv), 0, 255).astype(np.float32)
        want[j * B:(j + 1) * B] = (kk.astype(np.float64) * scale + lo).astype(np.float32)   # one rounding = fma
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))


def test_average_of_peers_is_the_exact_mean_when_sums_are_exact():
    """Peers whose decoded gradients are small dyadic numbers: the sum in peer order and the
    scaling by 1/P (P a power of two) are exact, so ghat is the true mean and, with a coarse
    explicit grid and a fixed shift, the step lands where exact arithmetic says."""
    B, n, P = 32, 64, 4
    rng = np.random.default_rng(2)
    gs, cs, ms = [], [], []
    for p in range(P):
        k = rng.integers(0, 16, size=n); k[::B] = 0; k[1::B] = 15
        g = (k.astype(np.float32) - 8.0) * np.float32(2.0 ** -6)
        c, m = ref.quantize_grad(g, 4, B, p)
        assert np.array_equal(ref.dequantize(c, m, n, 4, B), g)
        gs.append(g); cs.append(c); ms.append(m.reshape(-1))
    mean = np.mean(np.stack(gs).astype(np.float64), axis=0)
    x = (rng.integers(-64, 64, size=n).astype(np.float32)) * np.float32(2.0 ** -7)
    delta = 2.0 ** -5
    got, wc, wm, sat = ref.recv_step(x, np.stack(cs), np.stack(ms), P, 1.0 / P, 1.0, 8, 4, B, delta, 11,
                                     emit_codes=True)
    xi = float(ref.weight_shift(11))
    y = x.astype(np.float64) - mean                       # exact in binary32 for these inputs
    want = (np.rint(y / delta - xi) + xi) * delta          # Definition 1 on the lattice delta(Z + xi)
    assert sat == 0
    assert np.allclose(got, want, rtol=0, atol=2.0 ** -24)
    assert np.all(np.abs(got.astype(np.float64) - y) <= delta / 2 + 2.0 ** -24)
    assert np.array_equal(ref.dequantize(wc, wm, n, 8, B), got)


@pytest.mark.parametrize("P,gbits,wbits,B,n", [(8, 4, 8, 128, 1000), (3, 3, 5, 96, 500), (2, 8, 4, 1024, 3000)])
def test_unbiased_over_seeds_and_error_bounded(P, gbits, wbits, B, n):
    """E over the weight shift of the new iterate equals x - lr*ghat (the random-shift quantizer
    is unbiased; Section 4.1), and every element moves by at most half a cell."""
    rng = np.random.default_rng(P)
    _, cs, ms = _peers(n, P, gbits, B, 50, rng)
    x = (0.02 * rng.standard_normal(n)).astype(np.float32)
    ghat = ref.dequantize_add(cs, ms, P, n, gbits, B, 1.0 / P)
    y = x.astype(np.float64) - 1e-2 * ghat.astype(np.float64)
    acc = np.zeros(n)
    S = 400
    for seed in range(S):
        got, wc, wm, _ = ref.recv_step(x, cs, ms, P, 1.0 / P, 1e-2, wbits, gbits, B, 0.0, seed, emit_codes=True)
        scale = np.repeat(wm[:, 1], B)[:n].astype(np.float64)
        assert np.all(np.abs(got - y) <= 0.5 * scale * (1 + 1e-5) + 1e-9)
        acc += got
    scale = np.repeat(wm[:, 1], B)[:n].astype(np.float64)
    err = acc / S - y
    # uniform error on a cell: sd = scale / sqrt(12); allow 5 sd of the mean (edge cells clamp: skip them)
    inner = (np.abs(err) <= 5 * scale / np.sqrt(12 * S) + 1e-9)
    assert inner.mean() > 0.97


def test_rejects_bad_arguments():
    x = np.zeros(64, dtype=np.float32)
    c, m = ref.quantize_grad(x, 4, 32, 0)
    with pytest.raises(Exception):
        ref.recv_step(x, c[None], m.reshape(1, -1), 1, 1.0, 1e-3, 8, 4, 32, 0.0, 0, flags=ref.FLAG_GRAD_SHIFT)
    with pytest.raises(Exception):
        ref.recv_step(x, c[None], m.reshape(1, -1), 1, 1.0, float("inf"), 8, 4, 32, 0.0, 0)
