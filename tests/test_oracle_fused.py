"""Oracle pins, the quantized iteration x <- Q^w(x - lr * Q^g(g)) (Section 3.3 / 4.1)."""
import numpy as np
import pytest

from oracle import ref


def _unfused(x, g, lr, wbits, gbits, bucket, delta, seed, off=0):
    n = x.size
    gc, gm = ref.quantize_grad(g, gbits, bucket, seed, off)
    ghat = ref.dequantize(gc, gm, n, gbits, bucket)
    # y = x - lr*ghat with a single rounding, element by element
    y = np.array([np.float32(np.float64(x[i]) - np.float64(np.float32(lr)) * np.float64(ghat[i]))
                  for i in range(n)], dtype=np.float32)
    wc, wm, sat = ref.quantize_weight(y, wbits, bucket, delta, seed)
    return ref.dequantize(wc, wm, n, wbits, bucket), wc, wm, sat


@pytest.mark.parametrize("wbits,gbits,bucket,delta", [(8, 8, 1024, 0.0), (8, 4, 128, 0.0),
                                                      (6, 3, 96, 0.0), (8, 4, 128, 2.0**-10),
                                                      (4, 2, 32, 2.0**-6)])
def test_fused_equals_composition_of_the_entry_points(wbits, gbits, bucket, delta):
    rng = np.random.default_rng(wbits * 10 + gbits)
    n = 3 * bucket + 37
    x = (rng.normal(size=n) * 0.02).astype(np.float32)
    g = (rng.standard_t(3, size=n) * 1e-3).astype(np.float32)
    for seed in (0, 3):
        want, wc, wm, sat = _unfused(x, g, 1e-3, wbits, gbits, bucket, delta, seed)
        got, gc, gm, gsat = ref.fused_step(x, g, 1e-3, wbits, gbits, bucket, delta, seed, emit_codes=True)
        assert np.array_equal(got, want)
        assert np.array_equal(gc, wc) and np.array_equal(gm, wm) and sat == gsat
        got2, _, _, _ = ref.fused_step(x, g, 1e-3, wbits, gbits, bucket, delta, seed)
        assert np.array_equal(got2, want)


def test_iteration_mean_is_the_plain_sgd_step():
    """Both quantizers are unbiased, so E[x_{t+1} | x_t, g] = x_t - lr*g. Lattice mode keeps
    the weight grid fixed, which makes Q^w exactly unbiased over the shift."""
    rng = np.random.default_rng(0)
    n, B = 64, 32
    x = (rng.normal(size=n) * 0.02).astype(np.float32)
    g = (rng.standard_t(3, size=n) * 1e-1).astype(np.float32)
    lr, delta = 1e-2, 2.0**-10
    S = 20_000
    acc = np.zeros(n)
    acc2 = np.zeros(n)
    for seed in range(S):
        out, _, _, sat = ref.fused_step(x, g, lr, 8, 4, B, delta, seed)
        assert sat == 0
        d = out.astype(np.float64) - (x.astype(np.float64) - lr * g.astype(np.float64))
        acc += d
        acc2 += d * d
    mean, var = acc / S, acc2 / S
    assert np.all(np.abs(mean) <= 4.5 * np.sqrt(var / S) + 1e-9)
    # and the error is not degenerate: the quantizers did something
    assert var.max() > 0


def test_toy_quadratic_converges_to_the_grid_neighbourhood():
    """Sanity (Theorem 1's setting, f(x) = |x-c|^2/2, alpha = beta = 1): the iterates stay on
    the grid and end within a few cells of c."""
    rng = np.random.default_rng(1)
    n, B, delta, lr = 128, 32, 2.0**-8, 0.25
    c = rng.normal(size=n).astype(np.float32) * 0.05
    x = np.zeros(n, np.float32)
    for step in range(60):
        g = (x - c).astype(np.float32)
        x, _, _, sat = ref.fused_step(x, g, lr, 8, 8, B, delta, seed=step)
        assert sat == 0
    assert np.abs(x - c).max() <= 2 * delta
    xi = ref.weight_shift(59)
    coord = x.astype(np.float64) / delta - xi
    assert np.all(np.abs(coord - np.rint(coord)) < 1e-3)


def test_fused_shard_invariance_and_errors():
    rng = np.random.default_rng(2)
    B, n = 64, 64 * 6
    x = (rng.normal(size=n) * 0.02).astype(np.float32)
    g = (rng.normal(size=n) * 1e-3).astype(np.float32)
    whole, _, _, _ = ref.fused_step(x, g, 1e-3, 8, 4, B, 0.0, 9)
    part, _, _, _ = ref.fused_step(x[2 * B:5 * B], g[2 * B:5 * B], 1e-3, 8, 4, B, 0.0, 9, index_offset=2 * B)
    assert np.array_equal(part, whole[2 * B:5 * B])
    with pytest.raises(ValueError):
        ref.fused_step(x, g, 1e-3, 8, 4, B, -1.0, 0)
    with pytest.raises(ValueError):
        ref.fused_step(x, g, 1e-3, 9, 4, B, 0.0, 0)


@pytest.mark.parametrize("wbits,gbits,bucket,delta", [(8, 4, 128, 0.0), (4, 8, 64, 0.0), (6, 3, 96, 0.0),
                                                      (8, 4, 128, 2.0**-10)])
def test_code_resident_iteration_equals_the_fp32_resident_one(wbits, gbits, bucket, delta):
    """Every iterate lies on its bucket grids (the lattice domain of Section 4.1), so codes + meta
    hold it exactly: iterating on the codes gives, step after step, the iterates of the fp32
    iteration bit for bit."""
    rng = np.random.default_rng(7)
    n = 5 * bucket + 11
    x_init = (rng.normal(size=n) * 0.02).astype(np.float32)
    codes, meta, _ = ref.quantize_weight(x_init, wbits, bucket, delta, seed=100)
    x = ref.dequantize(codes, meta, n, wbits, bucket)
    for step in range(6):
        g = (rng.standard_t(3, size=n) * 1e-3).astype(np.float32)
        x, want_c, want_m, want_sat = ref.fused_step(x, g, 1e-2, wbits, gbits, bucket, delta, step, emit_codes=True)
        codes, meta, sat = ref.fused_step_codes(codes, meta, g, 1e-2, wbits, gbits, bucket, delta, step)
        assert np.array_equal(codes, want_c) and np.array_equal(meta, want_m) and sat == want_sat
        assert np.array_equal(ref.dequantize(codes, meta, n, wbits, bucket), x)
