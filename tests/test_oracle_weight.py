"""Oracle pins, weight quantizer Q^w (Definition 1, quantization by random shift).

Expectations come from the paper: Definition 1 (nearest point of delta*Z + r),
Lemma 3 (unbiasedness, variance delta^2 {x/delta}(1-{x/delta}), sparsity law
P[Q(x)-r = 0] = 1-|x/delta|), the rounding fact used in its proof (round(z+u) = 1
iff u >= 1/2 - z), Lemma 4/5 (finer grid => proportionally smaller error), and the
lattice domain delta*Z^n + r*1 (Section 4.1). The shift is enumerated on an even
grid of 2^12 values instead of sampled.
"""
import numpy as np
import pytest

from oracle import ref

XIS = (np.arange(4096) + 0.5) / 4096.0 - 0.5   # even cover of [-1/2, 1/2), no ties


def _lattice_outputs(x, delta, bits=8, bucket=32):
    """Decoded values for every shift in XIS. x must fit the b-bit window."""
    outs = np.empty((XIS.size, x.size))
    for a, xi in enumerate(XIS):
        codes, meta, sat = ref.quantize_weight_xi(x, bits, bucket, delta, xi)
        assert sat == 0
        outs[a] = ref.dequantize(ref.pack(codes, bits, bucket), meta, x.size, bits, bucket)
    return outs


def test_zero_shift_is_the_textbook_affine_quantizer():
    rng = np.random.default_rng(0)
    for bits in (2, 4, 8):
        L = 2**bits - 1
        x = (rng.normal(size=4 * 256) * 0.02).astype(np.float32)
        codes, meta, _ = ref.quantize_weight_xi(x, bits, 256, 0.0, 0.0)
        xb = x.reshape(4, 256).astype(np.float64)
        lo = xb.min(axis=1, keepdims=True)
        scale = (xb.max(axis=1, keepdims=True) - lo) / L
        t = (xb - lo) / scale
        want = np.rint(t)
        safe = np.abs(t - np.floor(t) - 0.5) > 1e-4      # away from rounding ties
        assert np.array_equal(codes.reshape(4, 256)[safe], want[safe].astype(np.uint8))
        assert np.mean(safe) > 0.99
        assert np.array_equal(meta[:, 0], x.reshape(4, 256).min(axis=1))  # base = lo when xi = 0


@pytest.mark.parametrize("delta", [2.0**-6, 2.0**-8, 0.013])
def test_lattice_membership_and_nearest_point(delta):
    rng = np.random.default_rng(1)
    x = (rng.normal(size=96) * 0.02).astype(np.float32)
    for xi in (-0.5, -0.3, 0.0, 0.25, 0.4999):
        codes, meta, sat = ref.quantize_weight_xi(x, 8, 32, delta, xi)
        out = ref.dequantize(ref.pack(codes, 8, 32), meta, x.size, 8, 32).astype(np.float64)
        assert sat == 0
        assert np.all(meta[:, 1] == np.float32(delta))
        coord = out / np.float32(delta) - np.float32(xi)          # must be an integer: out in delta*(Z+xi)
        assert np.all(np.abs(coord - np.rint(coord)) < 1e-3)
        assert np.all(np.abs(out - x) <= 0.5 * delta * (1 + 1e-4))  # nearest point of the grid


def test_bucket_grid_membership_and_nearest_point():
    rng = np.random.default_rng(2)
    x = (rng.normal(size=3 * 64) * 0.02).astype(np.float32)
    for bits in (3, 8):
        for xi in (-0.41, 0.0, 0.33):
            codes, meta, _ = ref.quantize_weight_xi(x, bits, 64, 0.0, xi)
            out = ref.dequantize(ref.pack(codes, bits, 64), meta, x.size, bits, 64)
            out = out.reshape(3, 64).astype(np.float64)
            xb = x.reshape(3, 64).astype(np.float64)
            lo = xb.min(axis=1, keepdims=True)
            scale = (xb.max(axis=1, keepdims=True) - lo) / (2**bits - 1)
            coord = (out - lo) / scale - xi                        # grid lo + scale*(Z + xi)
            assert np.all(np.abs(coord - np.rint(coord)) < 1e-3)
            # nearest grid point, except where the b-bit window [0, L] cuts the grid
            interior = (codes.reshape(3, 64) > 0) & (codes.reshape(3, 64) < 2**bits - 1)
            assert np.all(np.abs(out - xb)[interior] <= 0.5 * scale.repeat(64, 1)[interior] * (1 + 1e-4))
            assert np.all(np.abs(out - xb) <= scale * (1 + 1e-4))


def test_unbiased_and_variance_over_the_shift():
    """Lemma 3. Unbiasedness holds for Definition 1 as printed. The lemma's variance form
    delta^2 {x/delta}(1-{x/delta}) is the one of the lattice point delta*round((x-r)/delta)
    BEFORE the shift is added back (its proof drops the "+ r"); with the shift added back, as
    Definition 1 and the lattice domain require, x/delta - xi is uniform over a unit interval,
    so the error is uniform on [-delta/2, delta/2] with variance delta^2/12. Both are checked."""
    delta = 2.0**-8
    rng = np.random.default_rng(3)
    x = (rng.normal(size=32) * 0.02).astype(np.float32)
    outs = _lattice_outputs(x, delta)
    x64 = x.astype(np.float64)
    # E Q(x) = x ; a 2^12-point even cover of the shift leaves at most delta*2^-12
    assert np.all(np.abs(outs.mean(axis=0) - x64) <= delta * 2.0**-11)
    # decoded value: error uniform on [-delta/2, delta/2]
    err = outs - x64[None, :]
    assert np.all(np.abs(err) <= delta / 2 * (1 + 1e-6))
    assert np.all(np.abs((err**2).mean(axis=0) - delta**2 / 12) <= delta**2 * 2.0**-10)
    q = np.quantile(err / delta, [0.1, 0.25, 0.5, 0.75, 0.9], axis=0)
    assert np.all(np.abs(q - np.array([-0.4, -0.25, 0.0, 0.25, 0.4])[:, None]) < 2e-3)
    # lattice point before the shift back: a coin flip between the two neighbours of x/delta
    k = np.rint(outs / delta - XIS[:, None])
    z = x64 / delta
    frac = z - np.floor(z)
    assert np.all((k == np.floor(z)[None, :]) | (k == np.floor(z)[None, :] + 1))
    assert np.all(np.abs((k == np.floor(z)[None, :] + 1).mean(axis=0) - frac) <= 2.0**-11)
    emp = ((delta * k - x64[None, :])**2).mean(axis=0)
    var = delta**2 * frac * (1 - frac)
    assert np.all(np.abs(emp - var) <= delta**2 * 2.0**-10)
    assert abs(emp.sum() - var.sum()) <= 1e-3 * var.sum()


def test_round_up_iff_shift_small_enough():
    # for z in [0,1): round(z - xi) = 1 iff -xi >= 1/2 - z, which has probability z
    delta = 2.0**-4
    z = np.array([0.0, 0.125, 0.3, 0.5, 0.77, 0.999], dtype=np.float64)
    x = (z * delta + 3 * delta).astype(np.float32)        # cells [3,4): plus an anchor below
    x = np.concatenate([[np.float32(0.0)], x, np.zeros(32 - 1 - z.size, np.float32)])
    outs = _lattice_outputs(x, delta)[:, 1:1 + z.size]
    k = np.rint(outs / delta - XIS[:, None])
    up = (k == 4)
    assert np.all((k == 3) | (k == 4))
    want = (-XIS[:, None] >= 0.5 - (np.float32(z * delta + 3 * delta).astype(np.float64) / delta - 3))
    assert np.array_equal(up, want)
    assert np.all(np.abs(up.mean(axis=0) - z) < 2e-3)


def test_sparsity_law():
    delta = 2.0**-6
    x = np.array([0.0, 0.1, -0.25, 0.5, -0.9, 0.99, 1.0, -1.0, 1.7, -2.4], dtype=np.float64) * delta
    xs = np.concatenate([x, np.full(22, -3 * delta)]).astype(np.float32)
    outs = _lattice_outputs(xs, delta)[:, :x.size]
    k = np.rint(outs / delta - XIS[:, None])               # lattice coordinate before the shift back
    p_zero = (k == 0).mean(axis=0)
    want = np.where(np.abs(x / delta) < 1, 1 - np.abs(x / delta), 0.0)
    assert np.all(np.abs(p_zero - want) < 2e-3)
    # expected number of non-zeros is at most ||v||_1 / delta
    assert (1 - p_zero).sum() <= np.abs(x).sum() / delta + 1e-9


@pytest.mark.parametrize("ratio", [2, 4, 16])
def test_finer_grid_has_proportionally_smaller_error(ratio):
    """Lemma 4/5: for delta_star/delta an integer, E||Q_delta(x)-x||^2 <= (delta/delta_star) E||Q_delta_star(x)-x||^2."""
    delta_star = 2.0**-5
    delta = delta_star / ratio
    rng = np.random.default_rng(4)
    x = (rng.normal(size=32) * 0.02).astype(np.float32)
    fine = ((_lattice_outputs(x, delta) - x[None, :].astype(np.float64))**2).mean(axis=0)
    coarse = ((_lattice_outputs(x, delta_star) - x[None, :].astype(np.float64))**2).mean(axis=0)
    assert np.all(fine <= coarse / ratio * (1 + 5e-3) + 1e-12)
    assert fine.sum() <= coarse.sum() / ratio * (1 + 1e-3)


def test_idempotent_for_the_same_shift():
    delta = 2.0**-9
    x = (np.random.default_rng(5).normal(size=512) * 0.02).astype(np.float32)
    for seed in range(5):
        c1, m1, _ = ref.quantize_weight(x, 8, 128, delta, seed)
        y = ref.dequantize(c1, m1, x.size, 8, 128)
        c2, m2, _ = ref.quantize_weight(y, 8, 128, delta, seed)
        assert np.array_equal(ref.dequantize(c2, m2, x.size, 8, 128), y)


def test_saturation_is_counted_and_clamped():
    delta, bits = 2.0**-8, 4
    L = 2**bits - 1
    x = (np.random.default_rng(6).normal(size=256) * 0.02).astype(np.float32)
    xi = 0.2
    codes, meta, sat = ref.quantize_weight_xi(x, bits, 128, delta, xi)
    xb = x.reshape(2, 128).astype(np.float64)
    k = np.rint(xb / delta - xi)
    rel = k - k.min(axis=1, keepdims=True)
    assert sat == int((rel > L).sum()) and sat > 0
    assert np.array_equal(codes.reshape(2, 128), np.minimum(rel, L).astype(np.uint8))
    base = (k.min(axis=1) + xi) * delta
    assert np.allclose(meta[:, 0], base, rtol=1e-6, atol=0)


def test_constant_bucket_and_tail():
    x = np.concatenate([np.full(32, -0.07, np.float32), np.array([0.5, 0.25], np.float32)])
    for xi in (-0.5, 0.1, 0.49):
        codes, meta, _ = ref.quantize_weight_xi(x, 8, 32, 0.0, xi)
        out = ref.dequantize(ref.pack(codes, 8, 32), meta, x.size, 8, 32)
        assert np.array_equal(out[:32], x[:32])             # constant bucket: exact
        assert meta[0, 1] == 0
        assert abs(out[32] - 0.5) <= meta[1, 1] and abs(out[33] - 0.25) <= meta[1, 1]


def test_seeded_entry_point_uses_the_stream_shift():
    x = (np.random.default_rng(7).normal(size=300) * 0.02).astype(np.float32)
    for seed in (0, 4, 99):
        for delta in (0.0, 2.0**-8):
            c1, m1, s1 = ref.quantize_weight(x, 6, 64, delta, seed)
            c2, m2, s2 = ref.quantize_weight_xi(x, 6, 64, delta, ref.weight_shift(seed))
            assert np.array_equal(c1, ref.pack(c2, 6, 64)) and np.array_equal(m1, m2) and s1 == s2


def test_argument_errors():
    x = np.zeros(64, np.float32)
    for delta in (-1.0, float("nan"), float("inf")):
        with pytest.raises(ValueError):
            ref.quantize_weight(x, 8, 32, delta, 0)
