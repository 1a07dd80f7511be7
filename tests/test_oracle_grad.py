"""Oracle pins, gradient quantizer Q^g (coin-flip definition in bucket coordinates).

The expectations below come from the paper's statements, not from the oracle:
  * P(round up) = fractional position (coin-flip definition): exhaustive enumeration
    of all 2^16 values of the uniform; the fraction is rounded to 16 bits to nearest, so
    the rounding adds no bias of a preferred sign;
  * unbiasedness and the variance delta^2 {x/delta}(1-{x/delta}) (coin-flip lemma);
  * codes in [0, 2^b-1]; values already on the grid are reproduced exactly.
"""
import numpy as np
import pytest

from oracle import ref


def _dyadic_bucket(bits, B=32):
    """A bucket whose min-max grid has spacing 2^-6 and whose entries sit at exact
    multiples of 1/64 of a cell, so that every binary32 step of the quantizer is exact."""
    L = 2**bits - 1
    s = 2.0**-6
    rng = np.random.default_rng(bits)
    t = rng.integers(0, 64 * L + 1, size=B) / 64.0  # positions in [0, L], multiples of 1/64
    t[0], t[1] = 0.0, float(L)                       # pins min and max
    lo = -0.75
    return (lo + s * t).astype(np.float32), t, lo, s


@pytest.mark.parametrize("bits", [1, 2])
def test_coin_flip_probabilities_exhaustive(bits):
    B = 32
    g, t, lo, s = _dyadic_bucket(bits, B)
    H = 65536
    G = np.tile(g, H)
    U = np.repeat(np.arange(H, dtype=np.float32) / 65536.0, B)
    codes, meta = ref.quantize_grad_u(G, bits, B, U)
    codes = codes.reshape(H, B).astype(np.int64)
    assert np.all(meta[:, 0] == np.float32(lo)) and np.all(meta[:, 1] == np.float32(s))
    fl = np.floor(t)
    frac = t - fl
    ups = (codes - fl[None, :].astype(np.int64))
    assert ups.min() >= 0 and ups.max() <= 1
    # the number of 16-bit uniforms that round up is exactly frac*65536 for these dyadic fractions
    assert np.array_equal(ups.sum(axis=0), (frac * 65536).astype(np.int64))
    # and "up" happens exactly for the largest uniforms: floor((ti + h) / 2^16), ti = t * 2^16
    for i in range(B):
        k = int(frac[i] * 65536)
        assert ups[H - k:, i].all() and not ups[:H - k, i].any()


def test_fraction_is_rounded_to_16_bits_to_nearest_not_downward():
    """One-bit grid on [0, 1] (so t = g exactly): g = k * 2^-18 has the fraction k/4 units of 2^-16.
    Rounded to nearest (halves up) that is floor(k/4 + 1/2) uniforms out of 2^16 that round up;
    truncation would give floor(k/4) and a quantizer whose mean always falls short of g."""
    B, H = 32, 65536
    ks = np.array([1, 2, 3, 5, 6, 7, 9, 4 * 65536 - 3, 4 * 65536 - 2, 4 * 65536 - 1])
    g = np.zeros(B, np.float32)
    g[1] = 1.0
    g[2:2 + ks.size] = (ks * 2.0 ** -18).astype(np.float32)
    codes, meta = ref.quantize_grad_u(np.tile(g, H), 1, B, np.repeat(np.arange(H, dtype=np.float32) / 65536.0, B))
    assert np.all(meta[:, 0] == 0.0) and np.all(meta[:, 1] == 1.0)
    ups = codes.reshape(H, B)[:, 2:2 + ks.size].astype(np.int64).sum(axis=0)
    assert np.array_equal(ups, (ks + 2) // 4)
    # the mean over all uniforms is within half a unit of 2^-16 of g, on either side
    err = ups / 65536.0 - ks * 2.0 ** -18
    assert np.all(np.abs(err) <= 2.0 ** -17) and (err > 0).any() and (err < 0).any()


@pytest.mark.parametrize("bits", [1, 2])
def test_coin_flip_probabilities_generic_values(bits):
    B, H = 32, 65536
    L = 2**bits - 1
    g = (np.random.default_rng(5).standard_t(3, size=B) * 1e-3).astype(np.float32)
    codes, meta = ref.quantize_grad_u(np.tile(g, H), bits, B,
                                      np.repeat(np.arange(H, dtype=np.float32) / 65536.0, B))
    codes = codes.reshape(H, B).astype(np.int64)
    g64 = g.astype(np.float64)
    t = (g64 - g64.min()) / (g64.max() - g64.min()) * L
    fl = np.minimum(np.floor(t), L)
    frac = t - fl
    ups = codes - fl[None, :].astype(np.int64)
    near_integer = np.minimum(frac, 1 - frac) < 1e-5
    ok = ~near_integer
    assert ups[:, ok].min() >= 0 and ups[:, ok].max() <= 1
    want = np.floor(frac * 65536 + 0.5)
    assert np.all(np.abs(ups.sum(axis=0) - want)[ok] <= 1)
    assert codes.min() >= 0 and codes.max() <= L


@pytest.mark.parametrize("bits,bucket", [(8, 64), (4, 32), (3, 96), (2, 32)])
def test_unbiased_and_variance_monte_carlo(bits, bucket):
    """Many copies of one bucket in a long vector: every copy draws fresh uniforms from
    the counter-based stream, so the copies are independent trials."""
    L = 2**bits - 1
    T = 60_000
    rng = np.random.default_rng(100 + bits)
    g = (rng.standard_t(3, size=bucket) * 1e-3).astype(np.float32)
    G = np.tile(g, T)
    for seed in (0, 77):
        codes, meta = ref.quantize_grad(G, bits, bucket, seed)
        ghat = ref.dequantize(codes, meta, G.size, bits, bucket).reshape(T, bucket).astype(np.float64)
        g64 = g.astype(np.float64)
        scale = (g64.max() - g64.min()) / L
        t = (g64 - g64.min()) / scale
        frac = t - np.floor(t)
        var = scale**2 * frac * (1 - frac)           # closed form of the lemma
        err = ghat - g64[None, :]
        assert np.all(np.abs(err) <= scale * (1 + 1e-5))
        mean_err = err.mean(axis=0)
        # the uniforms have 16 bits: the bias is at most scale*2^-16 (plus fp32 rounding of t)
        tol = 4.5 * np.sqrt(var / T) + scale * 2.0**-15
        assert np.all(np.abs(mean_err) <= tol)
        emp_var = (err**2).mean(axis=0)
        # variance of the empirical second moment: <= scale^2 * var / T
        assert np.all(np.abs(emp_var - var) <= 5 * scale * np.sqrt(var / T) + scale**2 * 1e-4)
        # whole-vector form: E||Q(v)-v||^2 = sum of the above
        assert abs(emp_var.sum() - var.sum()) <= 0.02 * var.sum()


def test_codes_range_min_max_and_meta():
    rng = np.random.default_rng(1)
    for bits in range(1, 9):
        L = 2**bits - 1
        g = (rng.normal(size=5 * 128) * 1e-3).astype(np.float32)
        u = rng.random(g.size).astype(np.float32)
        codes, meta = ref.quantize_grad_u(g, bits, 128, u)
        assert codes.max() <= L
        gb = g.reshape(5, 128)
        assert np.array_equal(meta[:, 0], gb.min(axis=1))
        want_scale = ((gb.max(axis=1) - gb.min(axis=1)) / np.float32(L)).astype(np.float32)
        assert np.array_equal(meta[:, 1], want_scale)
        cb = codes.reshape(5, 128)
        rows = np.arange(5)
        assert np.all(cb[rows, gb.argmin(axis=1)] == 0)          # the minimum never rounds up
        assert np.all(cb[rows, gb.argmax(axis=1)] >= L - 1)      # the maximum sits at the top cell


def test_on_grid_values_are_reproduced_whatever_the_seed():
    bits, B = 4, 64
    L = 2**bits - 1
    rng = np.random.default_rng(2)
    k = rng.integers(0, L + 1, size=B)
    k[3], k[9] = 0, L
    g = (0.125 + 2.0**-9 * k).astype(np.float32)     # power-of-two spacing: exact in binary32
    for seed in range(20):
        codes, meta = ref.quantize_grad(g, bits, B, seed)
        out = ref.dequantize(codes, meta, B, bits, B)
        assert np.array_equal(out, g)
        assert np.array_equal(ref.unpack(codes, B, bits, B), k.astype(np.uint8))


def test_constant_bucket_short_tail_and_zero_signs():
    B = 32
    g = np.concatenate([np.full(B, 0.3, np.float32), np.array([-0.0, 0.0, -0.0], np.float32)])
    u = np.full(g.size, 0.999, np.float32)
    codes, meta = ref.quantize_grad_u(g, 8, B, u)
    assert not codes.any()
    assert meta[0, 0] == np.float32(0.3) and meta[0, 1] == 0
    # all-zero bucket of mixed signs: base is +0 bit-for-bit
    assert meta[1].view(np.uint32).tolist() == [0, 0]
    # tail bucket of 3 elements has its own min/max
    g2 = np.concatenate([np.linspace(-1, 1, B, dtype=np.float32), np.array([5, 6, 7], np.float32)])
    codes, meta = ref.quantize_grad_u(g2, 2, B, np.zeros(g2.size, np.float32))
    assert meta[1, 0] == 5 and meta[1, 1] == np.float32(2) / np.float32(3)
    assert codes[B:].tolist() == [0, 1, 3]  # t = 0, 1.5, 3; h = 0: floor(1.5 + 0) = 1
    codes, _ = ref.quantize_grad_u(g2, 2, B, np.full(g2.size, 0.5, np.float32))
    assert codes[B:].tolist() == [0, 2, 3]  # h = 2^15: floor(1.5 + 0.5) = 2; below that 1.5 rounds down
    codes, _ = ref.quantize_grad_u(g2, 2, B, np.full(g2.size, 0.5 - 2.0 ** -16, np.float32))
    assert codes[B:].tolist() == [0, 1, 3]


def test_shard_invariance():
    """Quantizing a bucket-aligned slice with index_offset gives the bytes of the whole."""
    bits, B = 4, 128
    g = (np.random.default_rng(3).normal(size=10 * B + 17) * 1e-3).astype(np.float32)
    codes, meta = ref.quantize_grad(g, bits, B, seed=5)
    wpb = B * bits // 32
    for lo_b, hi_b in [(0, 3), (3, 10), (7, 11)]:
        sl = g[lo_b * B: hi_b * B]
        c2, m2 = ref.quantize_grad(sl, bits, B, seed=5, index_offset=lo_b * B)
        assert np.array_equal(c2, codes[lo_b * wpb: lo_b * wpb + c2.size])
        assert np.array_equal(m2, meta[lo_b: lo_b + m2.shape[0]])
    # a different offset gives different roundings
    c3, _ = ref.quantize_grad(g[:3 * B], bits, B, seed=5, index_offset=8)
    assert not np.array_equal(c3, codes[:3 * wpb])


def test_argument_errors():
    g = np.zeros(64, np.float32)
    for bits, bucket in [(0, 32), (9, 32), (8, 100), (8, 16), (8, 16384)]:
        with pytest.raises(ValueError):
            ref.quantize_grad(g, bits, bucket, 0)
    with pytest.raises(ValueError):
        ref.quantize_grad(g, 8, 32, 0, index_offset=4)
