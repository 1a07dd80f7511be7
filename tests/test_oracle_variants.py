"""Oracle pins, quantizer variants the paper names as admissible: the random-shift operator used
on gradients (appendix: it satisfies the definition of an unbiased gradient quantizer),
deterministic rounding (shift 0), and the symmetric max-abs grid (the scaling of Section 3.2)."""
import numpy as np
import pytest

from oracle import ref
from oracle.ref import FLAG_GRAD_SHIFT, FLAG_NO_SHIFT, FLAG_SYMMETRIC

XIS = (np.arange(2048) + 0.5) / 2048.0 - 0.5


def _g(n, seed):
    return (np.random.default_rng(seed).standard_t(3, size=n) * 1e-3).astype(np.float32)


def test_grad_shift_stream(aten_philox):
    for seed in (0, 5, 2**50 + 1):
        w = aten_philox(seed, 2, 0)                       # stream 2, counter 0
        assert ref.grad_shift(seed) == (int(w[0]) >> 8) / 2.0**24 - 0.5
        assert ref.grad_shift(seed) != ref.weight_shift(seed)
    xs = np.array([ref.grad_shift(s) for s in range(20000)])
    assert abs(xs.mean()) < 4 * np.sqrt(1 / 12 / xs.size) and abs(xs.var() - 1 / 12) < 3e-3


def test_shared_shift_gradient_quantizer_is_the_random_shift_operator():
    g = _g(5 * 64 + 9, 1)
    for seed in (0, 3):
        for bits in (2, 4, 8):
            c, m = ref.quantize_grad(g, bits, 64, seed, flags=FLAG_GRAD_SHIFT)
            c2, m2, _ = ref.quantize_weight_xi(g, bits, 64, 0.0, ref.grad_shift(seed))
            assert np.array_equal(c, ref.pack(c2, bits, 64)) and np.array_equal(m, m2)
    # no per-element randomness: the index offset does not matter
    a, _ = ref.quantize_grad(g, 4, 64, 7, index_offset=0, flags=FLAG_GRAD_SHIFT)
    b, _ = ref.quantize_grad(g, 4, 64, 7, index_offset=8000, flags=FLAG_GRAD_SHIFT)
    assert np.array_equal(a, b)


def test_shared_shift_gradient_quantizer_is_unbiased_over_the_shift():
    bits, B = 3, 32
    g = _g(B, 2)
    outs = np.empty((XIS.size, B))
    for a, xi in enumerate(XIS):
        c, m, _ = ref.quantize_weight_xi(g, bits, B, 0.0, xi)
        outs[a] = ref.dequantize(ref.pack(c, bits, B), m, B, bits, B)
    scale = (g.max().astype(np.float64) - g.min()) / (2**bits - 1)
    assert np.all(np.abs(outs.mean(axis=0) - g) <= scale * 2.0**-10)
    assert np.all(np.abs(outs - g[None, :]) <= 0.5 * scale * (1 + 1e-4))


def test_no_shift_is_deterministic_round_to_nearest():
    x = (np.random.default_rng(3).normal(size=300) * 0.02).astype(np.float32)
    for flags in (FLAG_NO_SHIFT, FLAG_NO_SHIFT | FLAG_SYMMETRIC):
        want_c, want_m, _ = ref.quantize_weight_xi(x, 4, 64, 0.0, 0.0, flags=flags & FLAG_SYMMETRIC)
        for seed in (0, 1, 99):
            c, m, _ = ref.quantize_weight(x, 4, 64, 0.0, seed, flags=flags)
            assert np.array_equal(c, ref.pack(want_c, 4, 64)) and np.array_equal(m, want_m)
    g = _g(300, 4)
    a, am = ref.quantize_grad(g, 4, 64, 0, flags=FLAG_GRAD_SHIFT | FLAG_NO_SHIFT)
    b, bm = ref.quantize_grad(g, 4, 64, 5, flags=FLAG_GRAD_SHIFT | FLAG_NO_SHIFT)
    assert np.array_equal(a, b) and np.array_equal(am, bm)
    xb = g[:256].reshape(4, 64).astype(np.float64)
    t = (xb - xb.min(1, keepdims=True)) / ((xb.max(1, keepdims=True) - xb.min(1, keepdims=True)) / 15)
    codes = ref.unpack(a, 300, 4, 64)[:256].reshape(4, 64)
    safe = np.abs(t - np.floor(t) - 0.5) > 1e-4
    assert np.array_equal(codes[safe], np.rint(t)[safe].astype(np.uint8))


@pytest.mark.parametrize("bits", [2, 4, 8])
def test_symmetric_grid_closed_form_and_mirror(bits):
    L = 2**bits - 1
    B = 64
    x = (np.random.default_rng(5).normal(size=3 * B) * 0.02).astype(np.float32)
    x[7] = 0.11                                            # make max |x| positive in bucket 0
    c, m, _ = ref.quantize_weight_xi(x, bits, B, 0.0, 0.0, flags=FLAG_SYMMETRIC)
    a = np.abs(x.reshape(3, B)).max(axis=1)
    assert np.array_equal(m[:, 0], -a)                                        # base = -max|x|
    assert np.array_equal(m[:, 1], ((a + a) / np.float32(L)).astype(np.float32))  # scale = 2a/L
    out = ref.dequantize(ref.pack(c, bits, B), m, x.size, bits, B).reshape(3, B)
    assert np.all(np.abs(out - x.reshape(3, B)) <= 0.5 * m[:, 1:2].astype(np.float64) * (1 + 1e-5))
    # mirror symmetry: quantizing -x reflects the codes (away from rounding ties)
    cm, mm, _ = ref.quantize_weight_xi(-x, bits, B, 0.0, 0.0, flags=FLAG_SYMMETRIC)
    t = (x.reshape(3, B).astype(np.float64) + a[:, None]) / (2 * a[:, None].astype(np.float64) / L)
    safe = (np.abs(t - np.floor(t) - 0.5) > 1e-4).reshape(-1)
    assert np.array_equal(cm[safe], (L - c.astype(np.int64))[safe].astype(np.uint8))
    assert np.array_equal(mm, m)
    # an explicit delta ignores the flag
    c1, m1, s1 = ref.quantize_weight_xi(x, 8, B, 2.0**-9, 0.2, flags=FLAG_SYMMETRIC)
    c2, m2, s2 = ref.quantize_weight_xi(x, 8, B, 2.0**-9, 0.2)
    assert np.array_equal(c1, c2) and np.array_equal(m1, m2) and s1 == s2


def test_symmetric_coin_flip_is_unbiased():
    bits, B, T = 3, 32, 40000
    g = _g(B, 6)
    codes, meta = ref.quantize_grad(np.tile(g, T), bits, B, 11, flags=FLAG_SYMMETRIC)
    out = ref.dequantize(codes, meta, B * T, bits, B).reshape(T, B).astype(np.float64)
    a = np.abs(g).max().astype(np.float64)
    scale = 2 * a / (2**bits - 1)
    t = (g.astype(np.float64) + a) / scale
    frac = t - np.floor(t)
    var = scale**2 * frac * (1 - frac)
    assert np.all(np.abs(out.mean(axis=0) - g) <= 4.5 * np.sqrt(var / T) + scale * 2.0**-15)
    assert np.all(meta[:, 0] == np.float32(-a))


@pytest.mark.parametrize("flags", [FLAG_GRAD_SHIFT, FLAG_NO_SHIFT, FLAG_SYMMETRIC,
                                   FLAG_GRAD_SHIFT | FLAG_SYMMETRIC, FLAG_GRAD_SHIFT | FLAG_NO_SHIFT | FLAG_SYMMETRIC])
def test_fused_variants_equal_the_composition(flags):
    B, n = 64, 5 * 64 + 13
    x = (np.random.default_rng(8).normal(size=n) * 0.02).astype(np.float32)
    g = _g(n, 9)
    for delta in (0.0, 2.0**-9):
        gc, gm = ref.quantize_grad(g, 4, B, 3, flags=flags)
        ghat = ref.dequantize(gc, gm, n, 4, B)
        y = (x.astype(np.float64) - np.float64(np.float32(1e-2)) * ghat.astype(np.float64)).astype(np.float32)
        wc, wm, sat = ref.quantize_weight(y, 8, B, delta, 3, flags=flags)
        want = ref.dequantize(wc, wm, n, 8, B)
        got, c, m, s = ref.fused_step(x, g, 1e-2, 8, 4, B, delta, 3, emit_codes=True, flags=flags)
        assert np.array_equal(got, want) and np.array_equal(c, wc) and np.array_equal(m, wm) and s == sat


def test_unknown_flag_is_rejected():
    with pytest.raises(ValueError):
        ref.quantize_grad(np.zeros(64, np.float32), 4, 64, 0, flags=8)
