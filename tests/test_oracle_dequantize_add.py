"""Oracle pins, decode-and-sum of the peers' quantized gradient slices (the receive side of the
quantized gradient exchange in Algorithm 2)."""
import numpy as np
import pytest

from oracle import ref


def _slices(g, P, bits, B, seed0=0):
    cs, ms = [], []
    for p in range(P):
        c, m = ref.quantize_grad(g[p], bits, B, seed0 + p)
        cs.append(c)
        ms.append(m)
    return np.stack(cs), np.stack(ms)


@pytest.mark.parametrize("P,bits,B", [(1, 8, 64), (2, 4, 128), (8, 3, 96), (5, 8, 1024)])
def test_equals_sequential_float32_sum_of_the_decoded_slices(P, bits, B):
    n = 3 * B + 17
    rng = np.random.default_rng(P)
    g = (rng.standard_t(3, size=(P, n)) * 1e-3).astype(np.float32)
    codes, meta = _slices(g, P, bits, B)
    alpha = np.float32(1.0 / P)
    got = ref.dequantize_add(codes, meta, P, n, bits, B, alpha)
    acc = ref.dequantize(codes[0], meta[0], n, bits, B)
    for p in range(1, P):
        acc = (acc + ref.dequantize(codes[p], meta[p], n, bits, B)).astype(np.float32)  # one rounding each
    assert np.array_equal(got, (alpha * acc).astype(np.float32))
    if P == 1:
        assert np.array_equal(ref.dequantize_add(codes, meta, 1, n, bits, B, 1.0), ref.dequantize(codes[0], meta[0], n, bits, B))


def test_peer_order_matters_only_through_rounding_and_alpha_scales():
    P, bits, B, n = 4, 4, 64, 256
    g = (np.random.default_rng(0).normal(size=(P, n)) * 1e-3).astype(np.float32)
    codes, meta = _slices(g, P, bits, B)
    a = ref.dequantize_add(codes, meta, P, n, bits, B, 1.0)
    b = ref.dequantize_add(codes[::-1], meta[::-1], P, n, bits, B, 1.0)
    assert np.allclose(a, b, rtol=1e-6, atol=1e-9)
    c = ref.dequantize_add(codes, meta, P, n, bits, B, 0.25)
    assert np.array_equal(c, (np.float32(0.25) * a).astype(np.float32))


def test_averaging_independent_unbiased_quantizations_shrinks_the_error():
    """Q^g is unbiased with independent roundings, so the mean of P quantizations of the same
    gradient keeps the mean and has 1/P of the variance."""
    bits, B, n = 2, 32, 32 * 2000
    g1 = (np.random.default_rng(1).normal(size=n) * 1e-3).astype(np.float32)
    err = {}
    for P in (1, 4, 16):
        codes, meta = _slices(np.tile(g1, (P, 1)), P, bits, B, seed0=100)
        avg = ref.dequantize_add(codes, meta, P, n, bits, B, 1.0 / P).astype(np.float64)
        err[P] = ((avg - g1) ** 2).mean()
        assert abs((avg - g1).mean()) < 5 * np.sqrt(err[P] / n)
    assert 3.3 < err[1] / err[4] < 4.8 and 13 < err[1] / err[16] < 19.5


def test_argument_errors():
    codes = np.zeros((2, 16), np.uint32)
    meta = np.zeros((2, 2), np.float32)
    with pytest.raises(ValueError):
        ref.dequantize_add(codes, meta, 0, 64, 8, 64, 1.0)
    with pytest.raises(ValueError):
        ref.dequantize_add(codes, meta, 2, 64, 8, 64, float("nan"))
