"""Pins of the oracle's unbiased rounding onto learned (non-uniform) levels: the coin-flip
quantizer between the two levels that enclose the normalised value."""
import numpy as np
import pytest

from oracle import ref


def _table(bits, seed):
    """An irregular ascending table with end levels 0 and 1 (so that every normalised value is enclosed)."""
    rng = np.random.default_rng(seed)
    K = 1 << bits
    q = np.sort(rng.random(K)).astype(np.float32)
    q[0], q[-1] = 0.0, 1.0
    return q


def test_exhaustive_over_all_uniforms_gives_the_exact_up_count():
    """For one value between two levels, the uniforms h * 2^-16 that round up are the largest ones, those
    with 2^16 - (h + 1/2) < p * 2^16: round(p * 2^16) of them, p = (z - q_i) * (1 / (q_{i+1} - q_i)) in binary32
    (brute force over every h; the comparison is evaluated here in exact rational arithmetic)."""
    from fractions import Fraction
    q = np.array([0.0, 0.125, 0.5, 1.0], dtype=np.float32)
    B = 32
    u_all = (np.arange(1 << 16, dtype=np.float32) * np.float32(2.0 ** -16))
    for z, i in ((0.2, 1), (0.124, 0), (0.51, 2), (0.999, 2), (0.125, 1)):
        zf = np.float32(z)
        p = np.float32(zf - q[i]) * (np.float32(1.0) / np.float32(q[i + 1] - q[i]))   # binary32: gap, reciprocal, product
        # every one of the 2^16 uniforms once: buckets of B elements, one uniform per element
        codes_up = 0
        for start in range(0, 1 << 16, B):
            vv = np.full(B, zf, dtype=np.float32)
            vv[0], vv[1] = 0.0, 1.0
            uu = u_all[start:start + B].copy()
            c, _ = ref.quantize_levels_u(vv, 2, B, q, uu)
            codes_up += int(np.sum(c[2:] == i + 1))
            assert set(np.unique(c[2:])) <= {i, i + 1}
        # elements 0 and 1 of every bucket are the range markers: their two uniforms are not counted
        want = sum(1 for h in range(1 << 16)
                   if (h % B) >= 2 and 65536 - (h + Fraction(1, 2)) < Fraction(float(p)) * 65536)
        assert codes_up == want, (z, codes_up, want)
        total = (1 << 16) - 2 * ((1 << 16) // B)
        assert abs(codes_up / total - float(p)) < 2e-4


@pytest.mark.parametrize("bits", [2, 3, 5])
def test_unbiased_inside_the_table_and_clamped_outside(bits):
    """Mean of the decoded value over seeds equals the value (tables with end levels 0 and 1); a table
    that does not reach 0 or 1 clamps the values outside it to its end levels."""
    q = _table(bits, bits)
    rng = np.random.default_rng(1)
    B, n = 64, 256
    v = rng.standard_normal(n).astype(np.float32)
    S = 3000
    acc = np.zeros(n)
    for seed in range(S):
        c, m = ref.quantize_levels_stochastic(v, bits, B, q, seed)
        acc += ref.dequantize_levels(c, m, n, bits, B, q)
    rng_b = np.repeat(m[:, 1], B).astype(np.float64)
    gap = np.max(np.diff(q.astype(np.float64)))
    # sd of one draw <= gap * range / 2; 5 sd of the mean
    assert np.all(np.abs(acc / S - v) <= 5 * 0.5 * gap * rng_b / np.sqrt(S) + 1e-7)
    inner = q.copy()
    inner[0], inner[-1] = 0.25, 0.75
    inner = np.sort(inner)
    c, m = ref.quantize_levels_stochastic(v, bits, B, inner, 0)
    dec = ref.dequantize_levels(c, m, n, bits, B, inner)
    z = (v.reshape(-1, B) - m[:, :1]) / m[:, 1:]
    d = (dec.reshape(-1, B) - m[:, :1]) / m[:, 1:]
    assert np.allclose(d[z < inner[0]], inner[0], atol=1e-6) and np.allclose(d[z > inner[-1]], inner[-1], atol=1e-6)


def test_value_on_a_level_is_reproduced_and_neighbours_enclose():
    q = _table(4, 9)
    B = 32
    v = np.empty(B, dtype=np.float32)
    v[:16] = q
    v[16:] = q                                           # range [0, 1] → z = v exactly
    for seed in range(20):
        c, m = ref.quantize_levels_stochastic(v, 4, B, q, seed)
        assert np.array_equal(ref.dequantize_levels(c, m, B, 4, B, q).view(np.uint32), v.view(np.uint32))
    rng = np.random.default_rng(3)
    w = rng.random(4096).astype(np.float32)
    w[0], w[1] = 0.0, 1.0
    c, m = ref.quantize_levels_stochastic(w, 4, 4096, q, 5)
    codes = ref.unpack(c, 4096, 4, 4096)
    lower = np.searchsorted(q, w, side="right") - 1      # largest i with q_i <= z
    lower = np.clip(lower, 0, 15)
    assert np.all((codes == lower) | (codes == np.minimum(lower + 1, 15)))
    assert np.any(codes == lower + 1) and np.any(codes == lower)


def test_uniform_table_behaves_like_the_coin_flip_quantizer():
    """With the table k/L the up-probability is frac(z*L) up to rounding: codes differ from those of the
    uniform gradient quantizer at the same uniforms only where the two binary32 expressions of the
    fraction straddle the uniform (rare), and never by more than one level."""
    bits, B, n = 3, 128, 4096
    rng = np.random.default_rng(4)
    g = rng.standard_normal(n).astype(np.float32)
    u = rng.random(n).astype(np.float32)
    q = ref.levels_uniform(bits)
    a, _ = ref.quantize_levels_u(g, bits, B, q, u)
    b, _ = ref.quantize_grad_u(g, bits, B, u)
    assert np.max(np.abs(a.astype(int) - b.astype(int))) <= 1
    assert np.mean(a != b) < 2e-3


def test_seeded_form_uses_the_gradient_uniform_stream_and_shards():
    q = _table(3, 2)
    rng = np.random.default_rng(6)
    v = rng.standard_normal(512).astype(np.float32)
    c, m = ref.quantize_levels_stochastic(v, 3, 128, q, 77, index_offset=256)
    u = np.array([ref.grad_uniform(77, 256 + e) for e in range(512)], dtype=np.float32)
    cu, mu = ref.quantize_levels_u(v, 3, 128, q, u)
    assert np.array_equal(ref.unpack(c, 512, 3, 128), cu) and np.array_equal(m, mu)
    c2, _ = ref.quantize_levels_stochastic(v[256:], 3, 128, q, 77, index_offset=512)
    assert np.array_equal(c2, c[c.size // 2:])
