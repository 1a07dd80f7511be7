"""Oracle pins: wire format (bit packing), size helpers, decoding, bf16 rounding."""
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import ref


def _bit(words, p):
    return (int(words[p // 32]) >> (p % 32)) & 1


@pytest.mark.parametrize("bits", range(1, 9))
def test_pack_by_brute_force_bit_extraction(bits):
    B = 96
    n = 2 * B + 41                          # short last bucket
    rng = np.random.default_rng(bits)
    codes = rng.integers(0, 2**bits, size=n, dtype=np.uint8)
    words = ref.pack(codes, bits, B)
    wpb = B * bits // 32
    assert words.size == 3 * wpb
    for i in range(n):
        j, r = divmod(i, B)
        got = sum(_bit(words[j * wpb:(j + 1) * wpb], r * bits + q) << q for q in range(bits))
        assert got == codes[i]
    # slots past the end hold zeros
    tail = words[2 * wpb:]
    assert all(_bit(tail, p) == 0 for p in range(41 * bits, B * bits))
    assert np.array_equal(ref.unpack(words, n, bits, B), codes)


def test_size_helpers():
    for n, bits, bucket in [(1, 8, 1024), (1024, 8, 1024), (1025, 4, 1024), (10**6, 3, 128),
                            (1315723264, 4, 1024), (125226240, 8, 1024)]:
        nb = -(-n // bucket)
        assert ref.codes_bytes(n, bits, bucket) == nb * bucket * bits // 8
        assert ref.meta_bytes(n, bucket) == nb * 8


def test_dequantize_is_one_correctly_rounded_multiply_add():
    rng = np.random.default_rng(0)
    bits, B, n = 8, 32, 32 * 40
    codes = rng.integers(0, 256, size=n, dtype=np.uint8)
    meta = np.stack([rng.normal(size=40) * 0.02, np.abs(rng.normal(size=40)) * 1e-4], 1).astype(np.float32)
    out = ref.dequantize(ref.pack(codes, bits, B), meta, n, bits, B)
    for i in range(0, n, 7):
        base, scale = meta[i // B]
        exact = Fraction(int(codes[i])) * Fraction(float(scale)) + Fraction(float(base))
        r = out[i]
        err = abs(Fraction(float(r)) - exact)
        for nb_ in (np.nextafter(r, np.float32(np.inf)), np.nextafter(r, np.float32(-np.inf))):
            assert err <= abs(Fraction(float(nb_)) - exact)


def test_bf16_rounding_against_torch_exhaustively():
    hi = np.arange(65536, dtype=np.uint32) << 16
    for low in (0x0000, 0x0001, 0x7FFF, 0x8000, 0x8001, 0xFFFF, 0x1234, 0xC000):
        bits = hi | np.uint32(low)
        f = bits.view(np.float32)
        finite = np.isfinite(f)
        want = torch.from_numpy(f[finite].copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
        got = np.array([ref.f32_to_bf16(v) for v in f[finite]], dtype=np.uint16)
        ok = np.isfinite(want.astype(np.uint32).__lshift__(16).view(np.float32))  # skip overflow-to-inf cases alike
        assert np.array_equal(got[ok], want[ok])
        assert np.array_equal(got, want)


def test_f16_rounding_against_numpy_and_torch_on_every_half_boundary():
    """Every finite non-negative binary16 value h, the midpoint to its successor (a tie), and the float32
    neighbours of that midpoint, both signs; plus the overflow boundary, tiny values and a random sweep."""
    h = np.arange(0x7C00, dtype=np.uint16)
    lo = h.view(np.float16).astype(np.float64)
    nxt = np.append(lo[1:], 65536.0)                      # the value after 65504 would be 65536
    mid = ((lo + nxt) / 2).astype(np.float32)             # exact in float32 (12 significant bits)
    cases = np.concatenate([lo.astype(np.float32), mid, np.nextafter(mid, np.float32(0)),
                            np.nextafter(mid, np.float32(np.inf)),
                            np.float32([1e-10, 2.0 ** -25, 2.0 ** -24, 3e-8, 65519.9, 65520.0, 70000.0, 3e38])])
    rng = np.random.default_rng(5)
    cases = np.concatenate([cases, (rng.standard_normal(20000) * 10.0 ** rng.integers(-9, 6, 20000)).astype(np.float32)])
    cases = np.concatenate([cases, -cases])
    with np.errstate(over="ignore"):
        want = cases.astype(np.float16).view(np.uint16)
    got = np.array([ref.f32_to_f16(v) for v in cases], dtype=np.uint16)
    assert np.array_equal(got, want)
    want_t = torch.from_numpy(cases).to(torch.float16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(got, want_t)


def test_dequantize_f16_output():
    rng = np.random.default_rng(2)
    x = (rng.normal(size=1000) * 0.02).astype(np.float32)
    x[:4] = [6e-8, -3e-6, 1e-5, 0.0]                      # binary16 subnormals among the decoded values
    c, m, _ = ref.quantize_weight(x, 8, 128, 0.0, 3)
    f = ref.dequantize(c, m, x.size, 8, 128, ref.F32)
    h = ref.dequantize(c, m, x.size, 8, 128, ref.F16)
    assert np.array_equal(h, f.astype(np.float16).view(np.uint16))
    lv = np.sort(rng.random(16)).astype(np.float32)
    cl, ml = ref.quantize_levels(x, 4, 128, lv)
    hl = ref.dequantize_levels(cl, ml, x.size, 4, 128, lv, ref.F16)
    assert np.array_equal(hl, ref.dequantize_levels(cl, ml, x.size, 4, 128, lv).astype(np.float16).view(np.uint16))


def test_dequantize_bf16_output():
    rng = np.random.default_rng(1)
    x = (rng.normal(size=1000) * 0.02).astype(np.float32)
    c, m, _ = ref.quantize_weight(x, 8, 128, 0.0, 3)
    f = ref.dequantize(c, m, x.size, 8, 128, ref.F32)
    h = ref.dequantize(c, m, x.size, 8, 128, ref.BF16)
    want = torch.from_numpy(f).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(h, want)
