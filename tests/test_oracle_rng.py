"""Oracle pins, random numbers: Philox4x32-10 against a third-party implementation,
and the two streams (gradient uniforms, weight shift) against their definition."""
import numpy as np
import pytest

from oracle import ref


def test_philox_matches_third_party(aten_philox):
    rng = np.random.default_rng(7)
    cases = [(0, 0, 0), (1, 0, 0), (0, 1, 0), (0, 0, 1), (2**64 - 1, 2**64 - 1, 2**64 - 1),
             (0xDEADBEEFCAFEF00D, 5, 2**32 - 1), (3, 2**32, 2**32)]
    cases += [tuple(int(v) for v in rng.integers(0, 2**64, size=3, dtype=np.uint64))
              for _ in range(200)]
    for seed, sub, off in cases:
        want = aten_philox(seed, sub, off)
        got = ref.philox4x32_10(
            [off & 0xFFFFFFFF, off >> 32, sub & 0xFFFFFFFF, sub >> 32],
            [seed & 0xFFFFFFFF, seed >> 32])
        assert np.array_equal(got, want), (seed, sub, off)


def test_philox_is_a_bijection_on_small_counter_range():
    # a block cipher with a fixed key never maps two counters to one output
    outs = {tuple(ref.philox4x32_10([c, 0, 0, 0], [11, 22])) for c in range(4096)}
    assert len(outs) == 4096


def test_grad_uniform_layout(aten_philox):
    # element e: block e//8 of stream 0, 16-bit half (e%8): word (e%8)//2, low half first
    for seed in (0, 9, 2**40 + 3):
        for e in list(range(0, 40)) + [2**35 + 5, 2**35 + 8 * 77 + 7]:
            w = aten_philox(seed, 0, e // 8)
            j = e % 8
            h = (int(w[j // 2]) >> (16 * (j % 2))) & 0xFFFF
            assert ref.grad_uniform(seed, e) == h / 65536.0


def test_weight_shift_layout(aten_philox):
    for seed in (0, 1, 2, 12345, 2**63 + 1):
        w = aten_philox(seed, 1, 0)
        want = (int(w[0]) >> 8) / 2.0**24 - 0.5
        xi = ref.weight_shift(seed)
        assert xi == want
        assert -0.5 <= xi < 0.5


def test_grad_uniform_statistics():
    n = 200_000
    u = np.array([ref.grad_uniform(3, e) for e in range(n)])
    assert u.min() >= 0.0 and u.max() < 1.0
    assert np.all(u * 65536 == np.round(u * 65536))
    # mean and variance of U[0,1)
    assert abs(u.mean() - 0.5) < 4 * np.sqrt(1 / 12 / n)
    assert abs(u.var() - 1 / 12) < 1e-3
    # chi-square over 64 equal cells, 63 dof: mean 63, sd ~11.2
    counts = np.bincount((u * 64).astype(int), minlength=64)
    chi2 = ((counts - n / 64) ** 2 / (n / 64)).sum()
    assert chi2 < 63 + 6 * 11.3
    # lag-1 serial correlation, also across the 8 lanes of one block
    for lag in (1, 2, 7, 8):
        r = np.corrcoef(u[:-lag], u[lag:])[0, 1]
        assert abs(r) < 5 / np.sqrt(n)


def test_weight_shift_statistics():
    xi = np.array([ref.weight_shift(s) for s in range(50_000)])
    assert abs(xi.mean()) < 4 * np.sqrt(1 / 12 / xi.size)
    assert abs(xi.var() - 1 / 12) < 2e-3
    assert len(np.unique(xi)) > 49_000
