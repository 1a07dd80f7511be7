"""The plain streaming kernels bench.py times as the memory system's ceilings (libqsdp_bench.so) do what
their names say: a ceiling measured with a kernel that skips part of its traffic would be worthless."""
import numpy as np
import pytest
import torch

from paper_2302_02390_amd import bench_support as bs
from gpu_util import DEV

pytestmark = pytest.mark.gpu

N = 1024 * 4099  # whole tiles, not a multiple of the workgroup's four tiles


def _pair(seed):
    gen = torch.Generator(device=DEV).manual_seed(seed)
    return (torch.randn(N, device=DEV, generator=gen), torch.randn(N, device=DEV, generator=gen))


def test_fill_copy_and_read_touch_every_element():
    a, b = _pair(1)
    bs.fill(b, 0.5)
    assert bool((b == 0.5).all())
    bs.copy(a, b)
    assert torch.equal(a, b)
    sink = torch.zeros(4, dtype=torch.float32, device=DEV)
    bs.read(a, sink)            # reads only; the sink stays untouched for finite data
    torch.cuda.synchronize()
    assert bool((sink == 0).all())


@pytest.mark.parametrize("cap", [0, 27000, 50000])
def test_axpy_is_one_fused_multiply_add_per_element(cap):
    x, g = _pair(2)
    want = np.float32(np.float64(x.cpu().numpy()) - np.float64(np.float32(0.125)) * np.float64(g.cpu().numpy()))
    bs.axpy(x, g, 0.125, cap)
    assert np.array_equal(x.cpu().numpy(), want)   # lr a power of two: the product is exact, one rounding


@pytest.mark.parametrize("cap", [0, 60000])
def test_moments_update_all_three_streams(cap):
    x, g = _pair(3)
    m, v = _pair(4)
    x0, g0, m0, v0 = (t.cpu().numpy().astype(np.float64) for t in (x, g, m, v))
    bs.moments(x, g, m, v, 0.25, 0.5, cap)
    m1 = np.float32(0.5 * m0 + g0)
    v1 = np.float32(0.5 * v0 + np.float64(np.float32(g0 * g0)))
    x1 = np.float32(x0 - 0.25 * np.float64(m1))
    assert np.array_equal(m.cpu().numpy(), m1) and np.array_equal(v.cpu().numpy(), v1)
    assert np.array_equal(x.cpu().numpy(), x1)


@pytest.mark.parametrize("bits", [4, 8])
def test_encode_writes_the_stated_bytes_from_every_input_word(bits):
    a, _ = _pair(5)
    words = N * bits // 32
    out = torch.full((words + 64,), 0x5A5A5A5A, dtype=torch.int32, device=DEV)
    bs.encode(a, bits, out[:words])
    first = out[:words].clone()
    assert bool((out[words:] == 0x5A5A5A5A).all())
    assert float((first != 0x5A5A5A5A).float().mean()) > 0.99        # the whole output range was written
    # every input word feeds the output: flipping one element's bits anywhere changes the output
    for e in (0, 517, N // 2 + 3, N - 1):
        a2 = a.clone()
        a2[e] = -a2[e]
        bs.encode(a2, bits, out[:words])
        assert not torch.equal(out[:words], first), e
