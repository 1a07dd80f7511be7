"""Gradients handed over in a 16-bit format (Section 6, experimental setup: half-precision gradients
are converted to full precision before they are quantized). Widening to binary32 is exact, so the
expected result is the oracle's fp32 routine on the widened gradient; the widening itself is done
here by numpy (binary16) or by shifting the bit pattern (bf16), not by the library."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2302_02390_amd import binding as qb
from gpu_util import DEV, bits_equal, np_f32, np_u32, synth

pytestmark = pytest.mark.gpu


def _half_gradient(n, seed, dtype):
    """A heavy-tailed gradient rounded to `dtype`, with zeros of both signs, binary16 subnormals and
    the largest finite values; returns (GPU tensor of dtype, the same values widened to float32)."""
    _, g = synth(n, seed)
    g[:8] = [0.0, -0.0, 1e-7, -3e-6, 6.0e-8, 5.9e-5, -6.1e-5, 1.0]
    t = torch.from_numpy(g).to(dtype)
    if dtype == torch.float16:
        t[9], t[10] = 65504.0, -65504.0
        wide = t.view(torch.int16).numpy().view(np.float16).astype(np.float32)
    else:
        wide = (t.view(torch.int16).numpy().view(np.uint16).astype(np.uint32) << 16).view(np.float32)
    return t.to(DEV), wide


@pytest.mark.parametrize("dtype", [torch.float16, torch.bfloat16])
@pytest.mark.parametrize("B,bits,flags", [(1024, 4, 0), (128, 2, 0), (256, 3, 0), (512, 8, qb.QSDP_FLAG_GRAD_SHIFT),
                                          (2048, 5, 0), (4096, 8, qb.QSDP_FLAG_SYMMETRIC), (96, 4, 0), (32, 7, 0)])
def test_quantize_grad_16bit_input(dtype, B, bits, flags):
    n = 37 * B + B // 2 + 5
    g16, wide = _half_gradient(n, 700 + B, dtype)
    codes, meta = qb.alloc_packed(n, bits, B, DEV)
    qb.qsdp_quantize_grad_g16(g16, bits, B, 21, 4096, codes, meta.reshape(-1), flags)
    wc, wm = ref.quantize_grad(wide, bits, B, 21, index_offset=4096, flags=flags)
    assert np.array_equal(np_u32(meta), wm.view(np.uint32).reshape(-1))
    assert np.array_equal(np_u32(codes), wc)


@pytest.mark.parametrize("dtype", [torch.float16, torch.bfloat16])
@pytest.mark.parametrize("B,wbits,gbits,delta,flags", [(1024, 8, 4, 0.0, 0), (128, 4, 2, 0.0, 0),
                                                       (4096, 8, 8, 2.0**-10, 0), (512, 6, 3, 0.0, qb.QSDP_FLAG_KEEP_MASTER),
                                                       (96, 5, 4, 0.0, 0), (2048, 8, 4, 0.0, qb.QSDP_FLAG_GRAD_SHIFT)])
def test_fused_step_16bit_gradient(dtype, B, wbits, gbits, delta, flags):
    n = 29 * B + 3 * B // 4 + 1
    x, _ = synth(n, 710 + B)
    g16, wide = _half_gradient(n, 720 + B, dtype)
    want_x, want_c, want_m, want_sat = ref.fused_step(x, wide, 1e-3, wbits, gbits, B, delta, 5, index_offset=8,
                                                      emit_codes=True, flags=flags)
    xd = torch.from_numpy(x).to(DEV)
    codes, meta = qb.alloc_packed(n, wbits, B, DEV)
    sat = torch.zeros(1, dtype=torch.int64, device=DEV)
    qb.qsdp_fused_step_g16(xd, g16, 1e-3, wbits, gbits, B, delta, 5, 8, flags, codes, meta.reshape(-1), sat)
    assert bits_equal(np_f32(xd), want_x)
    assert np.array_equal(np_u32(codes), want_c) and np.array_equal(np_u32(meta), want_m.view(np.uint32).reshape(-1))
    assert int(sat) == want_sat
    x2 = torch.from_numpy(x).to(DEV)
    qb.qsdp_fused_step_g16(x2, g16, 1e-3, wbits, gbits, B, delta, 5, 8, flags)
    assert torch.equal(x2, xd)


@pytest.mark.parametrize("dtype", [torch.float16, torch.bfloat16])
def test_16bit_gradient_equals_the_fp32_entry_points_on_a_large_vector(dtype):
    """2^27 + a ragged tail: the 16-bit entry points against the fp32 ones on the widened gradient
    (those are checked against the oracle elsewhere), bit for bit."""
    n, B = (1 << 27) + 3 * 1024 + 77, 1024
    gen = torch.Generator(device=DEV).manual_seed(4242)
    g16 = (1e-3 * torch.randn(n, device=DEV, generator=gen)).to(dtype)
    x0 = 0.02 * torch.randn(n, device=DEV, generator=gen)
    wide = g16.float()
    c1, m1 = qb.alloc_packed(n, 4, B, DEV)
    c2, m2 = qb.alloc_packed(n, 4, B, DEV)
    qb.qsdp_quantize_grad_g16(g16, 4, B, 3, 0, c1, m1.reshape(-1))
    qb.qsdp_quantize_grad(wide, 4, B, 3, 0, c2, m2.reshape(-1))
    assert torch.equal(c1, c2) and torch.equal(m1, m2)
    xa, xb = x0.clone(), x0.clone()
    w1, wm1 = qb.alloc_packed(n, 8, B, DEV)
    w2, wm2 = qb.alloc_packed(n, 8, B, DEV)
    qb.qsdp_fused_step_g16(xa, g16, 1e-3, 8, 4, B, 0.0, 3, 0, 0, w1, wm1.reshape(-1))
    qb.qsdp_fused_step(xb, wide, 1e-3, 8, 4, B, 0.0, 3, 0, w2, wm2.reshape(-1))
    assert torch.equal(xa, xb) and torch.equal(w1, w2) and torch.equal(wm1, wm2)
