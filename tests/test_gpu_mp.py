"""The mixed-precision form of the fused step: gradient in fp32 / fp16 / bf16, and the new quantized weights
written once more in 16 bits. Expected values: the oracle's fused step on the widened gradient, and the
oracle's decode of the codes it emits, rounded to the 16-bit format (`ref.dequantize(..., BF16 / F16)`)."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2302_02390_amd import binding as qb
from gpu_util import DEV, bits_equal, np_f32, np_u32, synth

pytestmark = pytest.mark.gpu

REF_DT = {torch.bfloat16: ref.BF16, torch.float16: ref.F16}


def _h(t):
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


@pytest.mark.parametrize("gdtype", [torch.float32, torch.float16, torch.bfloat16])
@pytest.mark.parametrize("xdtype", [torch.bfloat16, torch.float16])
@pytest.mark.parametrize("B,wbits,gbits,delta,flags", [(1024, 8, 4, 0.0, 0), (128, 4, 2, 0.0, 0), (96, 5, 4, 0.0, 0),
                                                       (4096, 8, 8, 2.0**-10, 0), (2048, 6, 3, 0.0, qb.QSDP_FLAG_KEEP_MASTER),
                                                       (512, 8, 4, 0.0, qb.QSDP_FLAG_KEEP_MASTER | qb.QSDP_FLAG_GRAD_SHIFT)])
def test_fused_step_with_16bit_copy_of_the_new_weights(gdtype, xdtype, B, wbits, gbits, delta, flags):
    n = 19 * B + 2 * B // 3 + 3
    x, g = synth(n, 1300 + B)
    x[:B] *= np.float32(2e6)                  # a bucket whose values overflow binary16 / lose bf16 precision
    x[B:2 * B] *= np.float32(1e-4)            # and one in binary16's subnormal range
    gt = torch.from_numpy(g).to(gdtype)
    wide = gt.float().numpy()
    want_x, want_c, want_m, want_sat = ref.fused_step(x, wide, 1e-3, wbits, gbits, B, delta, 9, index_offset=16,
                                                      emit_codes=True, flags=flags)
    want16 = ref.dequantize(want_c, want_m, n, wbits, B, REF_DT[xdtype])
    xd = torch.from_numpy(x).to(DEV)
    x16 = torch.full((n + 16,), 7.0, dtype=xdtype, device=DEV)
    codes, meta = qb.alloc_packed(n, wbits, B, DEV)
    sat = torch.zeros(1, dtype=torch.int64, device=DEV)
    qb.qsdp_fused_step_mp(xd, gt.to(DEV), 1e-3, wbits, gbits, B, delta, 9, 16, flags, codes, meta.reshape(-1), x16[:n],
                          sat)
    assert bits_equal(np_f32(xd), want_x)
    assert np.array_equal(np_u32(codes), want_c) and np.array_equal(np_u32(meta), want_m.view(np.uint32).reshape(-1))
    assert int(sat) == want_sat
    assert np.array_equal(_h(x16[:n]), want16)
    assert bool((x16[n:] == 7.0).all())
    # without code output, and without the 16-bit copy: same x
    x2 = torch.from_numpy(x).to(DEV)
    y16 = torch.empty(n, dtype=xdtype, device=DEV)
    qb.qsdp_fused_step_mp(x2, gt.to(DEV), 1e-3, wbits, gbits, B, delta, 9, 16, flags, x16=y16)
    assert torch.equal(x2, xd) and np.array_equal(_h(y16), want16)
    x3 = torch.from_numpy(x).to(DEV)
    qb.qsdp_fused_step_mp(x3, gt.to(DEV), 1e-3, wbits, gbits, B, delta, 9, 16, flags)
    assert torch.equal(x3, xd)


def test_mixed_precision_step_argument_errors():
    n, B = 2048, 1024
    x = torch.zeros(n, device=DEV)
    g = torch.zeros(n, device=DEV)
    L = qb.lib()
    import ctypes as C
    p = lambda t: C.c_void_p(t.data_ptr())  # noqa: E731
    x16 = torch.zeros(n + 8, dtype=torch.bfloat16, device=DEV)
    # unknown gradient format, fp32 as the 16-bit output format, misaligned 16-bit output
    assert L.qsdp_fused_step_mp(p(x), p(g), 3, n, 1e-3, 8, 4, B, 0.0, 0, 0, 0, None, None, None, 1, None, None) == qb.QSDP_EINVAL
    assert L.qsdp_fused_step_mp(p(x), p(g), 0, n, 1e-3, 8, 4, B, 0.0, 0, 0, 0, None, None, p(x16), 0, None, None) == qb.QSDP_EINVAL
    assert L.qsdp_fused_step_mp(p(x), p(g), 0, n, 1e-3, 8, 4, B, 0.0, 0, 0, 0, None, None, p(x16[1:]), 1, None, None) == qb.QSDP_EALIGN
    with pytest.raises(ValueError):
        qb.qsdp_fused_step_mp(x, g, 1e-3, 8, 4, B, 0.0, 0, x16=x16[:100])


@pytest.mark.parametrize("gdtype,xdtype", [(torch.float16, torch.float16), (torch.bfloat16, torch.bfloat16),
                                           (torch.float32, torch.bfloat16)])
@pytest.mark.parametrize("B,wbits,gbits,flags", [(1024, 8, 4, 0), (128, 5, 4, qb.QSDP_FLAG_KEEP_MASTER), (96, 6, 3, 0)])
def test_segmented_mixed_precision_step(gdtype, xdtype, B, wbits, gbits, flags):
    """Per-layer tensors in one launch: every tensor equals the oracle's single-tensor step on the widened
    gradient (index_offset + the tensor's position), its 16-bit copy the oracle's decode of the emitted codes."""
    sizes = [768, 2304, 768 * 12, 8, 3072, 16, 1024 * 3 + 8, 4096 * 2, 24, 5000 + 3]
    n = sum(sizes)
    x, g = synth(n, 1350 + B)
    gt = torch.from_numpy(g).to(gdtype)
    wide = gt.float().numpy()
    segs = qb.Segments(sizes, B, DEV)
    xd = torch.from_numpy(x).to(DEV)
    x16 = torch.empty(n, dtype=xdtype, device=DEV)
    codes, meta = segs.alloc_packed(wbits)
    sat = torch.zeros(1, dtype=torch.int64, device=DEV)
    qb.qsdp_fused_step_segmented_mp(xd, gt.to(DEV), segs, 1e-3, wbits, gbits, 0.0, 4, 64, flags, codes,
                                    meta.reshape(-1), x16, sat)
    wx, wc, wm, w16, off = [], [], [], [], 0
    for s in sizes:
        a, c, m, _ = ref.fused_step(x[off:off + s], wide[off:off + s], 1e-3, wbits, gbits, B, 0.0, 4,
                                    index_offset=64 + off, emit_codes=True, flags=flags)
        wx.append(a); wc.append(c); wm.append(m.reshape(-1))
        w16.append(ref.dequantize(c, m, s, wbits, B, REF_DT[xdtype]))
        off += s
    assert bits_equal(np_f32(xd), np.concatenate(wx))
    assert np.array_equal(np_u32(codes), np.concatenate(wc)) and np.array_equal(np_u32(meta), np.concatenate(wm).view(np.uint32))
    assert np.array_equal(_h(x16), np.concatenate(w16))


@pytest.mark.parametrize("gdtype,xdtype", [(torch.float16, torch.float16), (torch.bfloat16, torch.bfloat16),
                                           (torch.float32, torch.float16)])
@pytest.mark.parametrize("B,wbits,gbits,flags", [(1024, 8, 4, 0), (4096, 5, 4, qb.QSDP_FLAG_KEEP_MASTER), (96, 6, 3, 0),
                                                 (128, 8, 2, qb.QSDP_FLAG_GRAD_SHIFT)])
def test_adamw_step_in_mixed_precision(gdtype, xdtype, B, wbits, gbits, flags):
    """Two AdamW steps with the gradient in 16 bits and the 16-bit copy of the new weights: moments, weights,
    codes as the oracle's AdamW step on the widened gradient, the copy as its decode of the emitted codes."""
    n = 9 * B + B // 2 + 5
    x, g = synth(n, 1400 + B)
    hyper = dict(lr=2e-4, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)
    xd = torch.from_numpy(x).to(DEV)
    md = torch.zeros(n, device=DEV)
    vd = torch.zeros(n, device=DEV)
    hx, hm, hv = x, np.zeros(n, np.float32), np.zeros(n, np.float32)
    for t in (1, 2):
        gt = torch.from_numpy((g * np.float32(1 + 0.3 * t)).astype(np.float32)).to(gdtype)
        wide = gt.float().numpy()
        c1, c2 = 1 - 0.9 ** t, 1 - 0.95 ** t
        codes, meta = qb.alloc_packed(n, wbits, B, DEV)
        x16 = torch.empty(n, dtype=xdtype, device=DEV)
        qb.qsdp_fused_adamw_step_mp(xd, gt.to(DEV), md, vd, bias1=c1, bias2=c2, wbits=wbits, gbits=gbits, bucket=B,
                                    delta=0.0, seed=t, index_offset=8, flags=flags, wcodes=codes,
                                    wmeta=meta.reshape(-1), x16=x16, **hyper)
        hx, hm, hv, wc, wm, _ = ref.fused_adamw_step(hx, wide, hm, hv, bias1=c1, bias2=c2, wbits=wbits, gbits=gbits,
                                                     bucket=B, delta=0.0, seed=t, index_offset=8, flags=flags,
                                                     emit_codes=True, **hyper)
        assert bits_equal(np_f32(xd), hx) and bits_equal(np_f32(md), hm) and bits_equal(np_f32(vd), hv), t
        assert np.array_equal(np_u32(codes), wc) and np.array_equal(np_u32(meta), wm.view(np.uint32).reshape(-1)), t
        assert np.array_equal(_h(x16), ref.dequantize(wc, wm, n, wbits, B, REF_DT[xdtype])), t
