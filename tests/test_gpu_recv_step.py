"""GPU parity of qsdp_recv_step (the shard owner's step with P workers: decode-and-average the
peers' quantized gradient slices, SGD step, Q^w) against the oracle, bit for bit."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2302_02390_amd import binding as qb
from gpu_util import DEV, bits_equal, np_f32, np_u32, synth

pytestmark = pytest.mark.gpu


def _peer_slices(n, P, gbits, B, seed):
    """P peers' gradients quantized by the oracle: (codes u32[P, words], meta f32[P, nb*2])."""
    cs, ms = [], []
    for p in range(P):
        _, g = synth(n, seed + 13 * p)
        c, m = ref.quantize_grad(g, gbits, B, 200 + p)
        cs.append(c); ms.append(m.reshape(-1))
    return np.stack(cs), np.stack(ms)


def _to_device_rows(a, dtype, pad_to):
    """Rows of `a` on the GPU with the row stride padded to a multiple of pad_to elements."""
    P, w = a.shape
    row = -(-w // pad_to) * pad_to
    t = torch.zeros((P, row), dtype=dtype, device=DEV)
    t[:, :w] = torch.from_numpy(a.view(np.int32) if dtype == torch.int32 else a).to(DEV)
    return t[:, :w]


CASES = [
    # n, P, wbits, gbits, B, delta, flags
    (300 * 1024 + 77, 8, 8, 4, 1024, 0.0, 0),
    (40 * 1024, 1, 8, 8, 1024, 0.0, 0),
    (17 * 128 + 5, 3, 4, 2, 128, 0.0, 0),
    (9 * 256 + 255, 5, 6, 3, 256, 0.0, 0),
    (33 * 512 + 8, 4, 3, 6, 512, 0.0, qb.QSDP_FLAG_SYMMETRIC),
    (7 * 2048 + 1000, 9, 8, 4, 2048, 0.0, 0),
    (5 * 4096 + 4095, 2, 2, 8, 4096, 0.0, qb.QSDP_FLAG_NO_SHIFT),
    (20 * 1024 + 300, 8, 8, 4, 1024, 2.0 ** -10, 0),
    (20 * 1024 + 300, 6, 4, 4, 1024, 2.0 ** -10, 0),       # saturating lattice
    (11 * 96 + 40, 4, 5, 7, 96, 0.0, 0),                   # generic bucket size: block kernel
    (6 * 1024 + 1, 3, 7, 4, 1024, 0.0, 0),                 # odd weight width
    (6 * 1024 + 1, 3, 8, 5, 1024, 0.0, 0),                 # odd gradient width
    (100, 2, 8, 4, 1024, 0.0, 0),                          # less than one bucket
]


@pytest.mark.parametrize("n,P,wbits,gbits,B,delta,flags", CASES)
@pytest.mark.parametrize("emit", [False, True])
def test_recv_step_matches_oracle(n, P, wbits, gbits, B, delta, flags, emit):
    x, _ = synth(n, 31 + n % 101)
    cs, ms = _peer_slices(n, P, gbits, B, 500 + P)
    alpha, lr, seed = 1.0 / P, 0.05, 9
    want_x, want_c, want_m, want_sat = ref.recv_step(x, cs, ms, P, alpha, lr, wbits, gbits, B, delta, seed, flags,
                                                     emit_codes=True)
    xd = torch.from_numpy(x).to(DEV)
    gc = _to_device_rows(cs, torch.int32, 4)
    gm = _to_device_rows(ms, torch.float32, 1)
    sat = torch.zeros(1, dtype=torch.int64, device=DEV)
    wc = wm = None
    if emit:
        wc, wm = qb.alloc_packed(n, wbits, B, DEV)
        wc.fill_(-1)
    qb.qsdp_recv_step(xd, gc, gm, P, alpha, lr, wbits, gbits, B, delta, seed, flags,
                      wc, None if wm is None else wm.reshape(-1), sat)
    assert bits_equal(np_f32(xd), want_x)
    assert int(sat) == want_sat
    if emit:
        assert np.array_equal(np_u32(wc), want_c)
        assert np.array_equal(np_u32(wm).reshape(-1), want_m.view(np.uint32).reshape(-1))


def test_recv_step_equals_decode_add_then_update_on_the_gpu():
    """The fused call against the two-call route on the GPU: qsdp_dequantize_add, then an exact
    axpy in torch, then qsdp_quantize_weight + qsdp_dequantize."""
    n, P, B = 64 * 1024 + 512, 8, 1024
    x, _ = synth(n, 3)
    cs, ms = _peer_slices(n, P, 4, B, 900)
    gc = _to_device_rows(cs, torch.int32, 4)
    gm = _to_device_rows(ms, torch.float32, 4)
    xd = torch.from_numpy(x).to(DEV)
    ghat = torch.empty(n, dtype=torch.float32, device=DEV)
    qb.qsdp_dequantize_add(gc.contiguous(), gm.contiguous(), P, n, 4, B, 1.0 / P, ghat)
    lr = 0.5                                   # power of two: x - lr*ghat in fp64 then rounded = fma
    y = (xd.double() - lr * ghat.double()).float()
    wc, wm = qb.alloc_packed(n, 8, B, DEV)
    qb.qsdp_quantize_weight(y, 8, B, 0.0, 4, wc, wm.reshape(-1))
    two_call = torch.empty(n, dtype=torch.float32, device=DEV)
    qb.qsdp_dequantize(wc, wm.reshape(-1), n, 8, B, two_call)
    wc2, wm2 = qb.alloc_packed(n, 8, B, DEV)
    qb.qsdp_recv_step(xd, gc, gm, P, 1.0 / P, lr, 8, 4, B, 0.0, 4, 0, wc2, wm2.reshape(-1))
    assert torch.equal(xd, two_call) and torch.equal(wc, wc2) and torch.equal(wm, wm2)


def test_recv_step_rejects_bad_arguments():
    x = torch.zeros(2048, dtype=torch.float32, device=DEV)
    gc = torch.zeros((2, 256), dtype=torch.int32, device=DEV)
    gm = torch.zeros((2, 4), dtype=torch.float32, device=DEV)
    with pytest.raises(qb.QsdpError):
        qb.qsdp_recv_step(x, gc, gm, 2, 0.5, 1e-3, 8, 4, 1024, 0.0, 0, qb.QSDP_FLAG_GRAD_SHIFT)
    with pytest.raises(ValueError):                                                  # the binding's size check
        qb.qsdp_recv_step(x, gc[:, :128], gm, 2, 0.5, 1e-3, 8, 8, 1024, 0.0, 0)     # rows shorter than a slice
    with pytest.raises(qb.QsdpError):
        qb.qsdp_recv_step(x, gc, gm, 2, float("nan"), 1e-3, 8, 4, 1024, 0.0, 0)
    qb.qsdp_recv_step(x, gc, gm, 2, 0.5, 1e-3, 8, 4, 1024, 0.0, 0)
