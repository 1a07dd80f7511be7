"""GPU parity of qsdp_dequantize_add against the oracle (bit-exact: same additions in the same
order)."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2302_02390_amd import binding as qb
from paper_2302_02390_amd import workloads as wl
from gpu_util import DEV, bits_equal, guarded, guards_intact, np_f32

pytestmark = pytest.mark.gpu


def _peer_slices(P, n, bits, B, seed):
    rng = np.random.default_rng(seed)
    g = (rng.standard_t(3, size=(P, n)) * 1e-3).astype(np.float32)
    cs, ms = [], []
    for p in range(P):
        c, m = ref.quantize_grad(g[p], bits, B, seed + p)
        cs.append(c)
        ms.append(m.reshape(-1))
    return np.stack(cs), np.stack(ms)


@pytest.mark.parametrize("B", [32, 96, 1024, 4096])
@pytest.mark.parametrize("P,bits", [(1, 8), (2, 4), (3, 3), (8, 8), (8, 2), (5, 6), (4, 1), (2, 5), (2, 7)])
def test_dequantize_add_bit_exact(P, bits, B):
    n = 5 * B + B // 2 + 3
    codes, meta = _peer_slices(P, n, bits, B, 10 * P + bits)
    alpha = 1.0 / P
    cd = torch.from_numpy(codes.view(np.int32)).to(DEV)
    md = torch.from_numpy(meta).to(DEV)
    ofull, out = guarded(n, torch.float32, 9.0)
    qb.qsdp_dequantize_add(cd, md, P, n, bits, B, alpha, out)
    torch.cuda.synchronize()
    assert guards_intact(ofull, n, 9.0)
    want = ref.dequantize_add(codes, meta, P, n, bits, B, alpha)
    assert bits_equal(np_f32(out), want)


def test_dequantize_add_gpt_block_eight_peers():
    """One d=2048 transformer block (50,358,272 elements), 8 peers, 4-bit gradients: the slices are
    produced by the library's quantizer, the sum is compared with the oracle on the whole block."""
    n, B, P, bits = wl.block_numel(2048), 1024, 8, 4
    nb = n // B
    codes = torch.empty((P, nb * B * bits // 32), dtype=torch.int32, device=DEV)
    meta = torch.empty((P, nb * 2), dtype=torch.float32, device=DEV)
    for p in range(P):
        g = wl.grads_student_t3(n, 500 + p, DEV)
        qb.qsdp_quantize_grad(g, bits, B, p, 0, codes[p], meta[p])
    out = torch.empty(n, dtype=torch.float32, device=DEV)
    qb.qsdp_dequantize_add(codes, meta, P, n, bits, B, 1.0 / P, out)
    ref.set_threads(8)
    want = ref.dequantize_add(codes.cpu().numpy().view(np.uint32), meta.cpu().numpy(), P, n, bits, B, 1.0 / P)
    ref.set_threads(1)
    assert bits_equal(np_f32(out), want)


def test_dequantize_add_errors():
    codes = torch.zeros((2, 256), dtype=torch.int32, device=DEV)
    meta = torch.zeros((2, 2), dtype=torch.float32, device=DEV)
    out = torch.zeros(1024, dtype=torch.float32, device=DEV)
    L = qb.lib()
    import ctypes as C
    args = lambda **kw: None
    assert L.qsdp_dequantize_add(C.c_void_p(codes.data_ptr()), 1024, C.c_void_p(meta.data_ptr()), 8, 0, 1024, 8,
                                 1024, 1.0, C.c_void_p(out.data_ptr()), None) == qb.QSDP_EINVAL
    assert L.qsdp_dequantize_add(C.c_void_p(codes.data_ptr()), 512, C.c_void_p(meta.data_ptr()), 8, 2, 1024, 8,
                                 1024, 1.0, C.c_void_p(out.data_ptr()), None) == qb.QSDP_EINVAL  # stride < slice
    assert L.qsdp_dequantize_add(C.c_void_p(codes.data_ptr()), 1024, C.c_void_p(meta.data_ptr()), 8, 2, 1024, 8,
                                 1024, float("inf"), C.c_void_p(out.data_ptr()), None) == qb.QSDP_EINVAL
    torch.cuda.synchronize()
