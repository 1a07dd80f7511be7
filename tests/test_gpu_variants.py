"""GPU parity of the quantizer variants (flags) against the oracle."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2302_02390_amd import binding as qb
from gpu_util import DEV, bits_equal, np_f32, np_u32, synth

pytestmark = pytest.mark.gpu

FLAGS = [1, 2, 4, 1 | 2, 1 | 4, 2 | 4, 1 | 2 | 4]


@pytest.mark.parametrize("bucket", [32, 96, 128, 1024, 4096])
@pytest.mark.parametrize("flags", FLAGS)
def test_variant_quantizers_and_fused_step(flags, bucket):
    n = 6 * bucket + bucket // 2 + 3
    x, g = synth(n, 700 + flags)
    gd = torch.from_numpy(g).to(DEV)
    xd = torch.from_numpy(x).to(DEV)
    for bits in (3, 4, 8, 5):
        codes, meta = qb.alloc_packed(n, bits, bucket, DEV)
        qb.qsdp_quantize_grad_ex(gd, bits, bucket, 21, 16, flags, codes, meta.reshape(-1))
        wc, wm = ref.quantize_grad(g, bits, bucket, 21, index_offset=16, flags=flags)
        assert np.array_equal(np_u32(codes), wc) and np.array_equal(np_u32(meta), wm.view(np.uint32).reshape(-1))
        for delta in (0.0, 2.0**-9):
            sat = torch.zeros(1, dtype=torch.int64, device=DEV)
            qb.qsdp_quantize_weight_ex(xd, bits, bucket, delta, 21, flags, codes, meta.reshape(-1), sat)
            wc, wm, ws = ref.quantize_weight(x, bits, bucket, delta, 21, flags=flags)
            assert np.array_equal(np_u32(codes), wc) and np.array_equal(np_u32(meta), wm.view(np.uint32).reshape(-1))
            assert int(sat) == ws
    for wbits, gbits, delta in ((8, 4, 0.0), (6, 3, 0.0), (8, 4, 2.0**-10), (7, 5, 0.0)):
        x1 = xd.clone()
        codes, meta = qb.alloc_packed(n, wbits, bucket, DEV)
        sat = torch.zeros(1, dtype=torch.int64, device=DEV)
        qb.qsdp_fused_step_ex(x1, gd, 1e-2, wbits, gbits, bucket, delta, 5, 8, flags, codes, meta.reshape(-1), sat)
        want, wc, wm, ws = ref.fused_step(x, g, 1e-2, wbits, gbits, bucket, delta, 5, index_offset=8,
                                          emit_codes=True, flags=flags)
        assert bits_equal(np_f32(x1), want)
        assert np.array_equal(np_u32(codes), wc) and np.array_equal(np_u32(meta), wm.view(np.uint32).reshape(-1))
        assert int(sat) == ws
        x2 = xd.clone()
        qb.qsdp_fused_step_ex(x2, gd, 1e-2, wbits, gbits, bucket, delta, 5, 8, flags)
        assert torch.equal(x1, x2)


def test_unknown_flag_rejected():
    g = torch.zeros(1024, dtype=torch.float32, device=DEV)
    codes, meta = qb.alloc_packed(1024, 8, 1024, DEV)
    with pytest.raises(qb.QsdpError) as e:
        qb.qsdp_quantize_grad_ex(g, 8, 1024, 0, 0, 8, codes, meta.reshape(-1))
    assert e.value.status == qb.QSDP_EINVAL
