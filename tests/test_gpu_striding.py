"""The kernels launch one wave (or workgroup) per unit of work up to 2^20 workgroups and stride
beyond that. QSDP_DEBUG_MAXGRID lowers that cap, so the striding loops (and the double-buffered
LDS reductions of the multi-wave buckets) are checked for parity on small inputs."""
import os

import numpy as np
import pytest
import torch

from oracle import ref
from paper_2302_02390_amd import binding as qb
from gpu_util import DEV, bits_equal, np_f32, np_u32, synth

pytestmark = pytest.mark.gpu


@pytest.fixture(params=[1, 3])
def tiny_grid(request):
    os.environ["QSDP_DEBUG_MAXGRID"] = str(request.param)
    yield request.param
    del os.environ["QSDP_DEBUG_MAXGRID"]


@pytest.mark.parametrize("bucket", [96, 128, 1024, 2048, 4096])
def test_all_entry_points_with_a_tiny_grid(tiny_grid, bucket):
    n = 41 * bucket + bucket // 3 + 1
    x, g = synth(n, 1300 + bucket)
    xd, gd = torch.from_numpy(x).to(DEV), torch.from_numpy(g).to(DEV)
    codes, meta = qb.alloc_packed(n, 4, bucket, DEV)
    qb.qsdp_quantize_grad(gd, 4, bucket, 3, 0, codes, meta.reshape(-1))
    wc, wm = ref.quantize_grad(g, 4, bucket, 3)
    assert np.array_equal(np_u32(codes), wc) and np.array_equal(np_u32(meta), wm.view(np.uint32).reshape(-1))
    out = torch.empty(n, dtype=torch.float32, device=DEV)
    qb.qsdp_dequantize(codes, meta.reshape(-1), n, 4, bucket, out)
    assert bits_equal(np_f32(out), ref.dequantize(wc, wm, n, 4, bucket))
    outh = torch.empty(n, dtype=torch.bfloat16, device=DEV)
    qb.qsdp_dequantize(codes, meta.reshape(-1), n, 4, bucket, outh)
    assert np.array_equal(outh.view(torch.int16).cpu().numpy().view(np.uint16),
                          ref.dequantize(wc, wm, n, 4, bucket, ref.BF16))
    c2 = torch.stack([codes, codes])
    m2 = torch.stack([meta.reshape(-1), meta.reshape(-1)])
    qb.qsdp_dequantize_add(c2, m2, 2, n, 4, bucket, 0.5, out)
    assert bits_equal(np_f32(out), ref.dequantize_add(np.stack([wc, wc]), np.stack([wm.reshape(-1)] * 2), 2, n, 4,
                                                     bucket, 0.5))
    wcodes, wmeta = qb.alloc_packed(n, 8, bucket, DEV)
    x1 = xd.clone()
    qb.qsdp_fused_step(x1, gd, 1e-3, 8, 4, bucket, 0.0, 5, 0, wcodes, wmeta.reshape(-1))
    want, fc, fm, _ = ref.fused_step(x, g, 1e-3, 8, 4, bucket, 0.0, 5, emit_codes=True)
    assert bits_equal(np_f32(x1), want)
    assert np.array_equal(np_u32(wcodes), fc) and np.array_equal(np_u32(wmeta), fm.view(np.uint32).reshape(-1))
    qb.qsdp_fused_step_codes(wcodes, wmeta.reshape(-1), gd, 1e-3, 8, 4, bucket, 0.0, 6)
    hc, hm, _ = ref.fused_step_codes(fc, fm, g, 1e-3, 8, 4, bucket, 0.0, 6)
    assert np.array_equal(np_u32(wcodes), hc) and np.array_equal(np_u32(wmeta), hm.view(np.uint32).reshape(-1))
    sat = torch.zeros(1, dtype=torch.int64, device=DEV)
    qb.qsdp_quantize_weight(xd, 4, bucket, 2.0**-8, 9, codes, meta.reshape(-1), sat)
    wc, wm, ws = ref.quantize_weight(x, 4, bucket, 2.0**-8, 9)
    assert np.array_equal(np_u32(codes), wc) and int(sat) == ws
