"""GPU parity of the learned-level codec and of the level fitting against the oracle. Codes, meta
and the fitted levels are bit-exact (the fit accumulates exact fixed-point sums and updates in
binary64 in the oracle's order)."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2302_02390_amd import binding as qb
from paper_2302_02390_amd import workloads as wl
from gpu_util import DEV, bits_equal, np_f32, np_u32, synth

pytestmark = pytest.mark.gpu


def _levels(bits, seed):
    """A sorted non-uniform table in [0,1] with a duplicate pair."""
    rng = np.random.default_rng(seed)
    lv = np.sort(rng.random(1 << bits)).astype(np.float32)
    lv[0], lv[-1] = 0.0, 1.0
    if bits >= 2:
        lv[2] = lv[1]
    return lv


@pytest.mark.parametrize("bucket", [32, 96, 128, 1024, 2048, 4096])
@pytest.mark.parametrize("bits", range(1, 9))
def test_quantize_and_dequantize_levels(bits, bucket):
    n = 5 * bucket + bucket // 2 + 3
    x, _ = synth(n, 900 + bits)
    for lv in (ref.levels_uniform(bits), _levels(bits, bits)):
        lvd = torch.from_numpy(lv).to(DEV)
        codes, meta = qb.alloc_packed(n, bits, bucket, DEV)
        qb.qsdp_quantize_levels(torch.from_numpy(x).to(DEV), bits, bucket, lvd, codes, meta.reshape(-1))
        wc, wm = ref.quantize_levels(x, bits, bucket, lv)
        assert np.array_equal(np_u32(meta), wm.view(np.uint32).reshape(-1))
        assert np.array_equal(np_u32(codes), wc)
        out = torch.empty(n, dtype=torch.float32, device=DEV)
        qb.qsdp_dequantize_levels(codes, meta.reshape(-1), n, bits, bucket, lvd, out)
        assert bits_equal(np_f32(out), ref.dequantize_levels(wc, wm, n, bits, bucket, lv))
        outh = torch.empty(n, dtype=torch.bfloat16, device=DEV)
        qb.qsdp_dequantize_levels(codes, meta.reshape(-1), n, bits, bucket, lvd, outh)
        assert np.array_equal(outh.view(torch.int16).cpu().numpy().view(np.uint16),
                              ref.dequantize_levels(wc, wm, n, bits, bucket, lv, ref.BF16))


@pytest.mark.parametrize("bits,bucket", [(2, 1024), (4, 1024), (5, 128), (8, 1024), (3, 96), (1, 32), (6, 4096)])
def test_fit_levels_bit_exact(bits, bucket):
    n = 150 * bucket + 17
    x, g = synth(n, 950 + bits)
    for data in (x, g):
        start = qb.levels_uniform(bits, DEV)
        assert np.array_equal(start.cpu().numpy(), ref.levels_uniform(bits))
        lv = start.clone()
        qb.qsdp_fit_levels(torch.from_numpy(data).to(DEV), bits, bucket, 0.01, lv)
        want = ref.fit_levels(data, bits, bucket, 0.01, ref.levels_uniform(bits))
        assert np.array_equal(lv.cpu().numpy().view(np.uint32), want.view(np.uint32))
        lv2 = start.clone()
        qb.qsdp_fit_levels(torch.from_numpy(data).to(DEV), bits, bucket, 0.05, lv2, max_batches=20)
        want2 = ref.fit_levels(data, bits, bucket, 0.05, ref.levels_uniform(bits), max_batches=20)
        assert np.array_equal(lv2.cpu().numpy().view(np.uint32), want2.view(np.uint32))


def test_learned_levels_lower_the_error_on_a_gpt_block():
    """The use the paper makes of it (Appendix C): fit on one d=768 attention matrix (W5) and on its
    gradient (G4), compare the relative L2 compression error with the uniform levels."""
    n, B = 768 * 768 * 3, 1024
    for bits, data in ((5, wl.weights(n, 31, DEV)), (4, wl.grads_student_t3(n, 32, DEV))):
        uni = qb.levels_uniform(bits, DEV)
        fit = uni.clone()
        qb.qsdp_fit_levels(data, bits, B, 0.01, fit)
        errs = []
        for lv in (uni, fit):
            codes, meta = qb.alloc_packed(n, bits, B, DEV)
            qb.qsdp_quantize_levels(data, bits, B, lv, codes, meta.reshape(-1))
            out = torch.empty(n, dtype=torch.float32, device=DEV)
            qb.qsdp_dequantize_levels(codes, meta.reshape(-1), n, bits, B, lv, out)
            errs.append(float(torch.linalg.vector_norm(out - data) / torch.linalg.vector_norm(data)))
        assert errs[1] < errs[0]
        assert torch.all(fit[1:] >= fit[:-1])
