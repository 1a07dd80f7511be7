"""GPU parity of the AdamW-flavoured quantized step against the oracle. Moments, iterate, codes and
meta are compared bit for bit (same binary32 operations in the same order, IEEE division and
square root on both sides)."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2302_02390_amd import binding as qb
from paper_2302_02390_amd import workloads as wl
from gpu_util import DEV, bits_equal, gather_rows, np_f32, np_u32, sample_bucket_ids, synth

pytestmark = pytest.mark.gpu

HYPER = dict(lr=2e-4, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)


@pytest.mark.parametrize("bucket", [32, 96, 128, 1024, 2048, 4096])
@pytest.mark.parametrize("wbits,gbits,delta,flags", [(8, 4, 0.0, 0), (8, 8, 0.0, 0), (6, 3, 0.0, 0), (5, 7, 0.0, 0),
                                                     (8, 4, 2.0**-10, 0), (8, 4, 0.0, 1), (4, 2, 0.0, 4),
                                                     (8, 4, 0.0, 7)])
def test_adamw_steps_bit_exact(wbits, gbits, delta, flags, bucket):
    n = 6 * bucket + bucket // 2 + 7
    x, g = synth(n, 1100 + wbits + gbits)
    xd = torch.from_numpy(x).to(DEV)
    md = torch.zeros(n, dtype=torch.float32, device=DEV)
    vd = torch.zeros(n, dtype=torch.float32, device=DEV)
    hx, hm, hv = x, np.zeros(n, np.float32), np.zeros(n, np.float32)
    rng = np.random.default_rng(bucket)
    for t in range(1, 4):
        gt = (g * np.float32(1 + 0.1 * t) + rng.normal(size=n).astype(np.float32) * 1e-4).astype(np.float32)
        gd = torch.from_numpy(gt).to(DEV)
        bc1, bc2 = 1 - 0.9**t, 1 - 0.95**t
        codes, meta = qb.alloc_packed(n, wbits, bucket, DEV)
        sat = torch.zeros(1, dtype=torch.int64, device=DEV)
        emit = t % 2 == 1
        qb.qsdp_fused_adamw_step(xd, gd, md, vd, bias1=bc1, bias2=bc2, wbits=wbits, gbits=gbits, bucket=bucket,
                                 delta=delta, seed=t, index_offset=16, flags=flags,
                                 wcodes=codes if emit else None, wmeta=meta.reshape(-1) if emit else None,
                                 n_saturated=sat, **HYPER)
        hx, hm, hv, wc, wm, ws = ref.fused_adamw_step(hx, gt, hm, hv, bias1=bc1, bias2=bc2, wbits=wbits,
                                                      gbits=gbits, bucket=bucket, delta=delta, seed=t,
                                                      index_offset=16, flags=flags, emit_codes=emit, **HYPER)
        assert bits_equal(np_f32(md), hm) and bits_equal(np_f32(vd), hv), t
        assert np.all(np.abs(np_f32(xd).astype(np.float64) - hx) <= 1e-6 * np.maximum(np.abs(hx), 1e-30))
        assert bits_equal(np_f32(xd), hx), t
        assert int(sat) == ws
        if emit:
            assert np.array_equal(np_u32(codes), wc) and np.array_equal(np_u32(meta), wm.view(np.uint32).reshape(-1))


def test_adamw_on_gpt350m_sampled_buckets():
    n, B = wl.model_numel(wl.GPT_350M), 1024
    x = wl.weights(n, 1238, DEV)
    g = wl.grads_student_t3(n, 1239, DEV)
    m = torch.zeros(n, dtype=torch.float32, device=DEV)
    v = torch.zeros(n, dtype=torch.float32, device=DEV)
    ids = sample_bucket_ids(n // B, 128, 3)
    gb = gather_rows(g, ids, B)
    for t in (1, 2):
        xb, mb, vb = gather_rows(x, ids, B), gather_rows(m, ids, B), gather_rows(v, ids, B)
        bc1, bc2 = 1 - 0.9**t, 1 - 0.95**t
        qb.qsdp_fused_adamw_step(x, g, m, v, bias1=bc1, bias2=bc2, wbits=8, gbits=4, bucket=B, delta=0.0, seed=t,
                                 **HYPER)
        xa, ma, va = gather_rows(x, ids, B), gather_rows(m, ids, B), gather_rows(v, ids, B)
        for r, j in enumerate(ids):
            hx, hm, hv, _, _, _ = ref.fused_adamw_step(xb[r], gb[r], mb[r], vb[r], bias1=bc1, bias2=bc2, wbits=8,
                                                       gbits=4, bucket=B, delta=0.0, seed=t,
                                                       index_offset=int(j) * B, **HYPER)
            assert bits_equal(xa[r], hx) and bits_equal(ma[r], hm) and bits_equal(va[r], hv), (t, int(j))


def test_adamw_argument_errors():
    z = torch.zeros(1024, dtype=torch.float32, device=DEV)
    base = dict(lr=1e-3, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.0, bias1=0.1, bias2=0.05, wbits=8,
                gbits=4, bucket=1024, delta=0.0, seed=0)
    for kw in (dict(beta1=1.0), dict(eps=0.0), dict(bias2=0.0), dict(flags=16), dict(wbits=9)):
        a = dict(base)
        a.update(kw)
        with pytest.raises(qb.QsdpError) as e:
            qb.qsdp_fused_adamw_step(z, z.clone(), z.clone(), z.clone(), **a)
        assert e.value.status == qb.QSDP_EINVAL


@pytest.mark.parametrize("bucket", [32, 96, 128, 512, 1024, 2048, 4096])
@pytest.mark.parametrize("wbits,gbits,delta,flags", [(8, 4, 0.0, 0), (6, 3, 0.0, 0), (5, 7, 0.0, 1), (8, 4, 2.0**-10, 0),
                                                     (4, 2, 0.0, 4), (1, 8, 0.0, 2)])
def test_adamw_steps_on_code_resident_weights(wbits, gbits, delta, flags, bucket):
    """Three AdamW steps with the weights held only as codes + meta: every step equals the oracle's decode
    followed by its AdamW step with code output (codes, meta, moments, saturation count bit for bit)."""
    n = 6 * bucket + bucket // 2 + 7
    x, g = synth(n, 1150 + wbits + gbits)
    hc, hm_, _ = ref.quantize_weight(x, wbits, bucket, delta, 77)
    codes = torch.from_numpy(hc.view(np.int32)).to(DEV)
    meta = torch.from_numpy(hm_.reshape(-1)).to(DEV)
    md = torch.zeros(n, dtype=torch.float32, device=DEV)
    vd = torch.zeros(n, dtype=torch.float32, device=DEV)
    hmom, hvar = np.zeros(n, np.float32), np.zeros(n, np.float32)
    for t in range(1, 4):
        gt = (g * np.float32(1 + 0.1 * t)).astype(np.float32)
        bc1, bc2 = 1 - 0.9**t, 1 - 0.95**t
        sat = torch.zeros(1, dtype=torch.int64, device=DEV)
        qb.qsdp_fused_adamw_step_codes(codes, meta, torch.from_numpy(gt).to(DEV), md, vd, bias1=bc1, bias2=bc2,
                                       wbits=wbits, gbits=gbits, bucket=bucket, delta=delta, seed=t, index_offset=16,
                                       flags=flags, n_saturated=sat, **HYPER)
        xt = ref.dequantize(hc, hm_, n, wbits, bucket)
        _, hmom, hvar, hc, hm_, ws = ref.fused_adamw_step(xt, gt, hmom, hvar, bias1=bc1, bias2=bc2, wbits=wbits,
                                                          gbits=gbits, bucket=bucket, delta=delta, seed=t,
                                                          index_offset=16, flags=flags, emit_codes=True, **HYPER)
        assert np.array_equal(np_u32(codes), hc) and np.array_equal(np_u32(meta), hm_.view(np.uint32).reshape(-1)), t
        assert bits_equal(np_f32(md), hmom) and bits_equal(np_f32(vd), hvar), t
        assert int(sat) == ws


def test_code_resident_adamw_rejects_keep_master():
    n, B = 2048, 1024
    codes, meta = qb.alloc_packed(n, 8, B, DEV)
    z = torch.zeros(n, dtype=torch.float32, device=DEV)
    with pytest.raises(qb.QsdpError):
        qb.qsdp_fused_adamw_step_codes(codes, meta.reshape(-1), z, z.clone(), z.clone(), bias1=0.1, bias2=0.05,
                                       wbits=8, gbits=4, bucket=B, delta=0.0, seed=0,
                                       flags=qb.QSDP_FLAG_KEEP_MASTER, **HYPER)
