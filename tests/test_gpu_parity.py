"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle on the same
seeded inputs. Packed codes, meta-data and saturation counts must be bit-exact; decoded and
stepped fp32 values must agree to 1e-6 relative (they are expected to be bit-exact too, and
the tests record whether they are); bf16 outputs to 1 ulp."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2302_02390_amd import binding as qb
from gpu_util import (DEV, bits_equal, gpu_dequantize, gpu_fused_step, gpu_quantize_grad,
                      gpu_quantize_weight, np_f32, np_u32, synth)

pytestmark = pytest.mark.gpu

BUCKETS = [32, 96, 128, 256, 512, 1024, 2048, 4096, 8192]
REL = 1e-6


def close(a, b):
    a = np.asarray(a, np.float64)
    b = np.asarray(b, np.float64)
    return np.all(np.abs(a - b) <= REL * np.maximum(np.abs(b), 1e-30))


@pytest.fixture(scope="module", autouse=True)
def _oracle_threads():
    ref.set_threads(8)
    yield
    ref.set_threads(1)


def _n_for(bucket, k=9, tail=True):
    return k * bucket + (bucket // 2 + 5 if tail else 0)


@pytest.mark.parametrize("bucket", BUCKETS)
@pytest.mark.parametrize("bits", range(1, 9))
def test_quantize_grad_bit_exact(bits, bucket):
    n = _n_for(bucket)
    _, g = synth(n, 1000 + bits)
    codes, meta = gpu_quantize_grad(g, bits, bucket, seed=bits)
    want_c, want_m = ref.quantize_grad(g, bits, bucket, seed=bits)
    assert np.array_equal(np_u32(meta), want_m.view(np.uint32).reshape(-1))
    assert np.array_equal(np_u32(codes), want_c)


@pytest.mark.parametrize("bucket", BUCKETS)
@pytest.mark.parametrize("bits", range(1, 9))
def test_quantize_weight_minmax_bit_exact(bits, bucket):
    n = _n_for(bucket)
    x, _ = synth(n, 2000 + bits)
    codes, meta, sat = gpu_quantize_weight(x, bits, bucket, 0.0, seed=bits + 3)
    want_c, want_m, want_sat = ref.quantize_weight(x, bits, bucket, 0.0, seed=bits + 3)
    assert np.array_equal(np_u32(meta), want_m.view(np.uint32).reshape(-1))
    assert np.array_equal(np_u32(codes), want_c)
    assert sat == want_sat == 0


@pytest.mark.parametrize("bucket", [96, 128, 512, 1024, 4096])
@pytest.mark.parametrize("bits,delta", [(4, 2.0**-6), (6, 2.0**-8), (8, 2.0**-10), (4, 2.0**-8),
                                        (8, 1.3e-4), (3, 0.004)])
def test_quantize_weight_lattice_bit_exact(bits, delta, bucket):
    n = _n_for(bucket)
    x, _ = synth(n, 3000 + bits)
    codes, meta, sat = gpu_quantize_weight(x, bits, bucket, delta, seed=11)
    want_c, want_m, want_sat = ref.quantize_weight(x, bits, bucket, delta, seed=11)
    assert np.array_equal(np_u32(meta), want_m.view(np.uint32).reshape(-1))
    assert np.array_equal(np_u32(codes), want_c)
    assert sat == want_sat


@pytest.mark.parametrize("bucket", [32, 128, 1024, 4096])
@pytest.mark.parametrize("bits", range(1, 9))
def test_dequantize_fp32_and_bf16(bits, bucket):
    n = _n_for(bucket, k=5)
    x, _ = synth(n, 4000 + bits)
    want_c, want_m, _ = ref.quantize_weight(x, bits, bucket, 0.0, seed=2)
    codes = torch.from_numpy(want_c.view(np.int32)).to(DEV)
    meta = torch.from_numpy(want_m.reshape(-1)).to(DEV)
    out = gpu_dequantize(codes, meta, n, bits, bucket, torch.float32)
    want = ref.dequantize(want_c, want_m, n, bits, bucket, ref.F32)
    assert close(np_f32(out), want)
    assert bits_equal(np_f32(out), want)
    outh = gpu_dequantize(codes, meta, n, bits, bucket, torch.bfloat16)
    wanth = ref.dequantize(want_c, want_m, n, bits, bucket, ref.BF16)
    got = outh.view(torch.int16).cpu().numpy().view(np.uint16).astype(np.int64)
    assert np.all(np.abs(got - wanth.astype(np.int64)) <= 1)
    assert np.array_equal(got, wanth.astype(np.int64))


@pytest.mark.parametrize("bucket", BUCKETS)
@pytest.mark.parametrize("wbits,gbits,delta", [(8, 8, 0.0), (8, 4, 0.0), (6, 3, 0.0), (4, 2, 0.0),
                                               (5, 7, 0.0), (8, 4, 2.0**-10), (4, 2, 2.0**-6),
                                               (6, 6, 3e-4)])
def test_fused_step(wbits, gbits, delta, bucket):
    n = _n_for(bucket)
    x, g = synth(n, 5000 + wbits + gbits)
    for emit in (False, True):
        out, wc, wm, sat = gpu_fused_step(x, g, 1e-3, wbits, gbits, bucket, delta, seed=4, emit=emit)
        want, want_c, want_m, want_sat = ref.fused_step(x, g, 1e-3, wbits, gbits, bucket, delta, 4,
                                                        emit_codes=emit)
        assert close(np_f32(out), want)
        assert bits_equal(np_f32(out), want)
        assert sat == want_sat
        if emit:
            assert np.array_equal(np_u32(wm), want_m.view(np.uint32).reshape(-1))
            assert np.array_equal(np_u32(wc), want_c)


@pytest.mark.parametrize("n", [1, 3, 7, 8, 9, 31, 33, 1023, 1024, 1025, 1027, 2048 + 6])
def test_ragged_sizes(n):
    x, g = synth(n, 6000 + n)
    for bucket in (32, 1024):
        codes, meta = gpu_quantize_grad(g, 8, bucket, seed=1)
        wc, wm = ref.quantize_grad(g, 8, bucket, seed=1)
        assert np.array_equal(np_u32(codes), wc) and np.array_equal(np_u32(meta), wm.view(np.uint32).reshape(-1))
        out = gpu_dequantize(codes, meta.reshape(-1), n, 8, bucket, torch.float32)
        assert bits_equal(np_f32(out), ref.dequantize(wc, wm, n, 8, bucket))
        out, _, _, _ = gpu_fused_step(x, g, 1e-3, 8, 4, bucket, 0.0, seed=2)
        want, _, _, _ = ref.fused_step(x, g, 1e-3, 8, 4, bucket, 0.0, 2)
        assert bits_equal(np_f32(out), want)


def test_degenerate_buckets():
    B = 1024
    x = np.concatenate([np.full(B, 0.25, np.float32),                   # constant
                        np.zeros(B, np.float32),                        # all zero
                        np.where(np.arange(B) % 2 == 0, 0.0, -0.0).astype(np.float32),  # signed zeros
                        np.full(B, 1e-42, np.float32),                  # subnormal constant
                        (np.arange(B) * 1e-45).astype(np.float32),      # subnormal range: L/range overflows
                        np.linspace(-1, 1, B, dtype=np.float32),
                        np.full(100, -3.0, np.float32)])                # short constant tail
    g = np.roll(x, 17).astype(np.float32)
    for bits in (1, 4, 8):
        codes, meta = gpu_quantize_grad(x, bits, B, seed=0)
        wc, wm = ref.quantize_grad(x, bits, B, seed=0)
        assert np.array_equal(np_u32(codes), wc) and np.array_equal(np_u32(meta), wm.view(np.uint32).reshape(-1))
        codes, meta, _ = gpu_quantize_weight(x, bits, B, 0.0, seed=0)
        wc, wm, _ = ref.quantize_weight(x, bits, B, 0.0, seed=0)
        assert np.array_equal(np_u32(codes), wc) and np.array_equal(np_u32(meta), wm.view(np.uint32).reshape(-1))
        out, _, _, _ = gpu_fused_step(x, g, 0.5, bits, bits, B, 0.0, seed=3)
        want, _, _, _ = ref.fused_step(x, g, 0.5, bits, bits, B, 0.0, 3)
        assert bits_equal(np_f32(out), want)


def test_shard_with_index_offset_matches_whole():
    B, bits = 1024, 4
    n = 64 * B
    x, g = synth(n, 7000)
    whole_c, whole_m = gpu_quantize_grad(g, bits, B, seed=5)
    whole_x, _, _, _ = gpu_fused_step(x, g, 1e-3, 8, bits, B, 0.0, seed=5)
    wpb = B * bits // 32
    for lo, hi in [(0, 16), (16, 48), (48, 64)]:
        c, m = gpu_quantize_grad(g[lo * B:hi * B], bits, B, seed=5, index_offset=lo * B)
        assert torch.equal(c, whole_c[lo * wpb:hi * wpb]) and torch.equal(m, whole_m[2 * lo:2 * hi])
        xs, _, _, _ = gpu_fused_step(x[lo * B:hi * B], g[lo * B:hi * B], 1e-3, 8, bits, B, 0.0, seed=5,
                                     index_offset=lo * B)
        assert torch.equal(xs, whole_x[lo * B:hi * B])


def test_deterministic_across_runs():
    x, g = synth(300 * 1024 + 77, 8000)
    first = None
    for _ in range(3):
        out, wc, wm, _ = gpu_fused_step(x, g, 1e-3, 8, 4, 1024, 0.0, seed=6, emit=True)
        cur = (out.clone(), wc.clone(), wm.clone())
        if first is None:
            first = cur
        else:
            assert all(torch.equal(a, b) for a, b in zip(first, cur))


def test_error_codes_launch_nothing():
    g = torch.zeros(2048, dtype=torch.float32, device=DEV)
    codes, meta = qb.alloc_packed(2048, 8, 1024, DEV)
    meta = meta.reshape(-1)
    for bits, bucket in [(0, 1024), (9, 1024), (8, 100), (8, 16), (8, 16384)]:
        with pytest.raises(qb.QsdpError) as e:
            qb.qsdp_quantize_grad(g, bits, bucket, 0, 0, codes, meta)
        assert e.value.status == qb.QSDP_EINVAL
    with pytest.raises(qb.QsdpError) as e:
        qb.qsdp_quantize_grad(g, 8, 1024, 0, 4, codes, meta)
    assert e.value.status == qb.QSDP_EINVAL
    with pytest.raises(qb.QsdpError) as e:
        qb.qsdp_quantize_grad(g[1:1025], 8, 1024, 0, 0, codes, meta)
    assert e.value.status == qb.QSDP_EALIGN
    with pytest.raises(qb.QsdpError) as e:
        qb.qsdp_quantize_weight(g, 8, 1024, -1.0, 0, codes, meta)
    assert e.value.status == qb.QSDP_EINVAL
    with pytest.raises(qb.QsdpError) as e:
        qb.qsdp_fused_step(g, g.clone(), 1e-3, 8, 4, 1024, 0.0, 0, 0, codes, None)
    assert e.value.status == qb.QSDP_EINVAL
    with pytest.raises(qb.QsdpError) as e:
        qb.qsdp_fused_step(g, g.clone(), float("nan"), 8, 4, 1024, 0.0, 0)
    assert e.value.status == qb.QSDP_EINVAL
    torch.cuda.synchronize()


def test_config1_all_entry_points():
    """The small benchmark configuration: 2^20 elements, W8 G8, bucket 1024, lr 1e-3, seed 0."""
    n, B = 1 << 20, 1024
    from paper_2302_02390_amd import workloads
    x = workloads.weights(n, 1235).numpy()
    g = workloads.grads_normal(n, 1236).numpy()
    codes, meta = gpu_quantize_grad(g, 8, B, seed=0)
    wc, wm = ref.quantize_grad(g, 8, B, seed=0)
    assert np.array_equal(np_u32(codes), wc) and np.array_equal(np_u32(meta), wm.view(np.uint32).reshape(-1))
    codes, meta, _ = gpu_quantize_weight(x, 8, B, 0.0, seed=0)
    wc, wm, _ = ref.quantize_weight(x, 8, B, 0.0, seed=0)
    assert np.array_equal(np_u32(codes), wc) and np.array_equal(np_u32(meta), wm.view(np.uint32).reshape(-1))
    out = gpu_dequantize(codes, meta.reshape(-1), n, 8, B, torch.float32)
    assert bits_equal(np_f32(out), ref.dequantize(wc, wm, n, 8, B))
    out, _, _, _ = gpu_fused_step(x, g, 1e-3, 8, 8, B, 0.0, seed=0)
    want, _, _, _ = ref.fused_step(x, g, 1e-3, 8, 8, B, 0.0, 0)
    assert close(np_f32(out), want) and bits_equal(np_f32(out), want)


def test_non_finite_inputs_do_not_disturb_their_neighbours():
    """Non-finite inputs are a precondition violation with unspecified codes, but memory addresses
    never depend on the data: the call completes, buckets without such values are unaffected."""
    B = 1024
    n = 8 * B
    x, g = synth(n, 9100)
    gbad, xbad = g.copy(), x.copy()
    gbad[3 * B + 5] = np.nan
    gbad[5 * B + 7] = np.inf
    xbad[3 * B + 9] = -np.inf
    clean = [0, 1, 2, 4, 6, 7]
    codes, meta = gpu_quantize_grad(gbad, 4, B, seed=1)
    wc, wm = ref.quantize_grad(g, 4, B, seed=1)
    wpb = B * 4 // 32
    got = np_u32(codes).reshape(8, wpb)
    assert np.array_equal(got[clean], wc.reshape(8, wpb)[clean])
    out, _, _, _ = gpu_fused_step(xbad, gbad, 1e-3, 8, 4, B, 0.0, seed=2)
    want, _, _, _ = ref.fused_step(x, g, 1e-3, 8, 4, B, 0.0, 2)
    assert bits_equal(np_f32(out).reshape(8, B)[clean], want.reshape(8, B)[clean])
    lv = torch.from_numpy(ref.levels_uniform(4)).to(DEV)
    c2, m2 = qb.alloc_packed(n, 4, B, DEV)
    qb.qsdp_quantize_levels(torch.from_numpy(xbad).to(DEV), 4, B, lv, c2, m2.reshape(-1))
    o2 = torch.empty(n, dtype=torch.float32, device=DEV)
    qb.qsdp_dequantize_levels(c2, m2.reshape(-1), n, 4, B, lv, o2)
    torch.cuda.synchronize()
    wc2, wm2 = ref.quantize_levels(x, 4, B, ref.levels_uniform(4))
    assert np.array_equal(np_u32(c2).reshape(8, wpb)[clean], wc2.reshape(8, wpb)[clean])
