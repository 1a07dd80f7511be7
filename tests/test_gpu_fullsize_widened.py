"""GPU parity of the widened entry points at the benchmark's size and launch configuration (the
1.3B vector, bucket 1024): the oracle recomputes a sample of buckets one by one."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2302_02390_amd import binding as qb
from paper_2302_02390_amd import workloads as wl
from gpu_util import DEV, bits_equal, gather_rows, sample_bucket_ids

pytestmark = pytest.mark.gpu

B = 1024


def u32(a):
    return np.ascontiguousarray(a).view(np.uint32)


@pytest.fixture(scope="module")
def gpt1p3b():
    n = wl.model_numel(wl.GPT_1P3B)
    x = wl.weights(n, 1240, DEV)
    g = wl.grads_student_t3(n, 1241, DEV)
    torch.cuda.synchronize()
    yield n, x, g
    del x, g
    torch.cuda.empty_cache()


@pytest.mark.parametrize("flags", [0, qb.QSDP_FLAG_GRAD_SHIFT])
def test_code_resident_steps_on_the_full_vector(gpt1p3b, flags):
    """Three steps with the weights held as 8-bit codes (4-bit gradients), seed = step index."""
    n, x0, g = gpt1p3b
    ids = sample_bucket_ids(n // B, 150, 21)
    wpb = B * 8 // 32
    wc, wm = qb.alloc_packed(n, 8, B, DEV)
    qb.qsdp_quantize_weight(x0, 8, B, 0.0, 99, wc, wm.reshape(-1))
    gb = gather_rows(g, ids, B)
    for step in range(3):
        c_before = u32(gather_rows(wc, ids, wpb))
        m_before = gather_rows(wm.reshape(-1), ids, 2)
        qb.qsdp_fused_step_codes(wc, wm.reshape(-1), g, 1e-3, 8, 4, B, 0.0, step, 0, None, flags)
        c_after = u32(gather_rows(wc, ids, wpb))
        m_after = u32(gather_rows(wm.reshape(-1), ids, 2))
        for r, j in enumerate(ids):
            want_c, want_m, _ = ref.fused_step_codes(c_before[r], m_before[r], gb[r], 1e-3, 8, 4, B, 0.0, step,
                                                     index_offset=int(j) * B, flags=flags)
            assert np.array_equal(c_after[r], want_c), (step, int(j))
            assert np.array_equal(m_after[r], u32(want_m).reshape(-1)), (step, int(j))


def test_adamw_steps_on_the_full_vector(gpt1p3b):
    """Two AdamW steps (the experiments' betas and eps, weight decay 0.1), W8 G4."""
    n, x0, g = gpt1p3b
    ids = sample_bucket_ids(n // B, 120, 22)
    x = x0.clone()
    m = torch.zeros_like(x)
    v = torch.zeros_like(x)
    gb = gather_rows(g, ids, B)
    b1, b2, eps, wd, lr = 0.9, 0.95, 1e-8, 0.1, 2e-4
    for step in range(2):
        xb, mb, vb = gather_rows(x, ids, B), gather_rows(m, ids, B), gather_rows(v, ids, B)
        c1, c2 = 1.0 - b1 ** (step + 1), 1.0 - b2 ** (step + 1)
        qb.qsdp_fused_adamw_step(x, g, m, v, lr, b1, b2, eps, wd, c1, c2, 8, 4, B, 0.0, step)
        xa, ma, va = gather_rows(x, ids, B), gather_rows(m, ids, B), gather_rows(v, ids, B)
        for r, j in enumerate(ids):
            wx, wm_, wv, _, _, _ = ref.fused_adamw_step(xb[r], gb[r], mb[r], vb[r], lr, b1, b2, eps, wd, c1, c2,
                                                        8, 4, B, 0.0, step, index_offset=int(j) * B)
            assert bits_equal(xa[r], wx) and bits_equal(ma[r], wm_) and bits_equal(va[r], wv), (step, int(j))
    del x, m, v
    torch.cuda.empty_cache()


def test_decode_and_sum_of_eight_peers_on_a_shard(gpt1p3b):
    """The receive side of the gradient exchange as the benchmark times it: 8 peers' 4-bit slices of
    one GPU's 1/8 shard (164,464,640 elements), averaged."""
    n, _, g = gpt1p3b
    peers = 8
    m = (n // peers) // B * B
    nbm = m // B
    wpb = B * 4 // 32
    pc = torch.empty((peers, nbm * wpb), dtype=torch.int32, device=DEV)
    pm = torch.empty((peers, nbm * 2), dtype=torch.float32, device=DEV)
    for p in range(peers):
        gp = g[p * m:(p + 1) * m]  # peer p's gradient for this shard: a different slice of g per peer
        qb.qsdp_quantize_grad(gp, 4, B, 100 + p, 0, pc[p], pm[p])
    out = torch.empty(m, dtype=torch.float32, device=DEV)
    qb.qsdp_dequantize_add(pc, pm, peers, m, 4, B, 1.0 / peers, out)
    ids = sample_bucket_ids(nbm, 200, 23)
    got = gather_rows(out, ids, B)
    idx = torch.from_numpy(ids).to(DEV)
    crow = pc.view(peers, nbm, wpb).index_select(1, idx).cpu().numpy().view(np.uint32)   # [peers, k, wpb]
    mrow = pm.view(peers, nbm, 2).index_select(1, idx).cpu().numpy()                    # [peers, k, 2]
    for r in range(len(ids)):
        want = ref.dequantize_add(crow[:, r, :], mrow[:, r, :], peers, B, 4, B, 1.0 / peers)
        assert bits_equal(got[r], want), int(ids[r])


@pytest.mark.parametrize("bits", [3, 4])
def test_learned_level_codec_on_the_full_vector(gpt1p3b, bits):
    """Nearest-level encoding against a fitted (non-uniform) table and its decode to bf16."""
    n, x0, _ = gpt1p3b
    start = ref.levels_uniform(bits)
    levels_np = ref.fit_levels(x0[:256 * B].cpu().numpy(), bits, B, 0.01, start)
    levels = torch.from_numpy(levels_np).to(DEV)
    codes, meta = qb.alloc_packed(n, bits, B, DEV)
    qb.qsdp_quantize_levels(x0, bits, B, levels, codes, meta.reshape(-1))
    out = torch.empty(n, dtype=torch.bfloat16, device=DEV)
    qb.qsdp_dequantize_levels(codes, meta.reshape(-1), n, bits, B, levels, out)
    ids = sample_bucket_ids(n // B, 200, 24 + bits)
    wpb = B * bits // 32
    rows = gather_rows(x0, ids, B)
    crow = u32(gather_rows(codes, ids, wpb))
    mrow = gather_rows(meta.reshape(-1), ids, 2)
    orow = gather_rows(out.view(torch.int16), ids, B).view(np.uint16)
    for r, j in enumerate(ids):
        wc, wm_ = ref.quantize_levels(rows[r], bits, B, levels_np)
        assert np.array_equal(crow[r], wc), int(j)
        assert np.array_equal(u32(mrow[r]), u32(wm_).reshape(-1)), int(j)
        assert np.array_equal(orow[r], ref.dequantize_levels(wc, wm_, B, bits, B, levels_np, ref.BF16)), int(j)


def test_segmented_codec_on_the_1p3b_layer_list(gpt1p3b):
    """All 292 layer tensors of the 1.3B model in one segmented encode and one segmented decode;
    every small tensor and a sample of the buckets of the large ones go through the oracle."""
    n, x0, _ = gpt1p3b
    sizes = [s for _, s in wl.model_tensors(wl.GPT_1P3B)]
    assert sum(sizes) == n
    segs = qb.Segments(sizes, B, DEV)
    codes, meta = segs.alloc_packed(8)
    qb.qsdp_quantize_weight_segmented(x0, segs, 8, 0.0, 31, codes, meta.reshape(-1))
    out = torch.full((n,), float("nan"), dtype=torch.float32, device=DEV)
    qb.qsdp_dequantize_segmented(codes, meta.reshape(-1), segs, 8, out)
    assert not bool(torch.isnan(out).any())          # every element of every tensor was written
    wpb = B * 8 // 32
    rng = np.random.default_rng(5)
    for t, (off, size, fb) in enumerate(segs.host.tolist()):
        nb = -(-size // B)
        local = range(nb) if nb <= 4 else sorted(set(rng.choice(nb, size=3, replace=False).tolist()) | {0, nb - 1})
        if nb > 4 and t % 6:
            continue
        for lb in local:
            lo, hi = off + lb * B, min(off + (lb + 1) * B, off + size)
            xs = x0[lo:hi].cpu().numpy()
            wc, wm_, _ = ref.quantize_weight(xs, 8, B, 0.0, 31)
            j = fb + lb
            assert np.array_equal(u32(codes[j * wpb:(j + 1) * wpb].cpu().numpy()), wc), (t, lb)
            assert np.array_equal(u32(meta[j].cpu().numpy()), u32(wm_).reshape(-1)), (t, lb)
            assert bits_equal(out[lo:hi].cpu().numpy(), ref.dequantize(wc, wm_, hi - lo, 8, B)), (t, lb)


@pytest.mark.parametrize("dtype", [torch.float16, torch.bfloat16])
def test_16bit_gradient_steps_on_the_full_vector(gpt1p3b, dtype):
    """Two fused steps (W8 G4, seed = step index) and the 4-bit gradient encoding with the gradient handed over
    in 16 bits; the oracle gets the sampled buckets widened by torch on the CPU."""
    n, x0, g = gpt1p3b
    ids = sample_bucket_ids(n // B, 150, 24)
    g16 = g.to(dtype)
    gh = g16.view(torch.int16)
    wide = torch.from_numpy(gather_rows(gh, ids, B)).view(dtype).float().numpy()
    x = x0.clone()
    for step in range(2):
        xb = gather_rows(x, ids, B)
        qb.qsdp_fused_step_g16(x, g16, 1e-3, 8, 4, B, 0.0, step)
        xa = gather_rows(x, ids, B)
        for r, j in enumerate(ids):
            want, _, _, _ = ref.fused_step(xb[r], wide[r], 1e-3, 8, 4, B, 0.0, step, index_offset=int(j) * B)
            assert bits_equal(xa[r], want), (step, int(j))
    del x
    gc, gm = qb.alloc_packed(n, 4, B, DEV)
    qb.qsdp_quantize_grad_g16(g16, 4, B, 5, 0, gc, gm.reshape(-1))
    cs, ms = u32(gather_rows(gc, ids, B * 4 // 32)), u32(gather_rows(gm.reshape(-1), ids, 2))
    for r, j in enumerate(ids):
        want_c, want_m = ref.quantize_grad(wide[r], 4, B, 5, index_offset=int(j) * B)
        assert np.array_equal(cs[r], want_c) and np.array_equal(ms[r], u32(want_m).reshape(-1)), int(j)
    del g16, gc, gm
    torch.cuda.empty_cache()
