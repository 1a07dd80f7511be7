"""GPU parity of the widened entry points at the benchmark's size and launch configuration (the
1.3B vector, bucket 1024): every output element against the bucket-parallel oracle, which runs its
own chain of steps on host copies of the same seeded inputs."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2302_02390_amd import binding as qb
from paper_2302_02390_amd import workloads as wl
from gpu_util import DEV, ORACLE_THREADS, first_mismatch

pytestmark = pytest.mark.gpu

B = 1024


def same_words(dev, host):
    """A device tensor against a host array of the same item size, bit for bit."""
    host = np.ascontiguousarray(host).reshape(-1)
    kind = {2: np.int16, 4: np.int32}[host.dtype.itemsize]
    return first_mismatch(dev.reshape(-1), host.view(kind)) == -1


def same_packed(codes, meta, want_codes, want_meta):
    return same_words(codes, want_codes) and same_words(meta, want_meta)


@pytest.fixture(scope="module")
def gpt1p3b():
    n = wl.model_numel(wl.GPT_1P3B)
    x = wl.weights(n, 1240, DEV)
    g = wl.grads_student_t3(n, 1241, DEV)
    torch.cuda.synchronize()
    x_np, g_np = x.cpu().numpy(), g.cpu().numpy()
    ref.set_threads(ORACLE_THREADS)
    yield {"n": n, "x": x, "g": g, "x_np": x_np, "g_np": g_np}
    ref.set_threads(1)
    del x, g
    torch.cuda.empty_cache()


@pytest.mark.parametrize("flags", [0, qb.QSDP_FLAG_GRAD_SHIFT])
def test_code_resident_steps_on_the_full_vector(gpt1p3b, flags):
    """Two steps with the weights held as 8-bit codes (4-bit gradients), seed = step index: codes and
    meta of the whole vector after the encoding and after each step."""
    n, x0, g, x_np, g_np = (gpt1p3b[k] for k in ("n", "x", "g", "x_np", "g_np"))
    wc, wm = qb.alloc_packed(n, 8, B, DEV)
    qb.qsdp_quantize_weight(x0, 8, B, 0.0, 99, wc, wm.reshape(-1))
    want_c, want_m, _ = ref.quantize_weight(x_np, 8, B, 0.0, 99)
    assert same_packed(wc, wm, want_c, want_m)
    for step in range(2):
        qb.qsdp_fused_step_codes(wc, wm.reshape(-1), g, 1e-3, 8, 4, B, 0.0, step, 0, None, flags)
        want_c, want_m, _ = ref.fused_step_codes(want_c, want_m, g_np, 1e-3, 8, 4, B, 0.0, step, flags=flags)
        assert same_packed(wc, wm, want_c, want_m), step
    del wc, wm
    torch.cuda.empty_cache()


def test_adamw_steps_on_the_full_vector(gpt1p3b):
    """Two AdamW steps (the experiments' betas and eps, weight decay 0.1), W8 G4: x, m and v of the
    whole vector after each step."""
    n, x0, g, x_np, g_np = (gpt1p3b[k] for k in ("n", "x", "g", "x_np", "g_np"))
    x = x0.clone()
    m = torch.zeros_like(x)
    v = torch.zeros_like(x)
    wx, wm_, wv = x_np, np.zeros(n, np.float32), np.zeros(n, np.float32)
    b1, b2, eps, wd, lr = 0.9, 0.95, 1e-8, 0.1, 2e-4
    for step in range(2):
        c1, c2 = 1.0 - b1 ** (step + 1), 1.0 - b2 ** (step + 1)
        qb.qsdp_fused_adamw_step(x, g, m, v, lr, b1, b2, eps, wd, c1, c2, 8, 4, B, 0.0, step)
        wx, wm_, wv, _, _, _ = ref.fused_adamw_step(wx, g_np, wm_, wv, lr, b1, b2, eps, wd, c1, c2, 8, 4, B, 0.0, step)
        assert same_words(x, wx) and same_words(m, wm_) and same_words(v, wv), step
    del x, m, v
    torch.cuda.empty_cache()


def test_receive_side_of_eight_peers_on_a_shard(gpt1p3b):
    """The receive side of the gradient exchange as the benchmark times it: 8 peers' 4-bit slices of
    one GPU's 1/8 shard (164,464,640 elements). Decode-and-average, the fused receive-side step
    (W8 codes out) and the receive-side AdamW step, every element of the shard."""
    n, x0, g, x_np, g_np = (gpt1p3b[k] for k in ("n", "x", "g", "x_np", "g_np"))
    peers = 8
    m = (n // peers) // B * B
    nbm = m // B
    wpb = B * 4 // 32
    pc = torch.empty((peers, nbm * wpb), dtype=torch.int32, device=DEV)
    pm = torch.empty((peers, nbm * 2), dtype=torch.float32, device=DEV)
    want_pc, want_pm = [], []
    for p in range(peers):
        sl = slice(p * m, (p + 1) * m)   # peer p's gradient for this shard: a different slice of g per peer
        qb.qsdp_quantize_grad(g[sl], 4, B, 100 + p, 0, pc[p], pm[p])
        c, mm = ref.quantize_grad(g_np[sl], 4, B, 100 + p)
        want_pc.append(c); want_pm.append(mm.reshape(-1))
    want_pc, want_pm = np.stack(want_pc), np.stack(want_pm)
    assert same_packed(pc, pm, want_pc, want_pm)

    out = torch.empty(m, dtype=torch.float32, device=DEV)
    qb.qsdp_dequantize_add(pc, pm, peers, m, 4, B, 1.0 / peers, out)
    assert same_words(out, ref.dequantize_add(want_pc, want_pm, peers, m, 4, B, 1.0 / peers))
    del out

    x = x0[:m].clone()
    wc, wm = qb.alloc_packed(m, 8, B, DEV)
    qb.qsdp_recv_step(x, pc, pm, peers, 1.0 / peers, 1e-3, 8, 4, B, 0.0, 7, 0, wc, wm.reshape(-1))
    wx, want_c, want_m, _ = ref.recv_step(x_np[:m], want_pc, want_pm, peers, 1.0 / peers, 1e-3, 8, 4, B, 0.0, 7,
                                          emit_codes=True)
    assert same_words(x, wx) and same_packed(wc, wm, want_c, want_m)

    x = x0[:m].clone()
    mo = torch.zeros_like(x)
    vo = torch.zeros_like(x)
    b1, b2, eps, wd, lr = 0.9, 0.95, 1e-8, 0.1, 2e-4
    qb.qsdp_recv_adamw_step(x, mo, vo, pc, pm, peers, 1.0 / peers, lr, b1, b2, eps, wd, 1.0 - b1, 1.0 - b2, 8, 4, B,
                            0.0, 8, qb.QSDP_FLAG_KEEP_MASTER, wc, wm.reshape(-1))
    wx, wmo, wvo, want_c, want_m, _ = ref.recv_adamw_step(
        x_np[:m], np.zeros(m, np.float32), np.zeros(m, np.float32), want_pc, want_pm, peers, 1.0 / peers, lr, b1, b2,
        eps, wd, 1.0 - b1, 1.0 - b2, 8, 4, B, 0.0, 8, flags=qb.QSDP_FLAG_KEEP_MASTER, emit_codes=True)
    assert same_words(x, wx) and same_words(mo, wmo) and same_words(vo, wvo)
    assert same_packed(wc, wm, want_c, want_m)
    del x, mo, vo, wc, wm, pc, pm
    torch.cuda.empty_cache()


@pytest.mark.parametrize("bits", [3, 4])
def test_learned_level_codec_on_the_full_vector(gpt1p3b, bits):
    """Nearest-level and coin-flip encoding against a fitted (non-uniform) table, and the decode of
    the nearest-level codes to bf16: every code word, meta entry and decoded element."""
    n, x0, x_np = (gpt1p3b[k] for k in ("n", "x", "x_np"))
    levels_np = ref.fit_levels(x_np[:256 * B], bits, B, 0.01, ref.levels_uniform(bits))
    assert np.unique(levels_np).size == 1 << bits and not np.array_equal(levels_np, ref.levels_uniform(bits))
    levels = torch.from_numpy(levels_np).to(DEV)
    codes, meta = qb.alloc_packed(n, bits, B, DEV)
    qb.qsdp_quantize_levels(x0, bits, B, levels, codes, meta.reshape(-1))
    want_c, want_m = ref.quantize_levels(x_np, bits, B, levels_np)
    assert same_packed(codes, meta, want_c, want_m)
    out = torch.empty(n, dtype=torch.bfloat16, device=DEV)
    qb.qsdp_dequantize_levels(codes, meta.reshape(-1), n, bits, B, levels, out)
    assert same_words(out, ref.dequantize_levels(want_c, want_m, n, bits, B, levels_np, ref.BF16))
    del out
    qb.qsdp_quantize_levels_stochastic(x0, bits, B, levels, 11, 0, codes, meta.reshape(-1))
    want_c, want_m = ref.quantize_levels_stochastic(x_np, bits, B, levels_np, 11)
    assert same_packed(codes, meta, want_c, want_m)
    del codes, meta
    torch.cuda.empty_cache()


def test_per_layer_level_tables_on_the_1p3b_layer_list(gpt1p3b):
    """Section 5.2's per-layer use: all 292 layer tensors of the 1.3B model, each with a level table
    of its own (fitted by the oracle on the tensor's first buckets; the uniform table for the small
    tensors), encoded in one launch: W5 to the nearest level, G4 by coin flip, and the W5 codes decoded
    to bf16. The oracle encodes tensor by tensor; every word of the whole model is compared."""
    n, x0, g, x_np, g_np = (gpt1p3b[k] for k in ("n", "x", "g", "x_np", "g_np"))
    sizes = [s for _, s in wl.model_tensors(wl.GPT_1P3B)]
    assert sum(sizes) == n and len(sizes) == 292
    segs = qb.Segments(sizes, B, DEV)
    for bits, src, src_np, stochastic in ((5, x0, x_np, False), (4, g, g_np, True)):
        tables = []
        off = 0
        for s in sizes:
            start = ref.levels_uniform(bits)
            tables.append(ref.fit_levels(src_np[off:off + s], bits, B, 0.01, start, 32) if s > 100_000 else start)
            off += s
        tables = np.stack(tables)
        lvd = torch.from_numpy(tables).to(DEV)
        codes, meta = segs.alloc_packed(bits)
        qb.qsdp_quantize_levels_segmented(src, segs, bits, lvd, codes, meta.reshape(-1), stochastic, seed=13)
        want_c, want_m, want_o = [], [], []
        off = 0
        for t, s in enumerate(sizes):
            if stochastic:
                c, m = ref.quantize_levels_stochastic(src_np[off:off + s], bits, B, tables[t], 13, index_offset=off)
            else:
                c, m = ref.quantize_levels(src_np[off:off + s], bits, B, tables[t])
                want_o.append(ref.dequantize_levels(c, m, s, bits, B, tables[t], ref.BF16))
            want_c.append(c); want_m.append(m.reshape(-1))
            off += s
        assert same_packed(codes, meta, np.concatenate(want_c), np.concatenate(want_m)), bits
        if not stochastic:
            out = torch.empty(n, dtype=torch.bfloat16, device=DEV)
            qb.qsdp_dequantize_levels_segmented(codes, meta.reshape(-1), segs, bits, lvd, out)
            assert same_words(out, np.concatenate(want_o))
            del out
        del codes, meta
        torch.cuda.empty_cache()


def test_segmented_codec_on_the_1p3b_layer_list(gpt1p3b):
    """All 292 layer tensors of the 1.3B model in one segmented encode and one segmented decode,
    every tensor against the oracle's single-tensor encoding."""
    n, x0, x_np = (gpt1p3b[k] for k in ("n", "x", "x_np"))
    sizes = [s for _, s in wl.model_tensors(wl.GPT_1P3B)]
    assert sum(sizes) == n
    segs = qb.Segments(sizes, B, DEV)
    codes, meta = segs.alloc_packed(8)
    qb.qsdp_quantize_weight_segmented(x0, segs, 8, 0.0, 31, codes, meta.reshape(-1))
    out = torch.full((n,), float("nan"), dtype=torch.float32, device=DEV)
    qb.qsdp_dequantize_segmented(codes, meta.reshape(-1), segs, 8, out)
    want_c, want_m, want_o = [], [], []
    off = 0
    for s in sizes:
        c, m, _ = ref.quantize_weight(x_np[off:off + s], 8, B, 0.0, 31)
        want_c.append(c); want_m.append(m.reshape(-1))
        want_o.append(ref.dequantize(c, m, s, 8, B))
        off += s
    assert same_packed(codes, meta, np.concatenate(want_c), np.concatenate(want_m))
    assert same_words(out, np.concatenate(want_o))
    del codes, meta, out
    torch.cuda.empty_cache()


@pytest.mark.parametrize("dtype", [torch.float16, torch.bfloat16])
def test_16bit_gradient_steps_on_the_full_vector(gpt1p3b, dtype):
    """Two fused steps (W8 G4, seed = step index), the second also writing the new weights in 16 bits,
    and the 4-bit gradient encoding, with the gradient handed over in 16 bits; the oracle gets that
    gradient widened by torch on the CPU. Every element."""
    n, x0, g, x_np = (gpt1p3b[k] for k in ("n", "x", "g", "x_np"))
    g16 = g.to(dtype)
    wide = g16.cpu().float().numpy()
    x = x0.clone()
    want = x_np.copy()
    x16 = torch.empty(n, dtype=dtype, device=DEV)
    want_c = np.zeros(ref.codes_bytes(n, 8, B) // 4, np.uint32)
    want_m = np.zeros(ref.meta_bytes(n, B) // 4, np.float32)
    for step in range(2):
        if step == 0:
            qb.qsdp_fused_step_g16(x, g16, 1e-3, 8, 4, B, 0.0, step)
        else:
            qb.qsdp_fused_step_mp(x, g16, 1e-3, 8, 4, B, 0.0, step, x16=x16)
        ref.fused_step_inplace(want, wide, 1e-3, 8, 4, B, 0.0, step, wcodes=want_c, wmeta=want_m)
        assert same_words(x, want), step
    narrow = ref.dequantize(want_c, want_m, n, 8, B, ref.F16 if dtype == torch.float16 else ref.BF16)
    assert same_words(x16, narrow)
    del x, x16
    gc, gm = qb.alloc_packed(n, 4, B, DEV)
    qb.qsdp_quantize_grad_g16(g16, 4, B, 5, 0, gc, gm.reshape(-1))
    assert same_packed(gc, gm, *ref.quantize_grad(wide, 4, B, 5))
    del g16, gc, gm
    torch.cuda.empty_cache()
