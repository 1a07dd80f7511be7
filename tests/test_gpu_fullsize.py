"""GPU parity at the benchmark's sizes and launch configuration: the GPT-shaped vectors of
the configurations, every output element compared with the bucket-parallel oracle run on host
copies of the same inputs, the vector of more than 2^32 elements included."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2302_02390_amd import binding as qb
from paper_2302_02390_amd import workloads as wl
from gpu_util import DEV, ORACLE_THREADS, first_mismatch, gather_rows, pinned_copy, pinned_empty, sample_bucket_ids

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpt1p3b():
    """The 1.3B vector and its gradient on the device, page-locked host copies of both for the
    oracle, and one more page-locked buffer of the same size for the oracle's iterate."""
    n = wl.model_numel(wl.GPT_1P3B)
    x = wl.weights(n, 1240, DEV)
    g = wl.grads_student_t3(n, 1241, DEV)
    torch.cuda.synchronize()
    x_h, x_np = pinned_copy(x)
    g_h, g_np = pinned_copy(g)
    work_h, work_np = pinned_empty(n, torch.float32)
    ref.set_threads(ORACLE_THREADS)
    yield {"n": n, "x": x, "g": g, "x_np": x_np, "g_np": g_np, "work_h": work_h, "work_np": work_np}
    ref.set_threads(1)
    del x, g, x_h, g_h, work_h
    torch.cuda.empty_cache()


def same_packed(codes, meta, want_codes, want_meta):
    """Packed codes and meta on the device against the oracle's, every word."""
    return first_mismatch(codes, want_codes.view(np.int32)) == -1 and \
        first_mismatch(meta.reshape(-1), want_meta.reshape(-1)) == -1


def test_config2_gpt125m_quantize_dequantize_bf16_fused():
    """125M vector (short tail bucket of 256 elements), W8 G8, bucket 1024: both quantizers, the
    decode to bf16 and the fused step, every output element against the oracle."""
    n, B = wl.model_numel(wl.GPT_125M), 1024
    assert n % B == 256
    x = wl.weights(n, 1236, DEV)
    g = wl.grads_student_t3(n, 1237, DEV)
    x_np, g_np = x.cpu().numpy(), g.cpu().numpy()
    ref.set_threads(ORACLE_THREADS)
    gc, gm = qb.alloc_packed(n, 8, B, DEV)
    qb.qsdp_quantize_grad(g, 8, B, 0, 0, gc, gm.reshape(-1))
    assert same_packed(gc, gm, *ref.quantize_grad(g_np, 8, B, 0))
    wc, wm = qb.alloc_packed(n, 8, B, DEV)
    qb.qsdp_quantize_weight(x, 8, B, 0.0, 0, wc, wm.reshape(-1))
    want_c, want_m, _ = ref.quantize_weight(x_np, 8, B, 0.0, 0)
    assert same_packed(wc, wm, want_c, want_m)
    out = torch.empty(n, dtype=torch.bfloat16, device=DEV)
    qb.qsdp_dequantize(wc, wm.reshape(-1), n, 8, B, out)
    want = ref.dequantize(want_c, want_m, n, 8, B, ref.BF16)
    assert first_mismatch(out, want.view(np.int16)) == -1
    fc, fm = qb.alloc_packed(n, 8, B, DEV)
    qb.qsdp_fused_step(x, g, 1e-3, 8, 8, B, 0.0, 0, 0, fc, fm.reshape(-1))
    want_x, want_c, want_m, _ = ref.fused_step(x_np, g_np, 1e-3, 8, 8, B, 0.0, 0, emit_codes=True)
    ref.set_threads(1)
    assert first_mismatch(x, want_x) == -1
    assert same_packed(fc, fm, want_c, want_m)


def test_config3_gpt350m_per_layer_tensors_whole_model():
    """350M as 292 separate per-layer tensors (bucketing restarts per tensor), W8 G4, bucket 1024.
    The oracle quantizes every tensor on its own; the library does the same once as one launch per
    tensor and once as a single multi-tensor launch, and both must reproduce the oracle on every
    element of every tensor (codes, meta, new weights)."""
    shape, B, seed = wl.GPT_350M, 1024, 3
    sizes = [s for _, s in wl.model_tensors(shape)]
    assert len(sizes) == 292 and all(s % 8 == 0 for s in sizes)
    n = sum(sizes)
    x = wl.weights(n, 1238, DEV)
    g = wl.grads_student_t3(n, 1239, DEV)
    x_np, g_np = x.cpu().numpy(), g.cpu().numpy()
    ref.set_threads(ORACLE_THREADS)
    want_x = x_np.copy()
    want_gc, want_gm, want_wc, want_wm, want_fc, want_fm = [], [], [], [], [], []
    off = 0
    for s in sizes:
        sl = slice(off, off + s)
        c, m = ref.quantize_grad(g_np[sl], 4, B, seed, index_offset=off)
        want_gc.append(c); want_gm.append(m)
        c, m, _ = ref.quantize_weight(x_np[sl], 8, B, 0.0, seed)
        want_wc.append(c); want_wm.append(m)
        fc = np.zeros(ref.codes_bytes(s, 8, B) // 4, np.uint32)
        fm = np.zeros(ref.meta_bytes(s, B) // 4, np.float32)
        ref.fused_step_inplace(want_x[sl], g_np[sl], 1e-3, 8, 4, B, 0.0, seed, index_offset=off, wcodes=fc, wmeta=fm)
        want_fc.append(fc); want_fm.append(fm)
        off += s
    ref.set_threads(1)
    want_gc, want_gm = np.concatenate(want_gc), np.concatenate(want_gm)
    want_wc, want_wm = np.concatenate(want_wc), np.concatenate(want_wm)
    want_fc, want_fm = np.concatenate(want_fc), np.concatenate(want_fm)

    # one multi-tensor launch per operation
    segs = qb.Segments(sizes, B, DEV)
    gc, gm = segs.alloc_packed(4)
    qb.qsdp_quantize_grad_segmented(g, segs, 4, seed, 0, gc, gm.reshape(-1))
    assert same_packed(gc, gm, want_gc, want_gm)
    wc, wm = segs.alloc_packed(8)
    qb.qsdp_quantize_weight_segmented(x, segs, 8, 0.0, seed, wc, wm.reshape(-1))
    assert same_packed(wc, wm, want_wc, want_wm)
    fc, fm = segs.alloc_packed(8)
    x_seg = x.clone()
    qb.qsdp_fused_step_segmented(x_seg, g, segs, 1e-3, 8, 4, 0.0, seed, 0, fc, fm.reshape(-1))
    assert first_mismatch(x_seg, want_x) == -1
    assert same_packed(fc, fm, want_fc, want_fm)
    out = torch.empty(n, dtype=torch.bfloat16, device=DEV)
    qb.qsdp_dequantize_segmented(fc, fm.reshape(-1), segs, 8, out)
    ref.set_threads(ORACLE_THREADS)
    want = ref.dequantize(want_fc, want_fm, n, 8, B, ref.BF16)   # every tensor is a whole number of buckets
    ref.set_threads(1)
    assert first_mismatch(out, want.view(np.int16)) == -1

    # one launch per tensor (each with buffers of its own: a tensor's meta need not start 16-byte aligned
    # inside the whole model's meta buffer)
    x_per = x.clone()
    per = {"gc": [], "gm": [], "wc": [], "wm": []}
    for (o, s, fb) in segs.host.tolist():
        c, m = qb.alloc_packed(s, 4, B, DEV)
        qb.qsdp_quantize_grad(g[o:o + s], 4, B, seed, o, c, m.reshape(-1))
        per["gc"].append(c); per["gm"].append(m)
        c, m = qb.alloc_packed(s, 8, B, DEV)
        qb.qsdp_quantize_weight(x[o:o + s], 8, B, 0.0, seed, c, m.reshape(-1))
        per["wc"].append(c); per["wm"].append(m)
        qb.qsdp_fused_step(x_per[o:o + s], g[o:o + s], 1e-3, 8, 4, B, 0.0, seed, o)
    assert same_packed(torch.cat(per["gc"]), torch.cat(per["gm"]), want_gc, want_gm)
    assert same_packed(torch.cat(per["wc"]), torch.cat(per["wm"]), want_wc, want_wm)
    assert first_mismatch(x_per, want_x) == -1


def test_config4_gpt1p3b_ten_fused_steps_whole_vector(gpt1p3b):
    """The headline workload in the benchmark's launch configuration: 10 fused steps, seed = step
    index, x carried, W8 G4, bucket 1024. The oracle carries its own iterate on the host; after every
    step all 1,315,723,264 weights are compared, and on the first and the last step the packed codes
    and the meta of the new weights as well."""
    w = gpt1p3b
    n, g, B = w["n"], w["g"], 1024
    assert n % B == 0
    x = w["x"].clone()
    xo = w["work_np"]
    np.copyto(xo, w["x_np"])
    wc, wm = qb.alloc_packed(n, 8, B, DEV)
    oc = np.zeros(ref.codes_bytes(n, 8, B) // 4, np.uint32)
    om = np.zeros(ref.meta_bytes(n, B) // 4, np.float32)
    for step in range(10):
        emit = step in (0, 9)
        if emit:
            qb.qsdp_fused_step(x, g, 1e-3, 8, 4, B, 0.0, step, 0, wc, wm.reshape(-1))
            ref.fused_step_inplace(xo, w["g_np"], 1e-3, 8, 4, B, 0.0, step, wcodes=oc, wmeta=om)
        else:
            qb.qsdp_fused_step(x, g, 1e-3, 8, 4, B, 0.0, step)
            ref.fused_step_inplace(xo, w["g_np"], 1e-3, 8, 4, B, 0.0, step)
        assert first_mismatch(x, w["work_h"]) == -1, step
        if emit:
            assert same_packed(wc, wm, oc, om), step
    # every iterate sits on its bucket's 8-bit grid: at most 256 distinct values per bucket
    rows = gather_rows(x, sample_bucket_ids(n // B, 50, 4), B)
    assert max(len(np.unique(r)) for r in rows) <= 256


def test_config4_eight_shards_reproduce_the_whole_vector(gpt1p3b):
    """How the path shards: every worker runs the same calls on its eighth of the vector with index_offset =
    the shard's first global element (the rounding uniforms follow the global index, the weight shift
    depends on the seed only). Eight such calls, on shards of unequal bucket-aligned sizes, must leave
    exactly the oracle's whole-vector result: the new weights, their codes and meta, and the gradient's codes."""
    w = gpt1p3b
    n, g, B = w["n"], w["g"], 1024
    nb = n // B
    # shard boundaries at even bucket numbers: the slices of the shared meta buffer stay 16-byte aligned
    cuts = [0] + [int(nb * f) // 2 * 2 * B for f in (0.11, 0.25, 0.37, 0.5, 0.68, 0.75, 0.93)] + [n]
    x = w["x"].clone()
    wc, wm = qb.alloc_packed(n, 8, B, DEV)
    gc, gm = qb.alloc_packed(n, 4, B, DEV)
    wm, gm = wm.reshape(-1), gm.reshape(-1)
    for lo, hi in zip(cuts[:-1], cuts[1:]):
        b0, b1 = lo // B, hi // B
        qb.qsdp_fused_step(x[lo:hi], g[lo:hi], 1e-3, 8, 4, B, 0.0, 5, lo, wc[b0 * 256:b1 * 256], wm[2 * b0:2 * b1])
        qb.qsdp_quantize_grad(g[lo:hi], 4, B, 5, lo, gc[b0 * 128:b1 * 128], gm[2 * b0:2 * b1])
    xo = w["work_np"]
    np.copyto(xo, w["x_np"])
    oc = np.zeros(ref.codes_bytes(n, 8, B) // 4, np.uint32)
    om = np.zeros(ref.meta_bytes(n, B) // 4, np.float32)
    ref.fused_step_inplace(xo, w["g_np"], 1e-3, 8, 4, B, 0.0, 5, wcodes=oc, wmeta=om)
    assert first_mismatch(x, w["work_h"]) == -1
    assert same_packed(wc, wm, oc, om)
    assert same_packed(gc, gm, *ref.quantize_grad(w["g_np"], 4, B, 5))


@pytest.mark.parametrize("B", [128, 512, 1024, 4096])
def test_config5_bit_and_bucket_sweep_on_a_16m_slice(gpt1p3b, B):
    """Every combination G in {2,3,4,6,8} x W in {4,6,8} at this bucket size on the first 2^24
    elements, each output element against the oracle."""
    w = gpt1p3b
    n = 1 << 24
    g, x0 = w["g"][:n], w["x"][:n]
    g_np, x_np = w["g_np"][:n], w["x_np"][:n]
    for gbits in (2, 3, 4, 6, 8):
        gc, gm = qb.alloc_packed(n, gbits, B, DEV)
        qb.qsdp_quantize_grad(g, gbits, B, 5, 0, gc, gm.reshape(-1))
        assert same_packed(gc, gm, *ref.quantize_grad(g_np, gbits, B, 5)), (gbits, B)
        for wbits in (4, 6, 8):
            x = x0.clone()
            wc, wm = qb.alloc_packed(n, wbits, B, DEV)
            qb.qsdp_fused_step(x, g, 1e-3, wbits, gbits, B, 0.0, 5, 0, wc, wm.reshape(-1))
            want_x, want_c, want_m, _ = ref.fused_step(x_np, g_np, 1e-3, wbits, gbits, B, 0.0, 5, emit_codes=True)
            assert first_mismatch(x, want_x) == -1, (wbits, gbits, B)
            assert same_packed(wc, wm, want_c, want_m), (wbits, gbits, B)
            # the emitted codes decode to the new x
            out = torch.empty(n, dtype=torch.float32, device=DEV)
            qb.qsdp_dequantize(wc, wm.reshape(-1), n, wbits, B, out)
            assert torch.equal(out, x)
    for wbits in (4, 6, 8):
        wc, wm = qb.alloc_packed(n, wbits, B, DEV)
        qb.qsdp_quantize_weight(x0, wbits, B, 0.0, 5, wc, wm.reshape(-1))
        want_c, want_m, _ = ref.quantize_weight(x_np, wbits, B, 0.0, 5)
        assert same_packed(wc, wm, want_c, want_m), (wbits, B)


@pytest.mark.parametrize("delta,wbits", [(2.0**-6, 4), (2.0**-8, 6), (2.0**-10, 8), (2.0**-10, 4)])
def test_config5_lattice_quantizer_full_vector(gpt1p3b, delta, wbits):
    """Explicit-delta random-shift quantizer on the whole 1.3B vector: codes, meta and the saturation
    count of the weight quantizer, then the new weights and the saturation count of a fused step on
    that grid, all against the oracle over the whole vector (the last pairing saturates heavily)."""
    w = gpt1p3b
    n, B = w["n"], 1024
    wc, wm = qb.alloc_packed(n, wbits, B, DEV)
    sat = torch.zeros(1, dtype=torch.int64, device=DEV)
    qb.qsdp_quantize_weight(w["x"], wbits, B, delta, 3, wc, wm.reshape(-1), sat)
    want_c, want_m, want_sat = ref.quantize_weight(w["x_np"], wbits, B, delta, 3)
    assert same_packed(wc, wm, want_c, want_m)
    assert int(sat) == want_sat
    if (delta, wbits) == (2.0**-10, 4):
        assert want_sat > n // 2          # 16 cells of 2^-10 against a spread of ~0.14
    else:
        assert want_sat <= n // 10**6     # the pairings of the configuration fit their buckets
    del want_c, want_m
    x = w["x"].clone()
    sat.zero_()
    qb.qsdp_fused_step(x, w["g"], 1e-3, wbits, 4, B, delta, 3, 0, None, None, sat)
    np.copyto(w["work_np"], w["x_np"])
    want_sat = ref.fused_step_inplace(w["work_np"], w["g_np"], 1e-3, wbits, 4, B, delta, 3)
    assert first_mismatch(x, w["work_h"]) == -1
    assert int(sat) == want_sat


@pytest.mark.parametrize("wbits,gbits,B", [(8, 4, 1024), (4, 2, 128), (8, 8, 4096), (6, 3, 512), (5, 4, 1024),
                                           (7, 5, 2048), (1, 1, 256)])
def test_config5_diagonal_full_vector(gpt1p3b, wbits, gbits, B):
    """The fused step with code output on the whole 1.3B vector for the diagonal of the sweep (and
    three more width / bucket pairs, so that every wave-kernel shape is run at full size): new
    weights, packed codes and meta, every element against the oracle."""
    w = gpt1p3b
    n = w["n"]
    x = w["x"].clone()
    wc, wm = qb.alloc_packed(n, wbits, B, DEV)
    qb.qsdp_fused_step(x, w["g"], 1e-3, wbits, gbits, B, 0.0, 8, 0, wc, wm.reshape(-1))
    np.copyto(w["work_np"], w["x_np"])
    oc = np.zeros(ref.codes_bytes(n, wbits, B) // 4, np.uint32)
    om = np.zeros(ref.meta_bytes(n, B) // 4, np.float32)
    ref.fused_step_inplace(w["work_np"], w["g_np"], 1e-3, wbits, gbits, B, 0.0, 8, wcodes=oc, wmeta=om)
    assert first_mismatch(x, w["work_h"]) == -1
    assert same_packed(wc, wm, oc, om)


def test_config5_layerwise_dequantize_to_bf16(gpt1p3b):
    """What a forward-pass weight gather needs: decode each d=2048 block (50,358,272 elements)
    to bf16. All 24 blocks are quantized and decoded; codes, meta and the bf16 output of every
    block are compared in full with the oracle."""
    w = gpt1p3b
    B = 1024
    d = wl.GPT_1P3B.d
    blk = wl.block_numel(d)
    start = (wl.VOCAB + wl.N_CTX) * d
    out = torch.empty(blk, dtype=torch.bfloat16, device=DEV)
    for layer in range(wl.GPT_1P3B.layers):
        lo, hi = start + layer * blk, start + (layer + 1) * blk
        wc, wm = qb.alloc_packed(blk, 8, B, DEV)
        qb.qsdp_quantize_weight(w["x"][lo:hi], 8, B, 0.0, layer, wc, wm.reshape(-1))
        qb.qsdp_dequantize(wc, wm.reshape(-1), blk, 8, B, out)
        want_c, want_m, _ = ref.quantize_weight(w["x_np"][lo:hi], 8, B, 0.0, layer)
        assert same_packed(wc, wm, want_c, want_m), layer
        want = ref.dequantize(want_c, want_m, blk, 8, B, ref.BF16)
        assert first_mismatch(out, want.view(np.int16)) == -1, layer


def test_more_than_2_to_32_elements():
    """Maximum sizes: a vector of 2^32 + 3*1024 + 5 elements (17 GB of fp32). Element indices,
    Philox counters and code offsets pass 32 bits, the grid passes 2^20 workgroups (so waves
    stride), and the vector ends in a short bucket. Gradient encoding, its decode to bf16 and the
    fused step in place, every output element against the oracle."""
    B = 1024
    n = (1 << 32) + 3 * B + 5

    def filled(std, seed0):
        t = torch.empty(n, dtype=torch.float32, device=DEV)
        for s in range(0, n, 1 << 28):                   # fill in chunks: bounded temporaries
            e = min(n, s + (1 << 28))
            t[s:e].normal_(0.0, std, generator=torch.Generator(device=DEV).manual_seed(seed0 + (s >> 28)))
        return t

    ref.set_threads(ORACLE_THREADS)
    g = filled(1e-3, 0)
    g_np = g.cpu().numpy()
    gc, gm = qb.alloc_packed(n, 4, B, DEV)
    qb.qsdp_quantize_grad(g, 4, B, 3, 0, gc, gm.reshape(-1))
    want_c, want_m = ref.quantize_grad(g_np, 4, B, 3)
    assert same_packed(gc, gm, want_c, want_m)
    out = torch.empty(n, dtype=torch.bfloat16, device=DEV)
    qb.qsdp_dequantize(gc, gm.reshape(-1), n, 4, B, out)
    want = ref.dequantize(want_c, want_m, n, 4, B, ref.BF16)
    assert first_mismatch(out, want.view(np.int16)) == -1
    del out, gc, gm, want, want_c, want_m
    torch.cuda.empty_cache()
    x = filled(0.02, 100)            # another 17 GB, updated in place
    want_x = x.cpu().numpy()
    qb.qsdp_fused_step(x, g, 1e-3, 8, 4, B, 0.0, 4)
    ref.fused_step_inplace(want_x, g_np, 1e-3, 8, 4, B, 0.0, 4)
    ref.set_threads(1)
    assert first_mismatch(x, want_x) == -1
    del x, g
    torch.cuda.empty_cache()
