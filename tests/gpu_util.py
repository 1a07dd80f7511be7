"""Helpers for the GPU parity tests: run the library through its binding, the oracle on the
host copy of the same inputs, and compare."""
import os

import numpy as np
import torch

from oracle import ref
from paper_2302_02390_amd import binding as qb

DEV = "cuda:0"


def np_u32(t):
    return t.detach().cpu().numpy().view(np.uint32).reshape(-1)


def np_f32(t):
    return t.detach().cpu().numpy().reshape(-1)


def bits_equal(a, b):
    """Bit-for-bit equality of two float32 arrays."""
    return np.array_equal(np.asarray(a, np.float32).view(np.uint32), np.asarray(b, np.float32).view(np.uint32))


def guarded(numel, dtype, fill):
    """A tensor with 64 sentinel elements before and after the payload view (16-byte aligned)."""
    pad = 64
    full = torch.full((numel + 2 * pad,), fill, dtype=dtype, device=DEV)
    return full, full[pad:pad + numel]


def guards_intact(full, numel, fill):
    pad = 64
    f = full.cpu()
    return bool((f[:pad] == fill).all() and (f[pad + numel:] == fill).all())


def gpu_quantize_grad(g_np, bits, bucket, seed, index_offset=0):
    g = torch.from_numpy(np.ascontiguousarray(g_np, np.float32)).to(DEV)
    n = g.numel()
    ncw = qb.codes_bytes(n, bits, bucket) // 4
    nb = qb.meta_bytes(n, bucket) // 8
    cfull, codes = guarded(ncw, torch.int32, 0x5A5A5A5A)
    mfull, meta = guarded(2 * nb, torch.float32, -777.0)
    qb.qsdp_quantize_grad(g, bits, bucket, seed, index_offset, codes, meta)
    torch.cuda.synchronize()
    assert guards_intact(cfull, ncw, 0x5A5A5A5A) and guards_intact(mfull, 2 * nb, -777.0)
    return codes, meta


def gpu_quantize_weight(x_np, bits, bucket, delta, seed):
    x = torch.from_numpy(np.ascontiguousarray(x_np, np.float32)).to(DEV)
    n = x.numel()
    ncw = qb.codes_bytes(n, bits, bucket) // 4
    nb = qb.meta_bytes(n, bucket) // 8
    cfull, codes = guarded(ncw, torch.int32, 0x5A5A5A5A)
    mfull, meta = guarded(2 * nb, torch.float32, -777.0)
    sat = torch.zeros(2, dtype=torch.int64, device=DEV)
    qb.qsdp_quantize_weight(x, bits, bucket, delta, seed, codes, meta, sat[:1])
    torch.cuda.synchronize()
    assert guards_intact(cfull, ncw, 0x5A5A5A5A) and guards_intact(mfull, 2 * nb, -777.0)
    assert int(sat[1]) == 0
    return codes, meta, int(sat[0])


def gpu_dequantize(codes, meta, n, bits, bucket, dtype):
    fill = 123.0
    ofull, out = guarded(n, dtype, fill)
    qb.qsdp_dequantize(codes, meta, n, bits, bucket, out)
    torch.cuda.synchronize()
    assert guards_intact(ofull, n, fill)
    return out


def gpu_fused_step(x_np, g_np, lr, wbits, gbits, bucket, delta, seed, index_offset=0, emit=False):
    n = x_np.size
    xfull, x = guarded(n, torch.float32, -555.0)
    x.copy_(torch.from_numpy(np.ascontiguousarray(x_np, np.float32)))
    g = torch.from_numpy(np.ascontiguousarray(g_np, np.float32)).to(DEV)
    wcodes = wmeta = None
    if emit:
        wcodes, wmeta = qb.alloc_packed(n, wbits, bucket, DEV)
        wmeta = wmeta.reshape(-1)
    sat = torch.zeros(1, dtype=torch.int64, device=DEV)
    qb.qsdp_fused_step(x, g, lr, wbits, gbits, bucket, delta, seed, index_offset, wcodes, wmeta, sat)
    torch.cuda.synchronize()
    assert guards_intact(xfull, n, -555.0)
    return x, wcodes, wmeta, int(sat[0])


def synth(n, seed, heavy=True):
    rng = np.random.default_rng(seed)
    x = (rng.normal(size=n) * 0.02).astype(np.float32)
    g = ((rng.standard_t(3, size=n) if heavy else rng.normal(size=n)) * 1e-3).astype(np.float32)
    return x, g


# ---------------------------------------------------------------------------------------
# Full-size checks: the oracle recomputes a sample of buckets one by one. A bucket of a
# long vector is a shard starting at a bucket boundary, so the oracle is called on the
# bucket's slice with index_offset = its global offset (shard invariance is pinned in the
# oracle's own tests).
# ---------------------------------------------------------------------------------------
def sample_bucket_ids(nb_full, k, seed):
    """k distinct full-bucket indices including the first and the last."""
    rng = np.random.default_rng(seed)
    k = min(k, nb_full)
    ids = set(rng.choice(nb_full, size=k, replace=False).tolist()) | {0, nb_full - 1}
    return np.array(sorted(ids), dtype=np.int64)


def gather_rows(t, ids, row_len):
    """Rows `ids` of the [*, row_len] view of the first full rows of flat tensor t, on the host."""
    nfull = t.numel() // row_len
    view = t[: nfull * row_len].view(nfull, row_len)
    idx = torch.from_numpy(ids).to(t.device)
    return view.index_select(0, idx).cpu().numpy()


# ---------------------------------------------------------------------------------------
# Whole-vector checks at full size: the bucket-parallel oracle recomputes every element on
# pinned host copies of the inputs, and the two results are compared bit for bit on the
# device, chunk by chunk.
# ---------------------------------------------------------------------------------------
ORACLE_THREADS = min(16, os.cpu_count() or 1)


def pinned_copy(t):
    """A page-locked host copy of tensor t, as (torch tensor, numpy view of the same memory)."""
    h = torch.empty(t.numel(), dtype=t.dtype, pin_memory=True)
    h.copy_(t.reshape(-1))
    return h, h.numpy()


def pinned_empty(numel, dtype):
    h = torch.empty(numel, dtype=dtype, pin_memory=True)
    return h, h.numpy()


def _as_ints(t):
    return t.view({1: torch.uint8, 2: torch.int16, 4: torch.int32, 8: torch.int64}[t.element_size()])


def first_mismatch(dev, host, chunk=1 << 27):
    """Index of the first element whose bit pattern differs between device tensor `dev` and host
    tensor (or numpy array) `host` of the same length and element size, or -1 when all are equal."""
    if isinstance(host, np.ndarray):
        host = torch.from_numpy(host)
    d, h = _as_ints(dev.reshape(-1)), _as_ints(host.reshape(-1))
    assert d.numel() == h.numel() and d.dtype == h.dtype, (d.shape, h.shape, d.dtype, h.dtype)
    for s in range(0, d.numel(), chunk):
        a = d[s:s + chunk]
        b = h[s:s + chunk].to(dev.device)
        if not torch.equal(a, b):
            return s + int((a != b).nonzero()[0])
    return -1
