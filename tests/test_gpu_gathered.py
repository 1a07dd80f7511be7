"""GPU parity of qsdp_dequantize_gathered: one launch decodes the slots of an all-gathered layer
(each peer's shard quantized on its own) into the whole layer; compared with the oracle's decode
of every slot."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2302_02390_amd import binding as qb
from gpu_util import DEV, bits_equal, synth

pytestmark = pytest.mark.gpu


def _slots(x, n, shard, bits, B, npeers, seed):
    """Per-peer oracle quantization of the shards: list of (codes u32, meta f32[nb,2], elements)."""
    out = []
    for p in range(npeers):
        xs = x[p * shard: min((p + 1) * shard, n)]
        c, m, _ = ref.quantize_weight(xs, bits, B, 0.0, seed)
        out.append((c, m, xs.size))
    return out


@pytest.mark.parametrize("n,shard,B,bits", [
    (8 * 4096 + 0, 4096, 1024, 8),          # 8 equal shards
    (5 * 3072 + 1000, 3072, 1024, 4),       # last shard short, ragged tail bucket
    (3 * 2048 + 8, 2048, 512, 6),           # last shard of 8 elements
    (7 * 384 + 200, 384, 128, 3),
    (4 * 960 + 37, 960, 96, 5),             # generic bucket size, odd code width
    (5000, 8192, 1024, 8),                  # one peer only
    (64 * 1024 * 9 + 512, 64 * 1024, 4096, 2),
])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("interleaved", [False, True])
def test_gathered_decode_matches_slotwise_oracle(n, shard, B, bits, dtype, interleaved):
    npeers = -(-n // shard)
    x, _ = synth(n, 800 + n % 97)
    slots = _slots(x, n, shard, bits, B, npeers, 17)
    cw = ref.codes_bytes(shard, bits, B) // 4          # words of a full shard
    mw = ref.meta_bytes(shard, B) // 4
    if interleaved:
        # one receive buffer, slot p = [codes | meta], each part padded to 16 bytes
        cpad = (cw + 3) // 4 * 4
        row = cpad + (mw + 3) // 4 * 4
        buf = torch.zeros((npeers, row), dtype=torch.int32, device=DEV)
        codes_v = buf[:, :cw]
        meta_v = buf.view(torch.float32)[:, cpad:cpad + mw]
    else:
        # rows padded so that every slot starts 16-byte aligned
        codes_v = torch.zeros((npeers, (cw + 3) // 4 * 4), dtype=torch.int32, device=DEV)
        meta_v = torch.zeros((npeers, (mw + 3) // 4 * 4), dtype=torch.float32, device=DEV)
    for p, (c, m, _) in enumerate(slots):
        codes_v[p, :c.size] = torch.from_numpy(c.view(np.int32)).to(DEV)
        meta_v[p, :m.size] = torch.from_numpy(m.reshape(-1)).to(DEV)
    pad = 32
    out = torch.full((n + pad,), 3.0, dtype=dtype, device=DEV)
    qb.qsdp_dequantize_gathered(codes_v, meta_v, npeers, n, shard, bits, B, out)
    want = np.concatenate([ref.dequantize(c, m, k, bits, B, ref.BF16 if dtype == torch.bfloat16 else ref.F32)
                           for c, m, k in slots])
    got = out.cpu()
    assert torch.all(got[n:] == 3.0)
    if dtype == torch.float32:
        assert bits_equal(got[:n].numpy(), want)
    else:
        assert np.array_equal(got[:n].view(torch.int16).numpy().view(np.uint16), want)


def test_gathered_decode_equals_unsharded_decode():
    """Shards cut at bucket boundaries and quantized with the same seed give the codes of the
    unsharded layer, so the gathered decode equals the plain decode of the whole layer."""
    n, shard, B, bits = 6 * 8192 + 100, 8192, 1024, 8
    x, _ = synth(n, 77)
    xd = torch.from_numpy(x).to(DEV)
    npeers = -(-n // shard)
    cw, mw = ref.codes_bytes(shard, bits, B) // 4, ref.meta_bytes(shard, B) // 4
    codes = torch.zeros((npeers, cw), dtype=torch.int32, device=DEV)
    meta = torch.zeros((npeers, mw), dtype=torch.float32, device=DEV)
    for p in range(npeers):
        xs = xd[p * shard: min((p + 1) * shard, n)]
        qb.qsdp_quantize_weight(xs, bits, B, 0.0, 5, codes[p], meta[p])
    out = torch.empty(n, dtype=torch.bfloat16, device=DEV)
    qb.qsdp_dequantize_gathered(codes, meta, npeers, n, shard, bits, B, out)
    wc, wm = qb.alloc_packed(n, bits, B, DEV)
    qb.qsdp_quantize_weight(xd, bits, B, 0.0, 5, wc, wm.reshape(-1))
    whole = torch.empty(n, dtype=torch.bfloat16, device=DEV)
    qb.qsdp_dequantize(wc, wm.reshape(-1), n, bits, B, whole)
    assert torch.equal(out.view(torch.int16), whole.view(torch.int16))


def test_gathered_decode_rejects_bad_arguments():
    c = torch.zeros((2, 1024), dtype=torch.int32, device=DEV)
    m = torch.zeros((2, 8), dtype=torch.float32, device=DEV)
    out = torch.zeros(8192, dtype=torch.float32, device=DEV)
    with pytest.raises(qb.QsdpError):
        qb.qsdp_dequantize_gathered(c, m, 2, 8192, 4000, 8, 1024, out)      # shard not a multiple of bucket
    with pytest.raises(qb.QsdpError):
        qb.qsdp_dequantize_gathered(c, m, 2, 8192, 2048, 8, 1024, out)      # npeers != ceil(n / shard)
    small = torch.zeros((2, 512), dtype=torch.int32, device=DEV)
    with pytest.raises(ValueError):                                         # caught by the binding's size check
        qb.qsdp_dequantize_gathered(small, m, 2, 8192, 4096, 8, 1024, out)  # slots closer than a shard's codes
    wide = torch.zeros((2, 2048), dtype=torch.int32, device=DEV)
    with pytest.raises(qb.QsdpError):                                       # rows long enough, stride too small
        qb.qsdp_dequantize_gathered(wide.view(-1)[:2048 + 1024].as_strided((2, 1024), (512, 1)), m, 2, 8192, 4096, 8,
                                    1024, out)
    qb.qsdp_dequantize_gathered(c, m, 2, 8192, 4096, 8, 1024, out)          # the valid form of the same call


@pytest.mark.parametrize("bits,dtype", [(3, torch.float32), (5, torch.bfloat16)])
def test_gathered_decode_with_a_learned_level_table(bits, dtype):
    n, shard, B = 5 * 2048 + 700, 2048, 1024
    npeers = -(-n // shard)
    x, _ = synth(n, 404)
    levels = ref.fit_levels(x[:4 * B], bits, B, 0.05, ref.levels_uniform(bits))
    cw, mw = ref.codes_bytes(shard, bits, B) // 4, ref.meta_bytes(shard, B) // 4
    codes = torch.zeros((npeers, (cw + 3) // 4 * 4), dtype=torch.int32, device=DEV)
    meta = torch.zeros((npeers, (mw + 3) // 4 * 4), dtype=torch.float32, device=DEV)
    want = []
    for p in range(npeers):
        xs = x[p * shard: min((p + 1) * shard, n)]
        c, m = ref.quantize_levels(xs, bits, B, levels)
        codes[p, :c.size] = torch.from_numpy(c.view(np.int32)).to(DEV)
        meta[p, :m.size] = torch.from_numpy(m.reshape(-1)).to(DEV)
        want.append(ref.dequantize_levels(c, m, xs.size, bits, B, levels,
                                          ref.BF16 if dtype == torch.bfloat16 else ref.F32))
    want = np.concatenate(want)
    out = torch.empty(n, dtype=dtype, device=DEV)
    qb.qsdp_dequantize_gathered(codes, meta, npeers, n, shard, bits, B, out, torch.from_numpy(levels).to(DEV))
    if dtype == torch.float32:
        assert bits_equal(out.cpu().numpy(), want)
    else:
        assert np.array_equal(out.view(torch.int16).cpu().numpy().view(np.uint16), want)
