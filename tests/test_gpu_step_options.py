"""GPU parity of the two options-block entry points (qsdp_fused_step_opts, qsdp_fused_adamw_step_opts): every
optional part of the fused step at once, against the oracle's single-tensor routines."""
import ctypes

import numpy as np
import pytest
import torch

from oracle import ref
from paper_2302_02390_amd import binding as qb
from gpu_util import DEV, bits_equal, np_f32, np_u32, synth

pytestmark = pytest.mark.gpu


def _bf16_round_trip(a):
    t = torch.from_numpy(a).to(torch.bfloat16)
    return t, t.to(torch.float32).numpy()


@pytest.mark.parametrize("B,wbits,gbits,delta", [(1024, 8, 4, 0.0), (128, 5, 3, 0.0), (2048, 6, 4, 2.0 ** -9), (96, 4, 2, 0.0)])
def test_sgd_step_with_every_option_at_once(B, wbits, gbits, delta):
    """Multi-tensor table + bfloat16 gradient + seed increment in device memory + variant flags + code output +
    16-bit copy of the new weights, one call; the oracle steps tensor by tensor on the widened gradient."""
    sizes = [768, 2304, 8, 1024 * 3 + 8, 4096 * 2, 24, 5000 + 3]
    n = sum(sizes)
    x, g = synth(n, 71 + B)
    g16, gw = _bf16_round_trip(g)
    flags = qb.QSDP_FLAG_SYMMETRIC
    seed, inc, off0 = 40, 7, 128
    want_x, want_c, want_m, want_sat = [], [], [], 0
    off = 0
    for s in sizes:
        sl = slice(off, off + s)
        xs, c, m, sat = ref.fused_step(x[sl], gw[sl], 1e-3, wbits, gbits, B, delta, seed + inc, index_offset=off0 + off,
                                       emit_codes=True, flags=flags)
        want_x.append(xs); want_c.append(c); want_m.append(m.reshape(-1)); want_sat += sat
        off += s
    want_x = np.concatenate(want_x)
    segs = qb.Segments(sizes, B, DEV)
    xd = torch.from_numpy(x).to(DEV)
    wc, wm = segs.alloc_packed(wbits)
    x16 = torch.empty(n, dtype=torch.bfloat16, device=DEV)
    sat = torch.zeros(1, dtype=torch.int64, device=DEV)
    counter = torch.full((1,), inc, dtype=torch.int64, device=DEV)
    qb.qsdp_fused_step_opts(xd, g16.to(DEV), 1e-3, wbits, gbits, B, delta, seed, off0, flags=flags, segs=segs, x16=x16,
                            seed_increment=counter, wcodes=wc, wmeta=wm.reshape(-1), n_saturated=sat)
    assert bits_equal(np_f32(xd), want_x)
    assert np.array_equal(np_u32(wc), np.concatenate(want_c))
    assert np.array_equal(np_u32(wm), np.concatenate(want_m).view(np.uint32))
    assert int(sat) == want_sat
    assert torch.equal(x16.cpu(), torch.from_numpy(want_x).to(torch.bfloat16))   # RNE of the decoded value


def test_adamw_step_options_match_the_oracle():
    B, wbits, gbits = 1024, 8, 4
    n = 5 * B + 300
    x, g = synth(n, 5)
    m0 = (1e-4 * np.arange(n) / n).astype(np.float32)
    v0 = (1e-8 * (1 + np.arange(n) % 7)).astype(np.float32)
    b1, b2, eps, wd, c1, c2 = 0.9, 0.95, 1e-8, 0.05, 0.19, 0.0975
    gh = torch.from_numpy(g).to(torch.float16)
    want = ref.fused_adamw_step(x, gh.to(torch.float32).numpy(), m0, v0, 2e-4, b1, b2, eps, wd, c1, c2, wbits, gbits, B,
                                0.0, 9, index_offset=64, flags=qb.QSDP_FLAG_KEEP_MASTER, emit_codes=True)
    xd, md, vd = (torch.from_numpy(a).to(DEV) for a in (x, m0, v0))
    wc, wm = qb.alloc_packed(n, wbits, B, DEV)
    qb.qsdp_fused_adamw_step_opts(xd, gh.to(DEV), md, vd, 2e-4, b1, b2, eps, wd, c1, c2, wbits, gbits, B, 0.0, 9, 64,
                                  flags=qb.QSDP_FLAG_KEEP_MASTER, wcodes=wc, wmeta=wm.reshape(-1))
    assert bits_equal(np_f32(xd), want[0]) and bits_equal(np_f32(md), want[1]) and bits_equal(np_f32(vd), want[2])
    assert np.array_equal(np_u32(wc), want[3]) and np.array_equal(np_u32(wm), want[4].view(np.uint32).reshape(-1))


def test_null_options_are_the_plain_fused_step_and_a_wrong_size_is_rejected():
    n, B = 3 * 1024 + 77, 1024
    x, g = synth(n, 6)
    want, _, _, _ = ref.fused_step(x, g, 1e-3, 8, 4, B, 0.0, 3)
    xd, gd = torch.from_numpy(x).to(DEV), torch.from_numpy(g).to(DEV)
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    L = qb.lib()
    assert L.qsdp_fused_step_opts(xd.data_ptr(), gd.data_ptr(), n, 1e-3, 8, 4, B, 0.0, 3, 0, None, stream) == qb.QSDP_OK
    torch.cuda.synchronize()
    assert bits_equal(np_f32(xd), want)
    o = qb.StepOptions()
    o.size = 8
    assert L.qsdp_fused_step_opts(xd.data_ptr(), gd.data_ptr(), n, 1e-3, 8, 4, B, 0.0, 3, 0, ctypes.byref(o),
                                  stream) == qb.QSDP_EINVAL
    # the AdamW call needs its moments
    o.size = ctypes.sizeof(qb.StepOptions)
    assert L.qsdp_fused_adamw_step_opts(xd.data_ptr(), gd.data_ptr(), n, 1e-3, 8, 4, B, 0.0, 3, 0, ctypes.byref(o),
                                        stream) == qb.QSDP_EINVAL
