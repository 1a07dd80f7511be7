"""Known-answer vectors of specification version 3 (tests/golden/spec_v3_vectors.txt, written by
tests/golden/make_golden.py from the oracle alone): the oracle must still reproduce them (CPU),
and the GPU path must produce the same digests (GPU)."""
import hashlib
import importlib.util
import os

import numpy as np
import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
_spec = importlib.util.spec_from_file_location("make_golden", os.path.join(HERE, "golden", "make_golden.py"))
make_golden = importlib.util.module_from_spec(_spec)
_spec.loader.exec_module(make_golden)


def stored():
    return open(os.path.join(HERE, "golden", "spec_v3_vectors.txt")).read().splitlines()


def test_oracle_reproduces_the_stored_vectors():
    assert make_golden.vectors() == stored()


@pytest.mark.gpu
def test_gpu_path_reproduces_the_stored_vectors():
    import torch
    from paper_2302_02390_amd import binding as qb
    dev = torch.device("cuda:0")
    lines = {ln.split(" ")[0] + " " + ln.split(" ")[1]: ln for ln in stored()}
    n, B = 3 * 1024 + 100, 1024
    x, g = make_golden.inputs(n)
    xd, gd = torch.from_numpy(x).to(dev), torch.from_numpy(g).to(dev)

    def dg(t):
        return hashlib.sha256(t.cpu().numpy().tobytes()).hexdigest()

    assert qb.spec_version() == 3
    c, m = qb.alloc_packed(n, 4, B, dev)
    qb.qsdp_quantize_grad(gd, 4, B, 5, 8192, c, m.reshape(-1))
    ln = lines["quantize_grad b4"]
    assert dg(c) in ln and dg(m) in ln
    c, m = qb.alloc_packed(n, 8, B, dev)
    qb.qsdp_quantize_weight(xd, 8, B, 0.0, 5, c, m.reshape(-1))
    ln = lines["quantize_weight b8"]
    assert dg(c) in ln and dg(m) in ln
    o = torch.empty(n, dtype=torch.bfloat16, device=dev)
    qb.qsdp_dequantize(c, m.reshape(-1), n, 8, B, o)
    assert dg(o.view(torch.int16)) in lines["dequantize b8"]
    c, m = qb.alloc_packed(n, 4, B, dev)
    sat = torch.zeros(1, dtype=torch.int64, device=dev)
    qb.qsdp_quantize_weight(xd, 4, B, 2.0 ** -8, 5, c, m.reshape(-1), sat)
    ln = lines["quantize_weight b4"]
    assert dg(c) in ln and dg(m) in ln and ln.endswith(f"sat {int(sat)}")
    for key, (wb, gb, bk, seed, off) in {"W8G4": (8, 4, 1024, 5, 8192), "W6G3": (6, 3, 96, 6, 0)}.items():
        y = xd.clone()
        c, m = qb.alloc_packed(n, wb, bk, dev)
        qb.qsdp_fused_step(y, gd, 1e-3, wb, gb, bk, 0.0, seed, off, c, m.reshape(-1))
        ln = [v for k, v in lines.items() if k.startswith("fused_step") and key in v][0]
        assert dg(y) in ln and dg(c) in ln and dg(m) in ln, key
