"""The C ABI used from a plain C program (examples/qsdp_client.c, built with gcc): no Python, no
torch in that process. Its outputs are compared with the oracle bit for bit."""
import os
import subprocess

import numpy as np
import pytest

from oracle import ref
from gpu_util import bits_equal, synth

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CLIENT = os.path.join(ROOT, "examples", "qsdp_client")


@pytest.mark.parametrize("n,wbits,gbits,bucket", [(300 * 1024 + 77, 8, 4, 1024), (5000, 5, 3, 96)])
def test_plain_c_client_matches_the_oracle(tmp_path, n, wbits, gbits, bucket):
    if not os.path.exists(CLIENT):
        pytest.fail("examples/qsdp_client is not built: run python -m paper_2302_02390_amd.build")
    x, g = synth(n, 4242 + n)
    x.tofile(tmp_path / "x.f32")
    g.tofile(tmp_path / "g.f32")
    prefix = str(tmp_path / "out")
    lr, seed = 1e-3, 77
    r = subprocess.run([CLIENT, str(tmp_path / "x.f32"), str(tmp_path / "g.f32"), str(n), str(wbits), str(gbits),
                        str(bucket), repr(lr), str(seed), prefix], capture_output=True, text=True, timeout=100)
    assert r.returncode == 0, r.stdout + r.stderr

    want_gc, want_gm = ref.quantize_grad(g, gbits, bucket, seed)
    want_ghat = ref.dequantize(want_gc, want_gm, n, gbits, bucket)
    want_x, want_wc, want_wm, _ = ref.fused_step(x, g, np.float32(lr), wbits, gbits, bucket, 0.0, seed,
                                                 emit_codes=True)
    assert np.array_equal(np.fromfile(prefix + ".gcodes", dtype=np.uint32), want_gc)
    assert np.array_equal(np.fromfile(prefix + ".gmeta", dtype=np.uint32), want_gm.view(np.uint32).reshape(-1))
    assert bits_equal(np.fromfile(prefix + ".ghat", dtype=np.float32), want_ghat)
    assert bits_equal(np.fromfile(prefix + ".x", dtype=np.float32), want_x)
    assert np.array_equal(np.fromfile(prefix + ".wcodes", dtype=np.uint32), want_wc)
    assert np.array_equal(np.fromfile(prefix + ".wmeta", dtype=np.uint32), want_wm.view(np.uint32).reshape(-1))
