"""Writes tests/golden/spec_v3_vectors.txt: known-answer vectors of arithmetic specification
version 3, computed by the CPU oracle ONLY (never by the GPU path) on inputs given by integer
formulas, so that an accidental change of the specification (rounding order, RNG mapping, wire
format) shows up as a diff. Not a pin of the oracle against the paper: those are the
test_oracle_*.py files.

    python tests/golden/make_golden.py
"""
import hashlib
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
from oracle import ref  # noqa: E402

OUT = os.path.join(os.path.dirname(os.path.abspath(__file__)), "spec_v3_vectors.txt")


def inputs(n):
    """Weights and gradients from a multiplicative hash of the index (exact in binary64)."""
    i = np.arange(n, dtype=np.uint64)
    hx = (i * np.uint64(2654435761)) % np.uint64(1 << 32)
    hg = (i * np.uint64(40503) + np.uint64(12345)) % np.uint64(1 << 16)
    x = ((hx.astype(np.float64) / 2.0 ** 32 - 0.5) * 0.04).astype(np.float32)
    t = hg.astype(np.float64) / 2.0 ** 16 - 0.5
    g = (t * t * t * 0.008).astype(np.float32)     # heavy in the middle, long tails: products only
    return x, g


def digest(a):
    return hashlib.sha256(np.ascontiguousarray(a).tobytes()).hexdigest()


def head(a, k=4):
    return " ".join(f"{int(v):08x}" for v in np.ascontiguousarray(a).view(np.uint32).reshape(-1)[:k])


def vectors():
    n, B = 3 * 1024 + 100, 1024
    x, g = inputs(n)
    lines = ["spec_version 3", f"n {n} bucket {B}", f"x {digest(x)} {head(x)}", f"g {digest(g)} {head(g)}"]
    c, m = ref.quantize_grad(g, 4, B, 5, index_offset=8192)
    lines.append(f"quantize_grad b4 seed5 off8192 codes {digest(c)} {head(c)} meta {digest(m)} {head(m)}")
    c, m, s = ref.quantize_weight(x, 8, B, 0.0, 5)
    lines.append(f"quantize_weight b8 seed5 codes {digest(c)} {head(c)} meta {digest(m)} {head(m)} sat {s}")
    o = ref.dequantize(c, m, n, 8, B, ref.BF16)
    lines.append(f"dequantize b8 bf16 {digest(o)} {head(o)}")
    c, m, s = ref.quantize_weight(x, 4, B, 2.0 ** -8, 5)
    lines.append(f"quantize_weight b4 delta2^-8 seed5 codes {digest(c)} {head(c)} meta {digest(m)} {head(m)} sat {s}")
    y, c, m, s = ref.fused_step(x, g, 1e-3, 8, 4, B, 0.0, 5, index_offset=8192, emit_codes=True)
    lines.append(f"fused_step W8G4 lr1e-3 seed5 off8192 x {digest(y)} {head(y)} codes {digest(c)} meta {digest(m)}")
    y, c, m, s = ref.fused_step(x, g, 1e-3, 6, 3, 96, 0.0, 6, emit_codes=True)
    lines.append(f"fused_step W6G3 bucket96 seed6 x {digest(y)} {head(y)} codes {digest(c)} meta {digest(m)}")
    lines.append(f"weight_shift seed5 {head(np.float32(ref.weight_shift(5)), 1)} grad_shift seed5 "
                 f"{head(np.float32(ref.grad_shift(5)), 1)}")
    return lines


if __name__ == "__main__":
    with open(OUT, "w") as f:
        f.write("\n".join(vectors()) + "\n")
    print(OUT)
