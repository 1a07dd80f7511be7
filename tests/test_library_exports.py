"""Host-only checks of the C ABI library: it loads without a GPU, exports every symbol the
header declares, and its size helpers and argument checks behave (no kernel is launched)."""
import ctypes
import os
import re

import pytest

from oracle import ref
from paper_2302_02390_amd import binding as qb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
C_INT_DEFAULT = ctypes.c_int   # what ctypes assumes when restype was never set
INT_RETURNING = {n for n in qb.EXPORTS if n not in ("qsdp_codes_bytes", "qsdp_meta_bytes", "qsdp_status_string",
                                                    "qsdp_segments_build", "qsdp_spec_version")}


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "qsdp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(qsdp_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    names = _declared_symbols()
    assert set(names) == set(qb.EXPORTS)
    lib = ctypes.CDLL(qb.LIB_PATH)
    for name in names:
        assert getattr(lib, name) is not None


def test_size_helpers_match_the_wire_format_and_the_oracle():
    for n, bits, bucket in [(1, 8, 1024), (1024, 8, 1024), (1025, 4, 1024), (10**6, 3, 128),
                            (1315723264, 4, 1024), (125226240, 8, 1024), (77, 1, 32)]:
        nb = -(-n // bucket)
        assert qb.codes_bytes(n, bits, bucket) == nb * bucket * bits // 8 == ref.codes_bytes(n, bits, bucket)
        assert qb.meta_bytes(n, bucket) == nb * 8 == ref.meta_bytes(n, bucket)
    assert qb.codes_bytes(0, 8, 1024) == 0 and qb.codes_bytes(10, 9, 1024) == 0
    assert qb.codes_bytes(10, 8, 100) == 0 and qb.meta_bytes(10, 8200) == 0
    assert qb.spec_version() == 3


def test_argument_errors_are_reported_before_any_launch():
    L = qb.lib()
    ok = ctypes.c_void_p(4096)
    odd = ctypes.c_void_p(4100)
    assert L.qsdp_quantize_grad(None, 10, 8, 1024, 0, 0, ok, ok, None) == qb.QSDP_EINVAL
    assert L.qsdp_quantize_grad(ok, 0, 8, 1024, 0, 0, ok, ok, None) == qb.QSDP_EINVAL
    assert L.qsdp_quantize_grad(ok, 10, 0, 1024, 0, 0, ok, ok, None) == qb.QSDP_EINVAL
    assert L.qsdp_quantize_grad(ok, 10, 8, 100, 0, 0, ok, ok, None) == qb.QSDP_EINVAL
    assert L.qsdp_quantize_grad(ok, 10, 8, 1024, 0, 12, ok, ok, None) == qb.QSDP_EINVAL
    assert L.qsdp_quantize_grad(odd, 10, 8, 1024, 0, 0, ok, ok, None) == qb.QSDP_EALIGN
    assert L.qsdp_quantize_weight(ok, 10, 8, 1024, -1.0, 0, ok, ok, None, None) == qb.QSDP_EINVAL
    assert L.qsdp_quantize_weight(ok, 10, 8, 1024, float("nan"), 0, ok, ok, None, None) == qb.QSDP_EINVAL
    assert L.qsdp_quantize_weight(ok, 10, 8, 1024, 0.0, 0, odd, ok, None, None) == qb.QSDP_EALIGN
    assert L.qsdp_dequantize(ok, ok, 10, 8, 1024, 3, ok, None) == qb.QSDP_EINVAL
    assert L.qsdp_dequantize(ok, ok, 10, 8, 1024, 1, odd, None) == qb.QSDP_EALIGN
    assert L.qsdp_fused_step(ok, ok, 10, 1e-3, 8, 4, 1024, 0.0, 0, 0, ok, None, None, None) == qb.QSDP_EINVAL
    assert L.qsdp_fused_step(ok, ok, 10, float("inf"), 8, 4, 1024, 0.0, 0, 0, None, None, None, None) == qb.QSDP_EINVAL
    assert L.qsdp_fused_step(ok, odd, 10, 1e-3, 8, 4, 1024, 0.0, 0, 0, None, None, None, None) == qb.QSDP_EALIGN
    # 16-bit gradient entry points: only the two 2-byte formats are inputs; the decoders never write binary16
    assert L.qsdp_quantize_grad_g16(ok, 0, 10, 8, 1024, 0, 0, 0, ok, ok, None) == qb.QSDP_EINVAL
    assert L.qsdp_quantize_grad_g16(ok, 3, 10, 8, 1024, 0, 0, 0, ok, ok, None) == qb.QSDP_EINVAL
    assert L.qsdp_quantize_grad_g16(odd, 2, 10, 8, 1024, 0, 0, 0, ok, ok, None) == qb.QSDP_EALIGN
    assert L.qsdp_fused_step_g16(ok, ok, 0, 10, 1e-3, 8, 4, 1024, 0.0, 0, 0, 0, None, None, None, None) == qb.QSDP_EINVAL
    assert L.qsdp_fused_step_g16(ok, ok, 1, 10, 1e-3, 8, 4, 1024, 0.0, 0, 4, 0, None, None, None, None) == qb.QSDP_EINVAL
    assert L.qsdp_dequantize_segmented(ok, ok, ok, 1, 1, 8, 1024, 3, ok, None) == qb.QSDP_EINVAL
    # the options block: its size field is checked, and its pointers like any argument
    o = qb.StepOptions()
    assert L.qsdp_fused_step_opts(ok, ok, 10, 1e-3, 8, 4, 1024, 0.0, 0, 0, ctypes.byref(o), None) == qb.QSDP_EINVAL
    o.size = ctypes.sizeof(qb.StepOptions)
    o.wcodes = 4096
    assert L.qsdp_fused_step_opts(ok, ok, 10, 1e-3, 8, 4, 1024, 0.0, 0, 0, ctypes.byref(o), None) == qb.QSDP_EINVAL
    o.wmeta = 4100
    assert L.qsdp_fused_step_opts(ok, ok, 10, 1e-3, 8, 4, 1024, 0.0, 0, 0, ctypes.byref(o), None) == qb.QSDP_EALIGN
    o.wmeta, o.g_dtype = 4096, 7
    assert L.qsdp_fused_step_opts(ok, ok, 10, 1e-3, 8, 4, 1024, 0.0, 0, 0, ctypes.byref(o), None) == qb.QSDP_EINVAL
    assert qb.status_string(qb.QSDP_EALIGN).startswith("pointer")


def test_header_is_plain_c(tmp_path):
    """include/qsdp.h is a C header: it compiles as strict C11 and every declared function can be
    named from C."""
    import subprocess
    names = [n for n in _declared_symbols()]
    src = tmp_path / "use_header.c"
    src.write_text('#include "qsdp.h"\n' + "const void* table[] = {" +
                   ", ".join(f"(const void*)(uintptr_t){n}" for n in names) + "};\n")
    subprocess.run(["gcc", "-std=c11", "-pedantic-errors", "-Wall", "-Werror", "-fsyntax-only",
                    "-I", os.path.join(ROOT, "include"), str(src)], check=True)


def test_binding_declares_the_signature_of_every_export():
    """ctypes guesses int for undeclared arguments, which truncates 64-bit sizes and pointers:
    every exported function must have its argument and result types set, and the number of
    arguments must match the header's declaration."""
    L = qb.lib()
    text = open(os.path.join(ROOT, "include", "qsdp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    for name in qb.EXPORTS:
        fn = getattr(L, name)
        assert fn.argtypes is not None, name
        decl = re.search(r"\b" + name + r"\s*\(([^)]*)\)", text).group(1).strip()
        params = [] if decl in ("", "void") else [" ".join(p_.split()) for p_ in decl.split(",")]
        assert len(fn.argtypes) == len(params), (name, len(fn.argtypes), len(params))
        assert fn.restype is not C_INT_DEFAULT or name in INT_RETURNING, name
        # ... and each argument's type must be the header's: a pointer, or the scalar of that width
        for k, (param, ctype) in enumerate(zip(params, fn.argtypes)):
            if "*" in param:
                want = ctypes.c_void_p
            else:
                base = param.rsplit(" ", 1)[0].replace("const ", "")
                want = {"uint64_t": ctypes.c_uint64, "uint32_t": ctypes.c_uint32, "int": ctypes.c_int,
                        "float": ctypes.c_float, "qsdp_dtype": ctypes.c_int}[base]
            assert ctype is want, (name, k, param, ctype)


def test_binding_rejects_undersized_buffers_before_calling_the_library():
    """The C ABI takes raw pointers; the binding is where buffer sizes can still be checked. CPU
    tensors fail the device check first, so the size helpers are exercised directly."""
    import torch
    codes = torch.zeros(255, dtype=torch.int32)
    meta = torch.zeros(2, dtype=torch.float32)
    with pytest.raises(ValueError):
        qb._packed_ok(codes, meta, 1024, 8, 1024)          # 256 words needed
    qb._packed_ok(torch.zeros(256, dtype=torch.int32), meta, 1024, 8, 1024)
    with pytest.raises(ValueError):
        qb._packed_ok(torch.zeros(512, dtype=torch.int32), meta, 1025, 8, 1024)   # two buckets: 4 meta floats
    with pytest.raises(ValueError):
        qb._rows_ok(torch.zeros((3, 100), dtype=torch.int32), torch.zeros((3, 2)), 1024, 4, 1024)
    qb._rows_ok(torch.zeros((3, 128), dtype=torch.int32), torch.zeros((3, 2)), 1024, 4, 1024)
    qb._packed_ok(codes, meta, 1024, 9, 1024)                # invalid bits: left to the library


def test_binding_rejects_tensors_on_different_devices():
    """A kernel runs on the device of its first tensor; memory of another device would fault there, so the
    binding refuses the call (shown with the `meta` device standing in for a second GPU)."""
    import torch
    x = torch.zeros(1024)
    g = torch.zeros(1024, device="meta")
    with pytest.raises(ValueError, match="tensors on"):
        qb.qsdp_fused_step(x, g, 1e-3, 8, 4, 1024, 0.0, 0)
    with pytest.raises(ValueError, match="tensors on"):
        qb.qsdp_dequantize(torch.zeros(256, dtype=torch.int32), torch.zeros(2), 1024, 8, 1024, out=g)
    with pytest.raises(TypeError):                             # same device, but not a GPU tensor
        qb.qsdp_fused_step(x, torch.zeros(1024), 1e-3, 8, 4, 1024, 0.0, 0)


def test_options_block_layout_matches_the_header(tmp_path):
    """binding.StepOptions mirrors qsdp_step_options field for field: same size and offsets as a C compiler gives."""
    import subprocess
    fields = [name for name, _ in qb.StepOptions._fields_]
    src = tmp_path / "layout.c"
    src.write_text('#include <stddef.h>\n#include <stdio.h>\n#include "qsdp.h"\nint main(void) {\n'
                   '    printf("%zu\\n", sizeof(qsdp_step_options));\n' +
                   "".join(f'    printf("%zu\\n", offsetof(qsdp_step_options, {f}));\n' for f in fields) +
                   "    return 0;\n}\n")
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-std=c11", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)], check=True)
    out = [int(v) for v in subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()]
    assert out[0] == ctypes.sizeof(qb.StepOptions)
    assert out[1:] == [getattr(qb.StepOptions, f).offset for f in fields]


def test_segments_build_writes_the_table_the_segmented_calls_require():
    """qsdp_segments_build (host only): tensors packed back to back, offsets multiples of 8, bucket numbers
    ascending with every tensor starting a new bucket; sizes that would break those invariants are refused."""
    import numpy as np
    L = qb.lib()

    def build(sizes, bucket):
        s = np.asarray(sizes, dtype=np.uint64)
        table = np.zeros((len(sizes), 3), dtype=np.uint64)
        total = int(L.qsdp_segments_build(s.ctypes.data_as(ctypes.c_void_p), len(sizes), bucket,
                                          table.ctypes.data_as(ctypes.c_void_p)))
        return total, table

    sizes = [768, 2304, 8, 1024 * 3 + 8, 4096, 24, 5000 + 3]
    for bucket in (32, 128, 1024, 4096):
        total, table = build(sizes, bucket)
        off = fb = 0
        for t, s in enumerate(sizes):
            assert table[t].tolist() == [off, s, fb]
            assert off % 8 == 0
            off += s
            fb += -(-s // bucket)
        assert total == fb
    assert build([1024, 0, 8], 1024)[0] == 0          # empty tensor
    assert build([1020, 8], 1024)[0] == 0             # a size other than the last not a multiple of 8
    assert build([1024], 100)[0] == 0                 # bucket not a multiple of 32
    assert build([1024, 1020], 1024)[0] == 2          # only the last size may be ragged
