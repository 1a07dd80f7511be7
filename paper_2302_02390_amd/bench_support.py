"""Binding of ``libqsdp_bench.so``: plain streaming kernels (read, fill, copy, axpy, moments, encode) with the fused
step's access pattern, which ``bench.py`` times beside the codec as the memory system's attainable
ceilings. Benchmark support only: not part of the codec's C ABI and used by no codec entry point.
"""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libqsdp_bench.so")
TILE = 1024  # n must be a multiple of this many elements

_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_2302_02390_amd.build`")
        L = C.CDLL(LIB_PATH)
        vp, u64, f32 = C.c_void_p, C.c_uint64, C.c_float
        L.qsdp_bench_read.argtypes = [vp, u64, vp, vp]
        L.qsdp_bench_fill.argtypes = [vp, u64, f32, vp]
        L.qsdp_bench_copy.argtypes = [vp, vp, u64, vp]
        L.qsdp_bench_axpy.argtypes = [vp, vp, u64, f32, C.c_uint, vp]
        L.qsdp_bench_encode.argtypes = [vp, u64, C.c_int, vp, vp]
        L.qsdp_bench_moments.argtypes = [vp, vp, vp, vp, u64, f32, f32, C.c_uint, vp]
        _lib = L
    return _lib


def _args(*tensors):
    for t in tensors:
        if not (t.is_cuda and t.dtype == torch.float32 and t.is_contiguous()):
            raise TypeError("expected contiguous float32 GPU tensors")
    return C.c_void_p(torch.cuda.current_stream(tensors[0].device).cuda_stream)


def _check(rc, what):
    if rc != 0:
        raise RuntimeError(f"{what}: status {rc}")


def read(a, sink):
    s = _args(a, sink)
    _check(lib().qsdp_bench_read(a.data_ptr(), a.numel(), sink.data_ptr(), s), "qsdp_bench_read")


def fill(a, value):
    s = _args(a)
    _check(lib().qsdp_bench_fill(a.data_ptr(), a.numel(), float(value), s), "qsdp_bench_fill")


def copy(a, b):
    s = _args(a, b)
    if a.numel() != b.numel():
        raise ValueError("size mismatch")
    _check(lib().qsdp_bench_copy(a.data_ptr(), b.data_ptr(), a.numel(), s), "qsdp_bench_copy")


def axpy(x, g, lr, resident_cap_lds=0):
    """x <- x - lr*g; resident_cap_lds: unused dynamic LDS per workgroup (caps the workgroups per compute unit)."""
    s = _args(x, g)
    if x.numel() != g.numel():
        raise ValueError("size mismatch")
    _check(lib().qsdp_bench_axpy(x.data_ptr(), g.data_ptr(), x.numel(), float(lr), int(resident_cap_lds), s),
           "qsdp_bench_axpy")


def moments(x, g, m, v, lr, b, resident_cap_lds=0):
    """m <- b*m + g, v <- b*v + g*g, x <- x - lr*m (four operands read, three written: the AdamW step's mix)."""
    s = _args(x, g, m, v)
    if not (x.numel() == g.numel() == m.numel() == v.numel()):
        raise ValueError("size mismatch")
    _check(lib().qsdp_bench_moments(x.data_ptr(), g.data_ptr(), m.data_ptr(), v.data_ptr(), x.numel(), float(lr),
                                    float(b), int(resident_cap_lds), s), "qsdp_bench_moments")


def encode(a, bits, out):
    """Read a, write bits/8 bytes per element into out (int32, at least a.numel() * bits / 32 words)."""
    s = _args(a)
    if not (out.is_cuda and out.dtype == torch.int32 and out.is_contiguous() and out.numel() * 32 >= a.numel() * bits):
        raise ValueError("out: contiguous int32 GPU tensor of a.numel() * bits / 32 words")
    _check(lib().qsdp_bench_encode(a.data_ptr(), a.numel(), int(bits), out.data_ptr(), s), "qsdp_bench_encode")
