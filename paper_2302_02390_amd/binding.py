"""Thin Python binding of the C ABI in ``include/qsdp.h`` (``libqsdp.so``).

Argument marshalling only: torch tensors supply device memory and the current stream; every
step of the computation runs in the HIP kernels. The functions have the names and argument
order of the C entry points. There is no fallback: if the library is not built, importing
the symbols raises.
"""
import ctypes as C
import functools
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libqsdp.so")

QSDP_OK, QSDP_EINVAL, QSDP_EALIGN, QSDP_ELAUNCH = 0, -1, -2, -3
QSDP_F32, QSDP_BF16, QSDP_F16 = 0, 1, 2
QSDP_FLAG_GRAD_SHIFT, QSDP_FLAG_NO_SHIFT, QSDP_FLAG_SYMMETRIC, QSDP_FLAG_KEEP_MASTER = 1, 2, 4, 8

# Signature of every export of include/qsdp.h: name -> (result, arguments). vp: pointer (device memory unless the
# header says host), the last vp of an entry point that launches work is the stream.
_u64, _u32, _i32, _f32, _vp = C.c_uint64, C.c_uint32, C.c_int, C.c_float, C.c_void_p
_SIGNATURES = {
    "qsdp_spec_version": (_u32, []),
    "qsdp_codes_bytes": (C.c_size_t, [_u64, _i32, _i32]),
    "qsdp_meta_bytes": (C.c_size_t, [_u64, _i32]),
    "qsdp_status_string": (C.c_char_p, [_i32]),
    "qsdp_quantize_grad": (_i32, [_vp, _u64, _i32, _i32, _u64, _u64, _vp, _vp, _vp]),
    "qsdp_quantize_grad_ex": (_i32, [_vp, _u64, _i32, _i32, _u64, _u64, _u32, _vp, _vp, _vp]),
    "qsdp_quantize_grad_g16": (_i32, [_vp, _i32, _u64, _i32, _i32, _u64, _u64, _u32, _vp, _vp, _vp]),
    "qsdp_quantize_weight": (_i32, [_vp, _u64, _i32, _i32, _f32, _u64, _vp, _vp, _vp, _vp]),
    "qsdp_quantize_weight_ex": (_i32, [_vp, _u64, _i32, _i32, _f32, _u64, _u32, _vp, _vp, _vp, _vp]),
    "qsdp_dequantize": (_i32, [_vp, _vp, _u64, _i32, _i32, _i32, _vp, _vp]),
    "qsdp_fused_step": (_i32, [_vp, _vp, _u64, _f32, _i32, _i32, _i32, _f32, _u64, _u64, _vp, _vp, _vp, _vp]),
    "qsdp_fused_step_ex": (_i32,
        [_vp, _vp, _u64, _f32, _i32, _i32, _i32, _f32, _u64, _u64, _u32, _vp, _vp, _vp, _vp]),
    "qsdp_fused_step_g16": (_i32,
        [_vp, _vp, _i32, _u64, _f32, _i32, _i32, _i32, _f32, _u64, _u64, _u32, _vp, _vp, _vp, _vp]),
    "qsdp_fused_step_mp": (_i32,
        [_vp, _vp, _i32, _u64, _f32, _i32, _i32, _i32, _f32, _u64, _u64, _u32, _vp, _vp, _vp, _i32, _vp, _vp]),
    "qsdp_fused_step_dseed": (_i32,
        [_vp, _vp, _u64, _f32, _i32, _i32, _i32, _f32, _u64, _vp, _u64, _u32, _vp, _vp, _vp, _vp]),
    "qsdp_fused_step_opts": (_i32, [_vp, _vp, _u64, _f32, _i32, _i32, _i32, _f32, _u64, _u64, _vp, _vp]),
    "qsdp_fused_adamw_step_opts": (_i32, [_vp, _vp, _u64, _f32, _i32, _i32, _i32, _f32, _u64, _u64, _vp, _vp]),
    "qsdp_fused_step_codes": (_i32, [_vp, _vp, _vp, _u64, _f32, _i32, _i32, _i32, _f32, _u64, _u64, _u32, _vp, _vp]),
    "qsdp_fused_adamw_step": (_i32,
        [_vp, _vp, _vp, _vp, _u64, _f32, _f32, _f32, _f32, _f32, _f32, _f32, _i32, _i32, _i32, _f32, _u64,
         _u64, _u32, _vp, _vp, _vp, _vp]),
    "qsdp_fused_adamw_step_mp": (_i32,
        [_vp, _vp, _i32, _vp, _vp, _u64, _f32, _f32, _f32, _f32, _f32, _f32, _f32, _i32, _i32, _i32, _f32, _u64,
         _u64, _u32, _vp, _vp, _vp, _i32, _vp, _vp]),
    "qsdp_fused_adamw_step_codes": (_i32,
        [_vp, _vp, _vp, _vp, _vp, _u64, _f32, _f32, _f32, _f32, _f32, _f32, _f32, _i32, _i32, _i32, _f32,
         _u64, _u64, _u32, _vp, _vp]),
    "qsdp_dequantize_add": (_i32, [_vp, _u64, _vp, _u64, _i32, _u64, _i32, _i32, _f32, _vp, _vp]),
    "qsdp_dequantize_gathered": (_i32, [_vp, _u64, _vp, _u64, _i32, _u64, _u64, _i32, _i32, _i32, _vp, _vp]),
    "qsdp_recv_step": (_i32,
        [_vp, _vp, _u64, _vp, _u64, _i32, _u64, _f32, _f32, _i32, _i32, _i32, _f32, _u64, _u32, _vp, _vp,
         _vp, _vp]),
    "qsdp_recv_adamw_step": (_i32,
        [_vp, _vp, _vp, _vp, _u64, _vp, _u64, _i32, _u64, _f32, _f32, _f32, _f32, _f32, _f32, _f32, _f32,
         _i32, _i32, _i32, _f32, _u64, _u32, _vp, _vp, _vp, _vp]),
    "qsdp_levels_uniform": (_i32, [_i32, _vp]),
    "qsdp_quantize_levels": (_i32, [_vp, _u64, _i32, _i32, _vp, _vp, _vp, _vp]),
    "qsdp_quantize_levels_stochastic": (_i32, [_vp, _u64, _i32, _i32, _vp, _u64, _u64, _vp, _vp, _vp]),
    "qsdp_dequantize_levels": (_i32, [_vp, _vp, _u64, _i32, _i32, _vp, _i32, _vp, _vp]),
    "qsdp_dequantize_levels_gathered": (_i32,
        [_vp, _u64, _vp, _u64, _i32, _u64, _u64, _i32, _i32, _vp, _i32, _vp, _vp]),
    "qsdp_fit_levels": (_i32, [_vp, _u64, _i32, _i32, _f32, _u64, _vp, _vp]),
    "qsdp_segments_build": (_u64, [_vp, _u32, _i32, _vp]),
    "qsdp_quantize_grad_segmented": (_i32, [_vp, _vp, _u32, _u64, _i32, _i32, _u64, _u64, _vp, _vp, _vp]),
    "qsdp_quantize_weight_segmented": (_i32, [_vp, _vp, _u32, _u64, _i32, _i32, _f32, _u64, _vp, _vp, _vp, _vp]),
    "qsdp_fused_step_segmented": (_i32,
        [_vp, _vp, _vp, _u32, _u64, _f32, _i32, _i32, _i32, _f32, _u64, _u64, _vp, _vp, _vp, _vp]),
    "qsdp_fused_step_segmented_mp": (_i32,
        [_vp, _vp, _i32, _vp, _u32, _u64, _f32, _i32, _i32, _i32, _f32, _u64, _u64, _u32, _vp, _vp, _vp, _i32,
         _vp, _vp]),
    "qsdp_dequantize_segmented": (_i32, [_vp, _vp, _vp, _u32, _u64, _i32, _i32, _i32, _vp, _vp]),
    "qsdp_fused_adamw_step_segmented": (_i32,
        [_vp, _vp, _vp, _vp, _vp, _u32, _u64, _f32, _f32, _f32, _f32, _f32, _f32, _f32, _i32, _i32, _i32,
         _f32, _u64, _u64, _u32, _vp, _vp, _vp, _vp]),
    "qsdp_fused_step_codes_segmented": (_i32,
        [_vp, _vp, _vp, _vp, _u32, _u64, _f32, _i32, _i32, _i32, _f32, _u64, _u64, _u32, _vp, _vp]),
    "qsdp_recv_step_segmented": (_i32,
        [_vp, _vp, _u32, _u64, _vp, _u64, _vp, _u64, _i32, _f32, _f32, _i32, _i32, _i32, _f32, _u64, _u32,
         _vp, _vp, _vp, _vp]),
    "qsdp_recv_adamw_step_segmented": (_i32,
        [_vp, _vp, _vp, _vp, _u32, _u64, _vp, _u64, _vp, _u64, _i32, _f32, _f32, _f32, _f32, _f32, _f32,
         _f32, _f32, _i32, _i32, _i32, _f32, _u64, _u32, _vp, _vp, _vp, _vp]),
    "qsdp_fit_levels_segmented": (_i32, [_vp, _vp, _u32, _i32, _i32, _f32, _u64, _vp, _vp]),
    "qsdp_quantize_levels_segmented": (_i32,
        [_vp, _vp, _u32, _u64, _i32, _i32, _vp, _i32, _u64, _u64, _vp, _vp, _vp]),
    "qsdp_dequantize_levels_segmented": (_i32, [_vp, _vp, _vp, _u32, _u64, _i32, _i32, _vp, _i32, _vp, _vp]),
}
EXPORTS = tuple(_SIGNATURES)

_lib = None


class QsdpError(RuntimeError):
    def __init__(self, status, what):
        self.status = status
        super().__init__(f"{what}: {status_string(status)} ({status})")


def lib():
    """Load libqsdp.so (built by ``python -m paper_2302_02390_amd.build``)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_2302_02390_amd.build`")
        L = C.CDLL(LIB_PATH)
        for name, (restype, argtypes) in _SIGNATURES.items():
            fn = getattr(L, name)
            fn.restype = restype
            fn.argtypes = argtypes
        _lib = L
    return _lib


def status_string(status):
    return lib().qsdp_status_string(int(status)).decode()


def spec_version():
    return int(lib().qsdp_spec_version())


def codes_bytes(n, bits, bucket):
    return int(lib().qsdp_codes_bytes(int(n), int(bits), int(bucket)))


def meta_bytes(n, bucket):
    return int(lib().qsdp_meta_bytes(int(n), int(bucket)))


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(t):
    return C.c_void_p(torch.cuda.current_stream(t.device).cuda_stream)


def _check(status, what):
    if status != QSDP_OK:
        raise QsdpError(status, what)


def _is(t, dtype):
    if not (t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise TypeError(f"expected a contiguous {dtype} tensor on the GPU")


def _out_dtype(out):
    """The decoders' output formats: float32, bfloat16 or float16 (IEEE binary16)."""
    dt = {torch.float32: QSDP_F32, torch.bfloat16: QSDP_BF16, torch.float16: QSDP_F16}.get(out.dtype)
    if dt is None:
        raise TypeError("out must be float32, bfloat16 or float16")
    return dt


def _is_rows(t, dtype):
    """A 2-D tensor whose rows are contiguous (the rows themselves may be strided apart)."""
    if not (t.is_cuda and t.dtype == dtype and t.dim() == 2 and (t.shape[1] == 1 or t.stride(1) == 1)):
        raise TypeError(f"expected a {dtype} GPU tensor [rows, row length] with contiguous rows")


def _need(t, numel, what):
    if t.numel() < numel:
        raise ValueError(f"{what} holds {t.numel()} elements, {numel} are needed")


def _packed_ok(codes, meta, n, bits, bucket):
    """The packed buffers are large enough for n elements (the C ABI takes raw pointers and cannot
    check this itself). Invalid n / bits / bucket are left to the library to report."""
    cb, mb = codes_bytes(n, bits, bucket), meta_bytes(n, bucket)
    if cb and mb:
        if codes is not None:
            _need(codes, cb // 4, "codes")
        if meta is not None:
            _need(meta, mb // 4, "meta")


def _rows_ok(codes, meta, n, bits, bucket):
    """Every row (peer slot) of the 2-D buffers is large enough for n elements."""
    cb, mb = codes_bytes(n, bits, bucket), meta_bytes(n, bucket)
    if cb and mb:
        if codes.shape[1] < cb // 4:
            raise ValueError(f"code rows hold {codes.shape[1]} words, {cb // 4} are needed")
        if meta.shape[1] < mb // 4:
            raise ValueError(f"meta rows hold {meta.shape[1]} floats, {mb // 4} are needed")


def alloc_packed(n, bits, bucket, device):
    """Empty (codes uint32-as-int32[...], meta float32[nb, 2]) buffers of the right size."""
    cb, mb = codes_bytes(n, bits, bucket), meta_bytes(n, bucket)
    if cb == 0 or mb == 0:
        raise QsdpError(QSDP_EINVAL, "alloc_packed")
    codes = torch.empty(cb // 4, dtype=torch.int32, device=device)
    meta = torch.empty((mb // 8, 2), dtype=torch.float32, device=device)
    return codes, meta


def qsdp_quantize_grad(g, bits, bucket, seed, index_offset, codes, meta):
    _is(g, torch.float32); _is(codes, torch.int32); _is(meta, torch.float32)
    _packed_ok(codes, meta, g.numel(), bits, bucket)
    with torch.cuda.device(g.device):
        _check(lib().qsdp_quantize_grad(_ptr(g), g.numel(), bits, bucket, seed, index_offset,
                                        _ptr(codes), _ptr(meta), _stream(g)), "qsdp_quantize_grad")


def qsdp_quantize_grad_ex(g, bits, bucket, seed, index_offset, flags, codes, meta):
    _is(g, torch.float32); _is(codes, torch.int32); _is(meta, torch.float32)
    _packed_ok(codes, meta, g.numel(), bits, bucket)
    with torch.cuda.device(g.device):
        _check(lib().qsdp_quantize_grad_ex(_ptr(g), g.numel(), bits, bucket, seed, index_offset, flags,
                                           _ptr(codes), _ptr(meta), _stream(g)), "qsdp_quantize_grad_ex")


def qsdp_quantize_weight_ex(x, bits, bucket, delta, seed, flags, codes, meta, n_saturated=None):
    _is(x, torch.float32); _is(codes, torch.int32); _is(meta, torch.float32)
    _packed_ok(codes, meta, x.numel(), bits, bucket)
    if n_saturated is not None:
        _is(n_saturated, torch.int64)
    with torch.cuda.device(x.device):
        _check(lib().qsdp_quantize_weight_ex(_ptr(x), x.numel(), bits, bucket, delta, seed, flags, _ptr(codes),
                                             _ptr(meta), _ptr(n_saturated), _stream(x)),
               "qsdp_quantize_weight_ex")


def qsdp_fused_step_ex(x, g, lr, wbits, gbits, bucket, delta, seed, index_offset, flags, wcodes=None,
                       wmeta=None, n_saturated=None):
    _is(x, torch.float32); _is(g, torch.float32)
    if g.numel() != x.numel():
        raise ValueError("x and g differ in size")
    for t, dt in ((wcodes, torch.int32), (wmeta, torch.float32), (n_saturated, torch.int64)):
        if t is not None:
            _is(t, dt)
    _packed_ok(wcodes, wmeta, x.numel(), wbits, bucket)
    with torch.cuda.device(x.device):
        _check(lib().qsdp_fused_step_ex(_ptr(x), _ptr(g), x.numel(), lr, wbits, gbits, bucket, delta, seed,
                                        index_offset, flags, _ptr(wcodes), _ptr(wmeta), _ptr(n_saturated),
                                        _stream(x)), "qsdp_fused_step_ex")


def qsdp_quantize_weight(x, bits, bucket, delta, seed, codes, meta, n_saturated=None):
    _is(x, torch.float32); _is(codes, torch.int32); _is(meta, torch.float32)
    _packed_ok(codes, meta, x.numel(), bits, bucket)
    if n_saturated is not None:
        _is(n_saturated, torch.int64)
    with torch.cuda.device(x.device):
        _check(lib().qsdp_quantize_weight(_ptr(x), x.numel(), bits, bucket, delta, seed, _ptr(codes),
                                          _ptr(meta), _ptr(n_saturated), _stream(x)),
               "qsdp_quantize_weight")


def qsdp_dequantize(codes, meta, n, bits, bucket, out):
    _is(codes, torch.int32); _is(meta, torch.float32)
    dt = _out_dtype(out)
    _is(out, out.dtype)
    if out.numel() < n:
        raise ValueError("out is too small")
    _packed_ok(codes, meta, n, bits, bucket)
    with torch.cuda.device(out.device):
        _check(lib().qsdp_dequantize(_ptr(codes), _ptr(meta), n, bits, bucket, dt, _ptr(out),
                                     _stream(out)), "qsdp_dequantize")


def levels_uniform(bits, device):
    """The uniform starting table k/(2^bits-1) as a device tensor."""
    import numpy as np
    host = np.zeros(1 << bits, dtype=np.float32)
    _check(lib().qsdp_levels_uniform(bits, host.ctypes.data_as(C.c_void_p)), "qsdp_levels_uniform")
    return torch.from_numpy(host).to(device)


def qsdp_quantize_levels(v, bits, bucket, levels, codes, meta):
    _is(v, torch.float32); _is(levels, torch.float32); _is(codes, torch.int32); _is(meta, torch.float32)
    if levels.numel() != (1 << bits):
        raise ValueError("levels must hold 2^bits entries")
    _packed_ok(codes, meta, v.numel(), bits, bucket)
    with torch.cuda.device(v.device):
        _check(lib().qsdp_quantize_levels(_ptr(v), v.numel(), bits, bucket, _ptr(levels), _ptr(codes), _ptr(meta),
                                          _stream(v)), "qsdp_quantize_levels")


def qsdp_quantize_levels_stochastic(v, bits, bucket, levels, seed, index_offset, codes, meta):
    _is(v, torch.float32); _is(levels, torch.float32); _is(codes, torch.int32); _is(meta, torch.float32)
    if levels.numel() != (1 << bits):
        raise ValueError("levels must hold 2^bits entries")
    _packed_ok(codes, meta, v.numel(), bits, bucket)
    with torch.cuda.device(v.device):
        _check(lib().qsdp_quantize_levels_stochastic(_ptr(v), v.numel(), bits, bucket, _ptr(levels), seed,
                                                     index_offset, _ptr(codes), _ptr(meta), _stream(v)),
               "qsdp_quantize_levels_stochastic")


def qsdp_dequantize_levels(codes, meta, n, bits, bucket, levels, out):
    _is(codes, torch.int32); _is(meta, torch.float32); _is(levels, torch.float32)
    if levels.numel() != (1 << bits):
        raise ValueError("levels must hold 2^bits entries")
    dt = _out_dtype(out)
    _is(out, out.dtype)
    if out.numel() < n:
        raise ValueError("out is too small")
    _packed_ok(codes, meta, n, bits, bucket)
    with torch.cuda.device(out.device):
        _check(lib().qsdp_dequantize_levels(_ptr(codes), _ptr(meta), n, bits, bucket, _ptr(levels), dt, _ptr(out),
                                            _stream(out)), "qsdp_dequantize_levels")


def qsdp_fit_levels(v, bits, bucket, lr, levels, max_batches=0):
    _is(v, torch.float32); _is(levels, torch.float32)
    if levels.numel() != (1 << bits):
        raise ValueError("levels must hold 2^bits entries")
    with torch.cuda.device(v.device):
        _check(lib().qsdp_fit_levels(_ptr(v), v.numel(), bits, bucket, lr, max_batches, _ptr(levels), _stream(v)),
               "qsdp_fit_levels")


def qsdp_dequantize_add(codes, meta, npeers, n, bits, bucket, alpha, out):
    """codes int32[npeers, words], meta float32[npeers, nb*2] (row p = peer p's slice)."""
    _is(codes, torch.int32); _is(meta, torch.float32); _is(out, torch.float32)
    if codes.dim() != 2 or meta.dim() != 2 or codes.shape[0] != npeers or meta.shape[0] != npeers:
        raise ValueError("codes and meta must be [npeers, ...]")
    if out.numel() < n:
        raise ValueError("out is too small")
    _rows_ok(codes, meta, n, bits, bucket)
    with torch.cuda.device(out.device):
        _check(lib().qsdp_dequantize_add(_ptr(codes), codes.stride(0) * 4, _ptr(meta), meta.stride(0) * 4,
                                         npeers, n, bits, bucket, alpha, _ptr(out), _stream(out)),
               "qsdp_dequantize_add")


def qsdp_fused_step(x, g, lr, wbits, gbits, bucket, delta, seed, index_offset=0, wcodes=None,
                    wmeta=None, n_saturated=None):
    _is(x, torch.float32); _is(g, torch.float32)
    if g.numel() != x.numel():
        raise ValueError("x and g differ in size")
    if wcodes is not None:
        _is(wcodes, torch.int32)
    if wmeta is not None:
        _is(wmeta, torch.float32)
    if n_saturated is not None:
        _is(n_saturated, torch.int64)
    _packed_ok(wcodes, wmeta, x.numel(), wbits, bucket)
    with torch.cuda.device(x.device):
        _check(lib().qsdp_fused_step(_ptr(x), _ptr(g), x.numel(), lr, wbits, gbits, bucket, delta, seed,
                                     index_offset, _ptr(wcodes), _ptr(wmeta), _ptr(n_saturated),
                                     _stream(x)), "qsdp_fused_step")


def qsdp_fused_adamw_step(x, g, m, v, lr, beta1, beta2, eps, weight_decay, bias1, bias2, wbits, gbits, bucket,
                          delta, seed, index_offset=0, flags=0, wcodes=None, wmeta=None, n_saturated=None):
    for t in (x, g, m, v):
        _is(t, torch.float32)
    if not (g.numel() == x.numel() == m.numel() == v.numel()):
        raise ValueError("x, g, m, v differ in size")
    for t, dt in ((wcodes, torch.int32), (wmeta, torch.float32), (n_saturated, torch.int64)):
        if t is not None:
            _is(t, dt)
    _packed_ok(wcodes, wmeta, x.numel(), wbits, bucket)
    with torch.cuda.device(x.device):
        _check(lib().qsdp_fused_adamw_step(_ptr(x), _ptr(g), _ptr(m), _ptr(v), x.numel(), lr, beta1, beta2, eps,
                                           weight_decay, bias1, bias2, wbits, gbits, bucket, delta, seed,
                                           index_offset, flags, _ptr(wcodes), _ptr(wmeta), _ptr(n_saturated),
                                           _stream(x)), "qsdp_fused_adamw_step")


def qsdp_fused_step_codes(wcodes, wmeta, g, lr, wbits, gbits, bucket, delta, seed, index_offset=0,
                          n_saturated=None, flags=0):
    _is(wcodes, torch.int32); _is(wmeta, torch.float32); _is(g, torch.float32)
    if n_saturated is not None:
        _is(n_saturated, torch.int64)
    _packed_ok(wcodes, wmeta, g.numel(), wbits, bucket)
    with torch.cuda.device(g.device):
        _check(lib().qsdp_fused_step_codes(_ptr(wcodes), _ptr(wmeta), _ptr(g), g.numel(), lr, wbits, gbits,
                                           bucket, delta, seed, index_offset, flags, _ptr(n_saturated),
                                           _stream(g)), "qsdp_fused_step_codes")


class Segments:
    """Host table built by qsdp_segments_build plus its device copy (an int64 tensor holding the
    {offset, n, first_bucket} triples)."""

    def __init__(self, sizes, bucket, device):
        import numpy as np
        sizes_np = np.ascontiguousarray(sizes, dtype=np.uint64)
        self.nseg = int(sizes_np.size)
        self.bucket = int(bucket)
        self.host = np.zeros((self.nseg, 3), dtype=np.uint64)
        self.total_buckets = int(lib().qsdp_segments_build(
            sizes_np.ctypes.data_as(C.c_void_p), self.nseg, self.bucket, self.host.ctypes.data_as(C.c_void_p)))
        if self.total_buckets == 0:
            raise QsdpError(QSDP_EINVAL, "qsdp_segments_build")
        self.n = int(sizes_np.sum())
        self.device = torch.from_numpy(self.host.view(np.int64).copy()).to(device)

    def check_packed(self, codes, meta, bits, rows=False):
        """codes / meta (or every row of them, for per-peer buffers) cover all buckets of the table."""
        words, floats = self.total_buckets * self.bucket * bits // 32, 2 * self.total_buckets
        for t, need, what in ((codes, words, "codes"), (meta, floats, "meta")):
            if t is None:
                continue
            have = t.shape[1] if rows else t.numel()
            if have < need:
                raise ValueError(f"{what} holds {have} elements{' per row' if rows else ''}, {need} are needed")

    def alloc_packed(self, bits):
        cb = self.total_buckets * self.bucket * bits // 8
        codes = torch.empty(cb // 4, dtype=torch.int32, device=self.device.device)
        meta = torch.empty((self.total_buckets, 2), dtype=torch.float32, device=self.device.device)
        return codes, meta


def qsdp_quantize_grad_segmented(g, segs, bits, seed, index_offset, codes, meta):
    _is(g, torch.float32); _is(codes, torch.int32); _is(meta, torch.float32)
    if g.numel() < segs.n:
        raise ValueError("g is smaller than the segments")
    segs.check_packed(codes, meta, bits)
    with torch.cuda.device(g.device):
        _check(lib().qsdp_quantize_grad_segmented(_ptr(g), _ptr(segs.device), segs.nseg, segs.total_buckets,
                                                  bits, segs.bucket, seed, index_offset, _ptr(codes),
                                                  _ptr(meta), _stream(g)), "qsdp_quantize_grad_segmented")


def qsdp_quantize_weight_segmented(x, segs, bits, delta, seed, codes, meta, n_saturated=None):
    _is(x, torch.float32); _is(codes, torch.int32); _is(meta, torch.float32)
    if x.numel() < segs.n:
        raise ValueError("x is smaller than the segments")
    if n_saturated is not None:
        _is(n_saturated, torch.int64)
    segs.check_packed(codes, meta, bits)
    with torch.cuda.device(x.device):
        _check(lib().qsdp_quantize_weight_segmented(_ptr(x), _ptr(segs.device), segs.nseg,
                                                    segs.total_buckets, bits, segs.bucket, delta, seed,
                                                    _ptr(codes), _ptr(meta), _ptr(n_saturated), _stream(x)),
               "qsdp_quantize_weight_segmented")


def qsdp_fused_step_segmented(x, g, segs, lr, wbits, gbits, delta, seed, index_offset=0, wcodes=None,
                              wmeta=None, n_saturated=None):
    _is(x, torch.float32); _is(g, torch.float32)
    if x.numel() < segs.n or g.numel() < segs.n:
        raise ValueError("x or g is smaller than the segments")
    if wcodes is not None:
        _is(wcodes, torch.int32)
    if wmeta is not None:
        _is(wmeta, torch.float32)
    if n_saturated is not None:
        _is(n_saturated, torch.int64)
    segs.check_packed(wcodes, wmeta, wbits)
    with torch.cuda.device(x.device):
        _check(lib().qsdp_fused_step_segmented(_ptr(x), _ptr(g), _ptr(segs.device), segs.nseg,
                                               segs.total_buckets, lr, wbits, gbits, segs.bucket, delta,
                                               seed, index_offset, _ptr(wcodes), _ptr(wmeta),
                                               _ptr(n_saturated), _stream(x)), "qsdp_fused_step_segmented")


def qsdp_dequantize_segmented(codes, meta, segs, bits, out):
    _is(codes, torch.int32); _is(meta, torch.float32)
    dt = _out_dtype(out)
    _is(out, out.dtype)
    if out.numel() < segs.n:
        raise ValueError("out is smaller than the segments")
    if codes.numel() * 32 < segs.total_buckets * segs.bucket * bits or meta.numel() < 2 * segs.total_buckets:
        raise ValueError("codes or meta is smaller than the segments")
    with torch.cuda.device(out.device):
        _check(lib().qsdp_dequantize_segmented(_ptr(codes), _ptr(meta), _ptr(segs.device), segs.nseg,
                                               segs.total_buckets, bits, segs.bucket, dt, _ptr(out),
                                               _stream(out)), "qsdp_dequantize_segmented")


def qsdp_dequantize_gathered(codes, meta, npeers, n, shard, bits, bucket, out, levels=None):
    """codes int32[npeers, >= words of a shard], meta float32[npeers, >= 2 * buckets of a shard]
    (row p = peer p's slot; rows may be views into one receive buffer); out float32/bfloat16[n].
    levels: the table the slots were encoded with by qsdp_quantize_levels, or None for uniform codes."""
    _is_rows(codes, torch.int32); _is_rows(meta, torch.float32)
    dt = _out_dtype(out)
    _is(out, out.dtype)
    if codes.shape[0] != npeers or meta.shape[0] != npeers:
        raise ValueError("codes and meta must be [npeers, ...]")
    if out.numel() < n:
        raise ValueError("out is too small")
    _rows_ok(codes, meta, min(n, shard) if shard > 0 else n, bits, bucket)
    with torch.cuda.device(out.device):
        if levels is not None:
            _is(levels, torch.float32)
            if levels.numel() != (1 << bits):
                raise ValueError("levels must hold 2^bits entries")
            _check(lib().qsdp_dequantize_levels_gathered(_ptr(codes), codes.stride(0) * 4, _ptr(meta),
                                                         meta.stride(0) * 4, npeers, n, shard, bits, bucket,
                                                         _ptr(levels), dt, _ptr(out), _stream(out)),
                   "qsdp_dequantize_levels_gathered")
            return
        _check(lib().qsdp_dequantize_gathered(_ptr(codes), codes.stride(0) * 4, _ptr(meta), meta.stride(0) * 4,
                                              npeers, n, shard, bits, bucket, dt, _ptr(out), _stream(out)),
               "qsdp_dequantize_gathered")


def qsdp_recv_step(x, gcodes, gmeta, npeers, alpha, lr, wbits, gbits, bucket, delta, seed, flags=0, wcodes=None,
                   wmeta=None, n_saturated=None):
    """gcodes int32[npeers, words], gmeta float32[npeers, nb*2] (row k = peer k's slice)."""
    _is(x, torch.float32); _is_rows(gcodes, torch.int32); _is_rows(gmeta, torch.float32)
    if gcodes.shape[0] != npeers or gmeta.shape[0] != npeers:
        raise ValueError("gcodes and gmeta must be [npeers, ...]")
    for t, dt in ((wcodes, torch.int32), (wmeta, torch.float32), (n_saturated, torch.int64)):
        if t is not None:
            _is(t, dt)
    _rows_ok(gcodes, gmeta, x.numel(), gbits, bucket)
    _packed_ok(wcodes, wmeta, x.numel(), wbits, bucket)
    with torch.cuda.device(x.device):
        _check(lib().qsdp_recv_step(_ptr(x), _ptr(gcodes), gcodes.stride(0) * 4, _ptr(gmeta), gmeta.stride(0) * 4,
                                    npeers, x.numel(), alpha, lr, wbits, gbits, bucket, delta, seed, flags,
                                    _ptr(wcodes), _ptr(wmeta), _ptr(n_saturated), _stream(x)), "qsdp_recv_step")


def qsdp_recv_adamw_step(x, m, v, gcodes, gmeta, npeers, alpha, lr, beta1, beta2, eps, weight_decay, bias1, bias2,
                         wbits, gbits, bucket, delta, seed, flags=0, wcodes=None, wmeta=None, n_saturated=None):
    """As qsdp_recv_step with the AdamW update; m, v float32[n] moment estimates, updated in place."""
    for t in (x, m, v):
        _is(t, torch.float32)
    if not (x.numel() == m.numel() == v.numel()):
        raise ValueError("x, m, v differ in size")
    _is_rows(gcodes, torch.int32); _is_rows(gmeta, torch.float32)
    if gcodes.shape[0] != npeers or gmeta.shape[0] != npeers:
        raise ValueError("gcodes and gmeta must be [npeers, ...]")
    for t, dt in ((wcodes, torch.int32), (wmeta, torch.float32), (n_saturated, torch.int64)):
        if t is not None:
            _is(t, dt)
    _rows_ok(gcodes, gmeta, x.numel(), gbits, bucket)
    _packed_ok(wcodes, wmeta, x.numel(), wbits, bucket)
    with torch.cuda.device(x.device):
        _check(lib().qsdp_recv_adamw_step(_ptr(x), _ptr(m), _ptr(v), _ptr(gcodes), gcodes.stride(0) * 4, _ptr(gmeta),
                                          gmeta.stride(0) * 4, npeers, x.numel(), alpha, lr, beta1, beta2, eps,
                                          weight_decay, bias1, bias2, wbits, gbits, bucket, delta, seed, flags,
                                          _ptr(wcodes), _ptr(wmeta), _ptr(n_saturated), _stream(x)),
               "qsdp_recv_adamw_step")


def qsdp_recv_step_segmented(x, segs, gcodes, gmeta, npeers, alpha, lr, wbits, gbits, delta, seed, flags=0,
                             wcodes=None, wmeta=None, n_saturated=None, adamw=None):
    """The receive-side step over the tensors of `segs` in one launch. adamw: None, or
    (m, v, beta1, beta2, eps, weight_decay, bias1, bias2) for the AdamW form."""
    _is(x, torch.float32); _is_rows(gcodes, torch.int32); _is_rows(gmeta, torch.float32)
    if x.numel() < segs.n:
        raise ValueError("x is smaller than the segments")
    if gcodes.shape[0] != npeers or gmeta.shape[0] != npeers:
        raise ValueError("gcodes and gmeta must be [npeers, ...]")
    for t, dt in ((wcodes, torch.int32), (wmeta, torch.float32), (n_saturated, torch.int64)):
        if t is not None:
            _is(t, dt)
    segs.check_packed(gcodes, gmeta, gbits, rows=True)
    segs.check_packed(wcodes, wmeta, wbits)
    with torch.cuda.device(x.device):
        if adamw is None:
            _check(lib().qsdp_recv_step_segmented(_ptr(x), _ptr(segs.device), segs.nseg, segs.total_buckets,
                                                  _ptr(gcodes), gcodes.stride(0) * 4, _ptr(gmeta),
                                                  gmeta.stride(0) * 4, npeers, alpha, lr, wbits, gbits, segs.bucket,
                                                  delta, seed, flags, _ptr(wcodes), _ptr(wmeta), _ptr(n_saturated),
                                                  _stream(x)), "qsdp_recv_step_segmented")
        else:
            m, v, b1, b2, eps, wd, c1, c2 = adamw
            _is(m, torch.float32); _is(v, torch.float32)
            if m.numel() < segs.n or v.numel() < segs.n:
                raise ValueError("m or v is smaller than the segments")
            _check(lib().qsdp_recv_adamw_step_segmented(_ptr(x), _ptr(m), _ptr(v), _ptr(segs.device), segs.nseg,
                                                        segs.total_buckets, _ptr(gcodes), gcodes.stride(0) * 4,
                                                        _ptr(gmeta), gmeta.stride(0) * 4, npeers, alpha, lr, b1, b2,
                                                        eps, wd, c1, c2, wbits, gbits, segs.bucket, delta, seed, flags,
                                                        _ptr(wcodes), _ptr(wmeta), _ptr(n_saturated), _stream(x)),
                   "qsdp_recv_adamw_step_segmented")


def qsdp_fused_adamw_step_segmented(x, g, m, v, segs, lr, beta1, beta2, eps, weight_decay, bias1, bias2, wbits, gbits,
                                    delta, seed, index_offset=0, flags=0, wcodes=None, wmeta=None, n_saturated=None):
    for t in (x, g, m, v):
        _is(t, torch.float32)
        if t.numel() < segs.n:
            raise ValueError("a tensor is smaller than the segments")
    for t, dt in ((wcodes, torch.int32), (wmeta, torch.float32), (n_saturated, torch.int64)):
        if t is not None:
            _is(t, dt)
    segs.check_packed(wcodes, wmeta, wbits)
    with torch.cuda.device(x.device):
        _check(lib().qsdp_fused_adamw_step_segmented(_ptr(x), _ptr(g), _ptr(m), _ptr(v), _ptr(segs.device), segs.nseg,
                                                     segs.total_buckets, lr, beta1, beta2, eps, weight_decay, bias1,
                                                     bias2, wbits, gbits, segs.bucket, delta, seed, index_offset, flags,
                                                     _ptr(wcodes), _ptr(wmeta), _ptr(n_saturated), _stream(x)),
               "qsdp_fused_adamw_step_segmented")


def qsdp_fused_step_codes_segmented(wcodes, wmeta, g, segs, lr, wbits, gbits, delta, seed, index_offset=0, flags=0,
                                    n_saturated=None):
    _is(wcodes, torch.int32); _is(wmeta, torch.float32); _is(g, torch.float32)
    if g.numel() < segs.n:
        raise ValueError("g is smaller than the segments")
    if n_saturated is not None:
        _is(n_saturated, torch.int64)
    segs.check_packed(wcodes, wmeta, wbits)
    with torch.cuda.device(g.device):
        _check(lib().qsdp_fused_step_codes_segmented(_ptr(wcodes), _ptr(wmeta), _ptr(g), _ptr(segs.device), segs.nseg,
                                                     segs.total_buckets, lr, wbits, gbits, segs.bucket, delta, seed,
                                                     index_offset, flags, _ptr(n_saturated), _stream(g)),
               "qsdp_fused_step_codes_segmented")


def qsdp_fit_levels_segmented(v, segs, bits, lr, levels, max_batches=0):
    """levels float32[nseg, 2^bits]: row t is the start table of tensor t and receives its fitted levels."""
    _is(v, torch.float32); _is(levels, torch.float32)
    if v.numel() < segs.n:
        raise ValueError("v is smaller than the segments")
    if levels.numel() != segs.nseg * (1 << bits):
        raise ValueError("levels must hold nseg * 2^bits entries")
    with torch.cuda.device(v.device):
        _check(lib().qsdp_fit_levels_segmented(_ptr(v), _ptr(segs.device), segs.nseg, bits, segs.bucket, lr,
                                               max_batches, _ptr(levels), _stream(v)), "qsdp_fit_levels_segmented")


def qsdp_fused_step_dseed(x, g, lr, wbits, gbits, bucket, delta, seed, seed_dev, index_offset=0, flags=0, wcodes=None,
                          wmeta=None, n_saturated=None):
    """qsdp_fused_step_ex with the seed in force = seed + seed_dev[0] (an int64 GPU tensor read by the
    kernel), so that a step captured in a graph can be replayed with an advancing seed."""
    _is(x, torch.float32); _is(g, torch.float32); _is(seed_dev, torch.int64)
    if g.numel() != x.numel():
        raise ValueError("x and g differ in size")
    for t, dt in ((wcodes, torch.int32), (wmeta, torch.float32), (n_saturated, torch.int64)):
        if t is not None:
            _is(t, dt)
    _packed_ok(wcodes, wmeta, x.numel(), wbits, bucket)
    with torch.cuda.device(x.device):
        _check(lib().qsdp_fused_step_dseed(_ptr(x), _ptr(g), x.numel(), lr, wbits, gbits, bucket, delta, seed,
                                           _ptr(seed_dev), index_offset, flags, _ptr(wcodes), _ptr(wmeta),
                                           _ptr(n_saturated), _stream(x)), "qsdp_fused_step_dseed")


def qsdp_quantize_levels_segmented(v, segs, bits, levels, codes, meta, stochastic=False, seed=0, index_offset=0):
    """levels float32[nseg, 2^bits]: row t is the level table of tensor t."""
    _is(v, torch.float32); _is(levels, torch.float32); _is(codes, torch.int32); _is(meta, torch.float32)
    if v.numel() < segs.n:
        raise ValueError("v is smaller than the segments")
    if levels.numel() != segs.nseg * (1 << bits):
        raise ValueError("levels must hold nseg * 2^bits entries")
    segs.check_packed(codes, meta, bits)
    with torch.cuda.device(v.device):
        _check(lib().qsdp_quantize_levels_segmented(_ptr(v), _ptr(segs.device), segs.nseg, segs.total_buckets, bits,
                                                    segs.bucket, _ptr(levels), int(bool(stochastic)), seed,
                                                    index_offset, _ptr(codes), _ptr(meta), _stream(v)),
               "qsdp_quantize_levels_segmented")


def qsdp_dequantize_levels_segmented(codes, meta, segs, bits, levels, out):
    _is(codes, torch.int32); _is(meta, torch.float32); _is(levels, torch.float32)
    dt = _out_dtype(out)
    _is(out, out.dtype)
    if out.numel() < segs.n:
        raise ValueError("out is smaller than the segments")
    if levels.numel() != segs.nseg * (1 << bits):
        raise ValueError("levels must hold nseg * 2^bits entries")
    segs.check_packed(codes, meta, bits)
    with torch.cuda.device(out.device):
        _check(lib().qsdp_dequantize_levels_segmented(_ptr(codes), _ptr(meta), _ptr(segs.device), segs.nseg,
                                                      segs.total_buckets, bits, segs.bucket, _ptr(levels), dt,
                                                      _ptr(out), _stream(out)), "qsdp_dequantize_levels_segmented")



_G16 = {torch.bfloat16: 1, torch.float16: 2}


def qsdp_quantize_grad_g16(g, bits, bucket, seed, index_offset, codes, meta, flags=0):
    """qsdp_quantize_grad_ex on a float16 or bfloat16 gradient (widened exactly to float32 inside the kernel)."""
    if g.dtype not in _G16:
        raise TypeError("g must be float16 or bfloat16")
    _is(g, g.dtype); _is(codes, torch.int32); _is(meta, torch.float32)
    _packed_ok(codes, meta, g.numel(), bits, bucket)
    with torch.cuda.device(g.device):
        _check(lib().qsdp_quantize_grad_g16(_ptr(g), _G16[g.dtype], g.numel(), bits, bucket, seed, index_offset, flags,
                                            _ptr(codes), _ptr(meta), _stream(g)), "qsdp_quantize_grad_g16")


def qsdp_fused_step_g16(x, g, lr, wbits, gbits, bucket, delta, seed, index_offset=0, flags=0, wcodes=None, wmeta=None,
                        n_saturated=None):
    """qsdp_fused_step_ex with a float16 or bfloat16 gradient (widened exactly to float32 inside the kernel)."""
    if g.dtype not in _G16:
        raise TypeError("g must be float16 or bfloat16")
    _is(x, torch.float32); _is(g, g.dtype)
    if g.numel() != x.numel():
        raise ValueError("x and g differ in size")
    for t, dt in ((wcodes, torch.int32), (wmeta, torch.float32), (n_saturated, torch.int64)):
        if t is not None:
            _is(t, dt)
    _packed_ok(wcodes, wmeta, x.numel(), wbits, bucket)
    with torch.cuda.device(x.device):
        _check(lib().qsdp_fused_step_g16(_ptr(x), _ptr(g), _G16[g.dtype], x.numel(), lr, wbits, gbits, bucket, delta,
                                         seed, index_offset, flags, _ptr(wcodes), _ptr(wmeta), _ptr(n_saturated),
                                         _stream(x)), "qsdp_fused_step_g16")


def qsdp_fused_adamw_step_codes(wcodes, wmeta, g, m, v, lr, beta1, beta2, eps, weight_decay, bias1, bias2, wbits, gbits,
                                bucket, delta, seed, index_offset=0, flags=0, n_saturated=None):
    """The AdamW step on weights held as packed codes + meta (updated in place); m, v float32, updated in place."""
    _is(wcodes, torch.int32); _is(wmeta, torch.float32); _is(g, torch.float32); _is(m, torch.float32)
    _is(v, torch.float32)
    n = g.numel()
    if m.numel() != n or v.numel() != n:
        raise ValueError("g, m and v differ in size")
    if n_saturated is not None:
        _is(n_saturated, torch.int64)
    _packed_ok(wcodes, wmeta, n, wbits, bucket)
    with torch.cuda.device(g.device):
        _check(lib().qsdp_fused_adamw_step_codes(_ptr(wcodes), _ptr(wmeta), _ptr(g), _ptr(m), _ptr(v), n, lr, beta1,
                                                 beta2, eps, weight_decay, bias1, bias2, wbits, gbits, bucket, delta,
                                                 seed, index_offset, flags, _ptr(n_saturated), _stream(g)),
               "qsdp_fused_adamw_step_codes")


def qsdp_fused_step_mp(x, g, lr, wbits, gbits, bucket, delta, seed, index_offset=0, flags=0, wcodes=None, wmeta=None,
                       x16=None, n_saturated=None):
    """The fused step with a float32 / float16 / bfloat16 gradient and, optionally, the new quantized weights
    written once more as float16 / bfloat16 into x16."""
    gdt = {torch.float32: QSDP_F32, torch.bfloat16: QSDP_BF16, torch.float16: QSDP_F16}.get(g.dtype)
    if gdt is None:
        raise TypeError("g must be float32, float16 or bfloat16")
    _is(x, torch.float32); _is(g, g.dtype)
    if g.numel() != x.numel():
        raise ValueError("x and g differ in size")
    xdt = QSDP_BF16
    if x16 is not None:
        if x16.dtype not in _G16:
            raise TypeError("x16 must be float16 or bfloat16")
        _is(x16, x16.dtype)
        _need(x16, x.numel(), "x16")
        xdt = _G16[x16.dtype]
    for t, dt in ((wcodes, torch.int32), (wmeta, torch.float32), (n_saturated, torch.int64)):
        if t is not None:
            _is(t, dt)
    _packed_ok(wcodes, wmeta, x.numel(), wbits, bucket)
    with torch.cuda.device(x.device):
        _check(lib().qsdp_fused_step_mp(_ptr(x), _ptr(g), gdt, x.numel(), lr, wbits, gbits, bucket, delta, seed,
                                        index_offset, flags, _ptr(wcodes), _ptr(wmeta), _ptr(x16), xdt,
                                        _ptr(n_saturated), _stream(x)), "qsdp_fused_step_mp")


def qsdp_fused_step_segmented_mp(x, g, segs, lr, wbits, gbits, delta, seed, index_offset=0, flags=0, wcodes=None,
                                 wmeta=None, x16=None, n_saturated=None):
    """qsdp_fused_step_mp over the tensors of a segment table, one launch."""
    gdt = {torch.float32: QSDP_F32, torch.bfloat16: QSDP_BF16, torch.float16: QSDP_F16}.get(g.dtype)
    if gdt is None:
        raise TypeError("g must be float32, float16 or bfloat16")
    _is(x, torch.float32); _is(g, g.dtype)
    _need(x, segs.n, "x"); _need(g, segs.n, "g")
    xdt = QSDP_BF16
    if x16 is not None:
        if x16.dtype not in _G16:
            raise TypeError("x16 must be float16 or bfloat16")
        _is(x16, x16.dtype)
        _need(x16, segs.n, "x16")
        xdt = _G16[x16.dtype]
    for t, dt in ((wcodes, torch.int32), (wmeta, torch.float32), (n_saturated, torch.int64)):
        if t is not None:
            _is(t, dt)
    segs.check_packed(wcodes, wmeta, wbits)
    with torch.cuda.device(x.device):
        _check(lib().qsdp_fused_step_segmented_mp(_ptr(x), _ptr(g), gdt, _ptr(segs.device), segs.nseg,
                                                  segs.total_buckets, lr, wbits, gbits, segs.bucket, delta, seed,
                                                  index_offset, flags, _ptr(wcodes), _ptr(wmeta), _ptr(x16), xdt,
                                                  _ptr(n_saturated), _stream(x)), "qsdp_fused_step_segmented_mp")


def qsdp_fused_adamw_step_mp(x, g, m, v, lr, beta1, beta2, eps, weight_decay, bias1, bias2, wbits, gbits, bucket, delta,
                             seed, index_offset=0, flags=0, wcodes=None, wmeta=None, x16=None, n_saturated=None):
    """qsdp_fused_adamw_step with a float32 / float16 / bfloat16 gradient and an optional float16 / bfloat16
    copy x16 of the new quantized weights."""
    gdt = {torch.float32: QSDP_F32, torch.bfloat16: QSDP_BF16, torch.float16: QSDP_F16}.get(g.dtype)
    if gdt is None:
        raise TypeError("g must be float32, float16 or bfloat16")
    _is(x, torch.float32); _is(g, g.dtype); _is(m, torch.float32); _is(v, torch.float32)
    n = x.numel()
    if g.numel() != n or m.numel() != n or v.numel() != n:
        raise ValueError("x, g, m and v differ in size")
    xdt = QSDP_BF16
    if x16 is not None:
        if x16.dtype not in _G16:
            raise TypeError("x16 must be float16 or bfloat16")
        _is(x16, x16.dtype)
        _need(x16, n, "x16")
        xdt = _G16[x16.dtype]
    for t, dt in ((wcodes, torch.int32), (wmeta, torch.float32), (n_saturated, torch.int64)):
        if t is not None:
            _is(t, dt)
    _packed_ok(wcodes, wmeta, n, wbits, bucket)
    with torch.cuda.device(x.device):
        _check(lib().qsdp_fused_adamw_step_mp(_ptr(x), _ptr(g), gdt, _ptr(m), _ptr(v), n, lr, beta1, beta2, eps,
                                              weight_decay, bias1, bias2, wbits, gbits, bucket, delta, seed,
                                              index_offset, flags, _ptr(wcodes), _ptr(wmeta), _ptr(x16), xdt,
                                              _ptr(n_saturated), _stream(x)), "qsdp_fused_adamw_step_mp")


class StepOptions(C.Structure):
    """qsdp_step_options of include/qsdp.h, field for field."""
    _fields_ = [("size", C.c_uint32), ("flags", C.c_uint32), ("g_dtype", C.c_int), ("x16_dtype", C.c_int),
                ("x16", C.c_void_p), ("segments", C.c_void_p), ("nseg", C.c_uint32), ("reserved", C.c_uint32),
                ("total_buckets", C.c_uint64), ("seed_increment", C.c_void_p), ("wcodes", C.c_void_p),
                ("wmeta", C.c_void_p), ("n_saturated", C.c_void_p), ("m", C.c_void_p), ("v", C.c_void_p),
                ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float), ("weight_decay", C.c_float),
                ("bias1", C.c_float), ("bias2", C.c_float)]


def _step_opts(entry, x, g, lr, wbits, gbits, bucket, delta, seed, index_offset, flags, segs, x16, seed_increment,
               wcodes, wmeta, n_saturated, adamw):
    gdt = {torch.float32: QSDP_F32, torch.bfloat16: QSDP_BF16, torch.float16: QSDP_F16}.get(g.dtype)
    if gdt is None:
        raise TypeError("g must be float32, float16 or bfloat16")
    _is(x, torch.float32); _is(g, g.dtype)
    n = x.numel() if segs is None else segs.n
    if x.numel() < n or g.numel() < n or (segs is None and g.numel() != n):
        raise ValueError("x and g do not cover the elements of the call")
    o = StepOptions()
    o.size = C.sizeof(StepOptions)
    o.flags = flags
    o.g_dtype = gdt
    if x16 is not None:
        if x16.dtype not in _G16:
            raise TypeError("x16 must be float16 or bfloat16")
        _is(x16, x16.dtype)
        _need(x16, n, "x16")
        o.x16, o.x16_dtype = x16.data_ptr(), _G16[x16.dtype]
    for t, dt in ((wcodes, torch.int32), (wmeta, torch.float32), (n_saturated, torch.int64),
                  (seed_increment, torch.int64)):
        if t is not None:
            _is(t, dt)
    if segs is None:
        _packed_ok(wcodes, wmeta, n, wbits, bucket)
    else:
        if bucket != segs.bucket:
            raise ValueError("bucket differs from the segment table's")
        segs.check_packed(wcodes, wmeta, wbits)
        o.segments, o.nseg, o.total_buckets = segs.device.data_ptr(), segs.nseg, segs.total_buckets
    for name, t in (("wcodes", wcodes), ("wmeta", wmeta), ("n_saturated", n_saturated),
                    ("seed_increment", seed_increment)):
        if t is not None:
            setattr(o, name, t.data_ptr())
    if adamw is not None:
        m, v, o.beta1, o.beta2, o.eps, o.weight_decay, o.bias1, o.bias2 = adamw
        _is(m, torch.float32); _is(v, torch.float32)
        _need(m, n, "m"); _need(v, n, "v")
        o.m, o.v = m.data_ptr(), v.data_ptr()
    with torch.cuda.device(x.device):
        _check(getattr(lib(), entry)(_ptr(x), _ptr(g), 0 if segs is not None else n, lr, wbits, gbits, bucket, delta,
                                     seed, index_offset, C.byref(o), _stream(x)), entry)


def qsdp_fused_step_opts(x, g, lr, wbits, gbits, bucket, delta, seed, index_offset=0, flags=0, segs=None, x16=None,
                         seed_increment=None, wcodes=None, wmeta=None, n_saturated=None):
    """The fused step with its optional parts in one options block (qsdp_step_options): gradient in float32 /
    float16 / bfloat16 (taken from g's dtype), a segment table, a 16-bit copy of the new weights, a device-resident
    seed increment, code output, the saturation counter."""
    _step_opts("qsdp_fused_step_opts", x, g, lr, wbits, gbits, bucket, delta, seed, index_offset, flags, segs, x16,
               seed_increment, wcodes, wmeta, n_saturated, None)


def qsdp_fused_adamw_step_opts(x, g, m, v, lr, beta1, beta2, eps, weight_decay, bias1, bias2, wbits, gbits, bucket,
                               delta, seed, index_offset=0, flags=0, segs=None, x16=None, seed_increment=None,
                               wcodes=None, wmeta=None, n_saturated=None):
    """The same with AdamW (moments m, v in float32, updated in place) between the two quantizers."""
    _step_opts("qsdp_fused_adamw_step_opts", x, g, lr, wbits, gbits, bucket, delta, seed, index_offset, flags, segs,
               x16, seed_increment, wcodes, wmeta, n_saturated, (m, v, beta1, beta2, eps, weight_decay, bias1, bias2))


def _one_device(fn):
    """Every tensor argument of an entry point (and a segment table) must live on the same device: the
    kernel runs on the device of the first one and would fault on memory of another."""
    @functools.wraps(fn)
    def checked(*args, **kwargs):
        device = None
        for a in list(args) + list(kwargs.values()):
            for t in (a if isinstance(a, (tuple, list)) else (a,)):
                if isinstance(t, Segments):
                    t = t.device
                if isinstance(t, torch.Tensor):
                    if device is None:
                        device = t.device
                    elif t.device != device:
                        raise ValueError(f"{fn.__name__}: tensors on {device} and on {t.device}")
        return fn(*args, **kwargs)
    return checked


for _name, _fn in list(globals().items()):
    if _name.startswith("qsdp_") and callable(_fn):
        globals()[_name] = _one_device(_fn)
del _name, _fn
