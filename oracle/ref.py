"""ctypes/numpy front end of the CPU oracle (``libqsdp_ref.so``).

TEST INFRASTRUCTURE ONLY: imported by tests, by the smoke check and by the
benchmark's CPU-baseline leg; never by the product package. Every function takes
and returns numpy arrays on the host and holds no arithmetic of its own: the
arithmetic is in ``qsdp_ref.c``.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

F32, BF16, F16 = 0, 1, 2
FLAG_GRAD_SHIFT, FLAG_NO_SHIFT, FLAG_SYMMETRIC, FLAG_KEEP_MASTER = 1, 2, 4, 8

_lib = None


def lib():
    global _lib
    if _lib is None:
        # QSDP_REF_LIB: load another build of the oracle (the mutation tests plant mistakes in
        # copies of the source to show that the pins catch them)
        path = os.environ.get("QSDP_REF_LIB") or _build.build(force=False)
        L = C.CDLL(path)
        u64, i32, f32, vp = C.c_uint64, C.c_int, C.c_float, C.c_void_p
        L.qsdp_ref_set_threads.argtypes = [i32]
        L.qsdp_ref_set_threads.restype = i32
        L.qsdp_ref_philox4x32_10.argtypes = [vp, vp, vp]
        L.qsdp_ref_philox4x32_10.restype = None
        L.qsdp_ref_grad_uniform.argtypes = [u64, u64]
        L.qsdp_ref_grad_uniform.restype = f32
        L.qsdp_ref_weight_shift.argtypes = [u64]
        L.qsdp_ref_weight_shift.restype = f32
        L.qsdp_ref_grad_shift.argtypes = [u64]
        L.qsdp_ref_grad_shift.restype = f32
        u32 = C.c_uint32
        L.qsdp_ref_quantize_grad_u_ex.argtypes = [vp, u64, i32, i32, vp, u32, vp, vp]
        L.qsdp_ref_quantize_weight_xi_ex.argtypes = [vp, u64, i32, i32, f32, f32, u32, vp, vp, vp]
        L.qsdp_ref_quantize_grad_ex.argtypes = [vp, u64, i32, i32, u64, u64, u32, vp, vp]
        L.qsdp_ref_quantize_weight_ex.argtypes = [vp, u64, i32, i32, f32, u64, u32, vp, vp, vp]
        L.qsdp_ref_fused_step_ex.argtypes = [vp, vp, u64, f32, i32, i32, i32, f32, u64, u64, u32, vp, vp, vp]
        L.qsdp_ref_codes_bytes.argtypes = [u64, i32, i32]
        L.qsdp_ref_codes_bytes.restype = C.c_size_t
        L.qsdp_ref_meta_bytes.argtypes = [u64, i32]
        L.qsdp_ref_meta_bytes.restype = C.c_size_t
        L.qsdp_ref_quantize_grad_u.argtypes = [vp, u64, i32, i32, vp, vp, vp]
        L.qsdp_ref_quantize_weight_xi.argtypes = [vp, u64, i32, i32, f32, f32, vp, vp, vp]
        L.qsdp_ref_pack.argtypes = [vp, u64, i32, i32, vp]
        L.qsdp_ref_pack.restype = None
        L.qsdp_ref_unpack.argtypes = [vp, u64, i32, i32, vp]
        L.qsdp_ref_unpack.restype = None
        L.qsdp_ref_f32_to_bf16.argtypes = [f32]
        L.qsdp_ref_f32_to_bf16.restype = C.c_uint16
        L.qsdp_ref_f32_to_f16.argtypes = [f32]
        L.qsdp_ref_f32_to_f16.restype = C.c_uint16
        L.qsdp_ref_quantize_grad.argtypes = [vp, u64, i32, i32, u64, u64, vp, vp]
        L.qsdp_ref_quantize_weight.argtypes = [vp, u64, i32, i32, f32, u64, vp, vp, vp]
        L.qsdp_ref_dequantize.argtypes = [vp, vp, u64, i32, i32, i32, vp]
        L.qsdp_ref_dequantize_add.argtypes = [vp, u64, vp, u64, i32, u64, i32, i32, f32, vp]
        L.qsdp_ref_fused_adamw_step.argtypes = [vp, vp, vp, vp, u64, f32, f32, f32, f32, f32, f32, f32, i32, i32,
                                                i32, f32, u64, u64, u32, vp, vp, vp]
        L.qsdp_ref_levels_uniform.argtypes = [i32, vp]
        L.qsdp_ref_quantize_levels.argtypes = [vp, u64, i32, i32, vp, vp, vp]
        L.qsdp_ref_dequantize_levels.argtypes = [vp, vp, u64, i32, i32, vp, i32, vp]
        L.qsdp_ref_fit_levels.argtypes = [vp, u64, i32, i32, f32, u64, vp]
        L.qsdp_ref_fit_levels_sequential.argtypes = [vp, u64, i32, i32, f32, u64, vp]
        L.qsdp_ref_quantize_levels_stochastic.argtypes = [vp, u64, i32, i32, vp, u64, u64, vp, vp]
        L.qsdp_ref_quantize_levels_u.argtypes = [vp, u64, i32, i32, vp, vp, vp, vp]
        L.qsdp_ref_fused_step_codes.argtypes = [vp, vp, vp, u64, f32, i32, i32, i32, f32, u64, u64, C.c_uint32, vp]
        L.qsdp_ref_fused_step.argtypes = [vp, vp, u64, f32, i32, i32, i32, f32, u64, u64,
                                          vp, vp, vp]
        L.qsdp_ref_recv_adamw_step.argtypes = [vp, vp, vp, vp, u64, vp, u64, i32, u64, f32, f32, f32, f32, f32, f32,
                                               f32, f32, i32, i32, i32, f32, u64, u32, vp, vp, vp]
        L.qsdp_ref_recv_step.argtypes = [vp, vp, u64, vp, u64, i32, u64, f32, f32, i32, i32, i32, f32, u64, u32,
                                         vp, vp, vp]
        _lib = L
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a.reshape(-1)


def _check(rc, what):
    if rc != 0:
        raise ValueError(f"{what}: oracle returned {rc}")


def set_threads(t):
    return lib().qsdp_ref_set_threads(int(t))


def philox4x32_10(ctr, key):
    ctr = np.asarray(ctr, dtype=np.uint32).copy()
    key = np.asarray(key, dtype=np.uint32).copy()
    out = np.zeros(4, dtype=np.uint32)
    lib().qsdp_ref_philox4x32_10(_p(ctr), _p(key), _p(out))
    return out


def grad_uniform(seed, e):
    return float(lib().qsdp_ref_grad_uniform(int(seed), int(e)))


def weight_shift(seed):
    return float(lib().qsdp_ref_weight_shift(int(seed)))


def grad_shift(seed):
    return float(lib().qsdp_ref_grad_shift(int(seed)))


def codes_bytes(n, bits, bucket):
    return int(lib().qsdp_ref_codes_bytes(int(n), int(bits), int(bucket)))


def meta_bytes(n, bucket):
    return int(lib().qsdp_ref_meta_bytes(int(n), int(bucket)))


def _nb(n, bucket):
    return (n + bucket - 1) // bucket


def quantize_grad_u(g, bits, bucket, u, flags=0):
    """Coin-flip quantizer with explicit uniforms. Returns (codes u8[n], meta f32[nb,2])."""
    g = _f32(g)
    u = _f32(u)
    n = g.size
    codes = np.zeros(n, dtype=np.uint8)
    meta = np.zeros((_nb(n, bucket), 2), dtype=np.float32)
    _check(lib().qsdp_ref_quantize_grad_u_ex(_p(g), n, bits, bucket, _p(u), flags, _p(codes), _p(meta)),
           "quantize_grad_u")
    return codes, meta


def quantize_weight_xi(x, bits, bucket, delta, xi, flags=0):
    """Random-shift quantizer with explicit shift. Returns (codes u8[n], meta, n_saturated)."""
    x = _f32(x)
    n = x.size
    codes = np.zeros(n, dtype=np.uint8)
    meta = np.zeros((_nb(n, bucket), 2), dtype=np.float32)
    sat = np.zeros(1, dtype=np.uint64)
    _check(lib().qsdp_ref_quantize_weight_xi_ex(_p(x), n, bits, bucket, float(delta), float(xi), flags,
                                                _p(codes), _p(meta), _p(sat)),
           "quantize_weight_xi")
    return codes, meta, int(sat[0])


def pack(codes, bits, bucket):
    codes = np.ascontiguousarray(codes, dtype=np.uint8).reshape(-1)
    n = codes.size
    words = np.zeros(codes_bytes(n, bits, bucket) // 4, dtype=np.uint32)
    lib().qsdp_ref_pack(_p(codes), n, bits, bucket, _p(words))
    return words


def unpack(words, n, bits, bucket):
    words = np.ascontiguousarray(words, dtype=np.uint32).reshape(-1)
    assert words.size * 4 == codes_bytes(n, bits, bucket)
    codes = np.zeros(n, dtype=np.uint8)
    lib().qsdp_ref_unpack(_p(words), n, bits, bucket, _p(codes))
    return codes


def f32_to_bf16(v):
    return int(lib().qsdp_ref_f32_to_bf16(float(v)))


def f32_to_f16(v):
    return int(lib().qsdp_ref_f32_to_f16(float(v)))


def quantize_grad(g, bits, bucket, seed, index_offset=0, flags=0):
    """Returns (packed codes u32[...], meta f32[nb,2])."""
    g = _f32(g)
    n = g.size
    codes = np.zeros(codes_bytes(n, bits, bucket) // 4, dtype=np.uint32)
    meta = np.zeros((_nb(n, bucket), 2), dtype=np.float32)
    _check(lib().qsdp_ref_quantize_grad_ex(_p(g), n, bits, bucket, int(seed), int(index_offset), flags,
                                           _p(codes), _p(meta)), "quantize_grad")
    return codes, meta


def quantize_weight(x, bits, bucket, delta, seed, flags=0):
    """Returns (packed codes, meta, n_saturated)."""
    x = _f32(x)
    n = x.size
    codes = np.zeros(codes_bytes(n, bits, bucket) // 4, dtype=np.uint32)
    meta = np.zeros((_nb(n, bucket), 2), dtype=np.float32)
    sat = np.zeros(1, dtype=np.uint64)
    _check(lib().qsdp_ref_quantize_weight_ex(_p(x), n, bits, bucket, float(delta), int(seed), flags,
                                             _p(codes), _p(meta), _p(sat)), "quantize_weight")
    return codes, meta, int(sat[0])


def dequantize(codes, meta, n, bits, bucket, out_dtype=F32):
    """Returns f32[n], or the bf16 / binary16 bit patterns as u16[n]."""
    codes = np.ascontiguousarray(codes, dtype=np.uint32).reshape(-1)
    meta = np.ascontiguousarray(meta, dtype=np.float32).reshape(-1)
    assert codes.size * 4 == codes_bytes(n, bits, bucket)
    assert meta.size == 2 * _nb(n, bucket)
    out = np.zeros(n, dtype=np.float32 if out_dtype == F32 else np.uint16)
    _check(lib().qsdp_ref_dequantize(_p(codes), _p(meta), n, bits, bucket, out_dtype, _p(out)),
           "dequantize")
    return out


def dequantize_add(codes, meta, npeers, n, bits, bucket, alpha):
    """codes u32[npeers, words], meta f32[npeers, nb, 2] -> f32[n] = alpha * sum over peers."""
    codes = np.ascontiguousarray(codes, dtype=np.uint32).reshape(npeers, -1)
    meta = np.ascontiguousarray(meta, dtype=np.float32).reshape(npeers, -1)
    assert codes.shape[1] * 4 == codes_bytes(n, bits, bucket) and meta.shape[1] == 2 * _nb(n, bucket)
    out = np.zeros(n, dtype=np.float32)
    _check(lib().qsdp_ref_dequantize_add(_p(codes), codes.shape[1], _p(meta), meta.shape[1], npeers, n,
                                         bits, bucket, float(alpha), _p(out)), "dequantize_add")
    return out


def fused_step(x, g, lr, wbits, gbits, bucket, delta, seed, index_offset=0, emit_codes=False, flags=0):
    """Returns (x_new f32[n], wcodes or None, wmeta or None, n_saturated). x is not modified."""
    x = _f32(x).copy()
    g = _f32(g)
    n = x.size
    assert g.size == n
    wcodes = wmeta = None
    if emit_codes:
        wcodes = np.zeros(codes_bytes(n, wbits, bucket) // 4, dtype=np.uint32)
        wmeta = np.zeros((_nb(n, bucket), 2), dtype=np.float32)
    sat = np.zeros(1, dtype=np.uint64)
    _check(lib().qsdp_ref_fused_step_ex(_p(x), _p(g), n, float(lr), wbits, gbits, bucket,
                                        float(delta), int(seed), int(index_offset), flags,
                                        _p(wcodes), _p(wmeta), _p(sat)), "fused_step")
    return x, wcodes, wmeta, int(sat[0])


def fused_step_inplace(x, g, lr, wbits, gbits, bucket, delta, seed, index_offset=0, wcodes=None, wmeta=None,
                       flags=0):
    """The fused step on caller-owned arrays, for vectors too large to copy: x (float32, C-contiguous) is
    updated in place; wcodes (uint32) and wmeta (float32), when given, receive the packed codes and the
    meta of the new x. Returns n_saturated."""
    for a, t in ((x, np.float32), (g, np.float32), (wcodes, np.uint32), (wmeta, np.float32)):
        assert a is None or (a.dtype == t and a.flags.c_contiguous)
    n = x.size
    assert g.size == n and x.flags.writeable
    if wcodes is not None:
        assert wcodes.size * 4 == codes_bytes(n, wbits, bucket) and wmeta.size == 2 * _nb(n, bucket)
    sat = np.zeros(1, dtype=np.uint64)
    _check(lib().qsdp_ref_fused_step_ex(_p(x), _p(g), n, float(lr), wbits, gbits, bucket, float(delta), int(seed),
                                        int(index_offset), flags, _p(wcodes), _p(wmeta), _p(sat)),
           "fused_step_inplace")
    return int(sat[0])


def fused_step_codes(wcodes, wmeta, g, lr, wbits, gbits, bucket, delta, seed, index_offset=0, flags=0):
    """Returns (new wcodes, new wmeta, n_saturated); inputs are not modified."""
    g = _f32(g)
    n = g.size
    wcodes = np.ascontiguousarray(wcodes, dtype=np.uint32).reshape(-1).copy()
    wmeta = np.ascontiguousarray(wmeta, dtype=np.float32).reshape(-1, 2).copy()
    assert wcodes.size * 4 == codes_bytes(n, wbits, bucket) and wmeta.shape[0] == _nb(n, bucket)
    sat = np.zeros(1, dtype=np.uint64)
    _check(lib().qsdp_ref_fused_step_codes(_p(wcodes), _p(wmeta), _p(g), n, float(lr), wbits, gbits, bucket,
                                           float(delta), int(seed), int(index_offset), flags, _p(sat)),
           "fused_step_codes")
    return wcodes, wmeta, int(sat[0])


def recv_step(x, gcodes, gmeta, npeers, alpha, lr, wbits, gbits, bucket, delta, seed, flags=0, emit_codes=False):
    """gcodes u32[npeers, words], gmeta f32[npeers, nb*2]. Returns (x_new, wcodes or None, wmeta or
    None, n_saturated); x is not modified."""
    x = _f32(x).copy()
    n = x.size
    gcodes = np.ascontiguousarray(gcodes, dtype=np.uint32).reshape(npeers, -1)
    gmeta = np.ascontiguousarray(gmeta, dtype=np.float32).reshape(npeers, -1)
    assert gcodes.shape[1] * 4 == codes_bytes(n, gbits, bucket) and gmeta.shape[1] == 2 * _nb(n, bucket)
    wcodes = wmeta = None
    if emit_codes:
        wcodes = np.zeros(codes_bytes(n, wbits, bucket) // 4, dtype=np.uint32)
        wmeta = np.zeros((_nb(n, bucket), 2), dtype=np.float32)
    sat = np.zeros(1, dtype=np.uint64)
    _check(lib().qsdp_ref_recv_step(_p(x), _p(gcodes), gcodes.shape[1], _p(gmeta), gmeta.shape[1], npeers, n,
                                    float(alpha), float(lr), wbits, gbits, bucket, float(delta), int(seed), flags,
                                    _p(wcodes), _p(wmeta), _p(sat)), "recv_step")
    return x, wcodes, wmeta, int(sat[0])


def recv_adamw_step(x, m, v, gcodes, gmeta, npeers, alpha, lr, beta1, beta2, eps, weight_decay, bias1, bias2, wbits,
                    gbits, bucket, delta, seed, flags=0, emit_codes=False):
    """Returns (x_new, m_new, v_new, wcodes or None, wmeta or None, n_saturated); inputs are not modified."""
    x = _f32(x).copy(); m = _f32(m).copy(); v = _f32(v).copy()
    n = x.size
    gcodes = np.ascontiguousarray(gcodes, dtype=np.uint32).reshape(npeers, -1)
    gmeta = np.ascontiguousarray(gmeta, dtype=np.float32).reshape(npeers, -1)
    assert gcodes.shape[1] * 4 == codes_bytes(n, gbits, bucket) and gmeta.shape[1] == 2 * _nb(n, bucket)
    wcodes = wmeta = None
    if emit_codes:
        wcodes = np.zeros(codes_bytes(n, wbits, bucket) // 4, dtype=np.uint32)
        wmeta = np.zeros((_nb(n, bucket), 2), dtype=np.float32)
    sat = np.zeros(1, dtype=np.uint64)
    _check(lib().qsdp_ref_recv_adamw_step(_p(x), _p(m), _p(v), _p(gcodes), gcodes.shape[1], _p(gmeta),
                                          gmeta.shape[1], npeers, n, float(alpha), float(lr), float(beta1),
                                          float(beta2), float(eps), float(weight_decay), float(bias1), float(bias2),
                                          wbits, gbits, bucket, float(delta), int(seed), flags, _p(wcodes), _p(wmeta),
                                          _p(sat)), "recv_adamw_step")
    return x, m, v, wcodes, wmeta, int(sat[0])


def levels_uniform(bits):
    lv = np.zeros(1 << bits, dtype=np.float32)
    _check(lib().qsdp_ref_levels_uniform(bits, _p(lv)), "levels_uniform")
    return lv


def quantize_levels(v, bits, bucket, levels):
    """Nearest-level encoding. Returns (packed codes, meta f32[nb,2] = {lo, hi-lo})."""
    v = _f32(v)
    levels = _f32(levels)
    n = v.size
    codes = np.zeros(codes_bytes(n, bits, bucket) // 4, dtype=np.uint32)
    meta = np.zeros((_nb(n, bucket), 2), dtype=np.float32)
    _check(lib().qsdp_ref_quantize_levels(_p(v), n, bits, bucket, _p(levels), _p(codes), _p(meta)),
           "quantize_levels")
    return codes, meta


def quantize_levels_stochastic(v, bits, bucket, levels, seed, index_offset=0):
    """Unbiased rounding onto the enclosing levels. Returns (packed codes, meta f32[nb,2] = {lo, hi-lo})."""
    v = _f32(v); levels = _f32(levels)
    n = v.size
    codes = np.zeros(codes_bytes(n, bits, bucket) // 4, dtype=np.uint32)
    meta = np.zeros((_nb(n, bucket), 2), dtype=np.float32)
    _check(lib().qsdp_ref_quantize_levels_stochastic(_p(v), n, bits, bucket, _p(levels), int(seed),
                                                     int(index_offset), _p(codes), _p(meta)),
           "quantize_levels_stochastic")
    return codes, meta


def quantize_levels_u(v, bits, bucket, levels, u):
    """The same with explicit uniforms. Returns (codes u8[n], meta)."""
    v = _f32(v); levels = _f32(levels); u = _f32(u)
    n = v.size
    codes = np.zeros(n, dtype=np.uint8)
    meta = np.zeros((_nb(n, bucket), 2), dtype=np.float32)
    _check(lib().qsdp_ref_quantize_levels_u(_p(v), n, bits, bucket, _p(levels), _p(u), _p(codes), _p(meta)),
           "quantize_levels_u")
    return codes, meta


def dequantize_levels(codes, meta, n, bits, bucket, levels, out_dtype=F32):
    codes = np.ascontiguousarray(codes, dtype=np.uint32).reshape(-1)
    meta = np.ascontiguousarray(meta, dtype=np.float32).reshape(-1)
    levels = _f32(levels)
    out = np.zeros(n, dtype=np.float32 if out_dtype == F32 else np.uint16)
    _check(lib().qsdp_ref_dequantize_levels(_p(codes), _p(meta), n, bits, bucket, _p(levels), out_dtype,
                                            _p(out)), "dequantize_levels")
    return out


def fit_levels(v, bits, bucket, lr, levels, max_batches=0):
    """Algorithm 1 (batched). Returns the fitted levels; `levels` is the start and is not modified."""
    v = _f32(v)
    lv = _f32(levels).copy()
    _check(lib().qsdp_ref_fit_levels(_p(v), v.size, bits, bucket, float(lr), int(max_batches), _p(lv)),
           "fit_levels")
    return lv


def fit_levels_sequential(v, bits, bucket, lr, levels, max_batches=0):
    """Algorithm 1 as printed (one value at a time against the current table). Returns the fitted levels;
    `levels` is the start and is not modified."""
    v = _f32(v)
    lv = _f32(levels).copy()
    _check(lib().qsdp_ref_fit_levels_sequential(_p(v), v.size, bits, bucket, float(lr), int(max_batches), _p(lv)),
           "fit_levels_sequential")
    return lv


def fused_adamw_step(x, g, m, v, lr, beta1, beta2, eps, weight_decay, bias1, bias2, wbits, gbits, bucket,
                     delta, seed, index_offset=0, flags=0, emit_codes=False):
    """Returns (x_new, m_new, v_new, wcodes, wmeta, n_saturated); inputs are not modified."""
    x = _f32(x).copy(); m = _f32(m).copy(); v = _f32(v).copy()
    g = _f32(g)
    n = x.size
    wcodes = wmeta = None
    if emit_codes:
        wcodes = np.zeros(codes_bytes(n, wbits, bucket) // 4, dtype=np.uint32)
        wmeta = np.zeros((_nb(n, bucket), 2), dtype=np.float32)
    sat = np.zeros(1, dtype=np.uint64)
    _check(lib().qsdp_ref_fused_adamw_step(_p(x), _p(g), _p(m), _p(v), n, float(lr), float(beta1), float(beta2),
                                           float(eps), float(weight_decay), float(bias1), float(bias2), wbits,
                                           gbits, bucket, float(delta), int(seed), int(index_offset), flags,
                                           _p(wcodes), _p(wmeta), _p(sat)), "fused_adamw_step")
    return x, m, v, wcodes, wmeta, int(sat[0])
