// Device-side building blocks of the QSDP codec for gfx950 (wave64).
//
// Arithmetic contract (binary32, round to nearest even, no contraction; this file is
// compiled with -ffp-contract=off, fused multiply-adds are written as fmaf):
//   bucket grid   lo = min + 0.0f, hi = max + 0.0f, range = hi - lo,
//                 scale = range / L, inv = L / range (0, 0 for a degenerate bucket)
//   Q^g           t = clamp((g - lo) * inv, 0, L); code = floor(t) + [u < t - floor(t)]
//   Q^w (min-max) k = clamp(rint((x - lo) * inv - xi), 0, L); base = fma(xi, scale, lo)
//   Q^w (lattice) k = rint(x / delta - xi); code = min(k - k0, L); base = (k0 + xi) * delta
//   decode        fma(code, scale, base)
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace qsdp {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef uint32_t u2 __attribute__((ext_vector_type(2)));
typedef uint32_t u4 __attribute__((ext_vector_type(4)));

// ---------------------------------------------------------------------------------------
// Philox4x32-10 (Salmon et al., SC'11). The key is wave-uniform, so its schedule lives in
// scalar registers; each round costs two 32x32->64 multiplies and three xors per lane.
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                              uint32_t k0, uint32_t k1, uint32_t (&out)[4]) {
#pragma unroll
    for (int round = 0; round < 10; ++round) {
        const uint64_t p0 = (uint64_t)0xD2511F53u * (uint64_t)c0;
        const uint64_t p1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        const uint32_t n1 = (uint32_t)p1;
        const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        const uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// Rounding uniforms of a row pair, as the 16-bit integers h (u = h * 2^-16) converted to float
// (exact). Lane l holds elements (r*G + l)*4 .. +3 of rows r = 2c and 2c+1. A Philox block (8
// elements) spans the lane pair (l even, l+1) of one row: the even lane computes the block of
// row 2c, the odd lane that of row 2c+1, and the pair swaps the halves the other needs.
// h[0..3] serve row 2c, h[4..7] row 2c+1. bucket_block = index of the bucket's first block.
template <int G>
__device__ __forceinline__ void grad_uniforms_rows(uint64_t bucket_block, int c, int l, uint32_t k0,
                                                   uint32_t k1, float (&h)[8]) {
    const int odd = l & 1;
    const uint64_t block = bucket_block + (uint64_t)(((2 * c + odd) * G + (l - odd)) >> 1);
    uint32_t w[4];
    philox4x32_10((uint32_t)block, (uint32_t)(block >> 32), 0u, 0u, k0, k1, w);
    const uint32_t send0 = odd ? w[0] : w[2];
    const uint32_t send1 = odd ? w[1] : w[3];
    const uint32_t recv0 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)send0, 0xB1, 0xF, 0xF, false);
    const uint32_t recv1 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)send1, 0xB1, 0xF, 0xF, false);
    const uint32_t a0 = odd ? recv0 : w[0], a1 = odd ? recv1 : w[1];  // row 2c
    const uint32_t b0 = odd ? w[2] : recv0, b1 = odd ? w[3] : recv1;  // row 2c+1
    h[0] = (float)(a0 & 0xFFFFu); h[1] = (float)(a0 >> 16);
    h[2] = (float)(a1 & 0xFFFFu); h[3] = (float)(a1 >> 16);
    h[4] = (float)(b0 & 0xFFFFu); h[5] = (float)(b0 >> 16);
    h[6] = (float)(b1 & 0xFFFFu); h[7] = (float)(b1 >> 16);
}

// A shift xi in [-1/2, 1/2): counter 0 of stream 1 (weights) or 2 (shared-shift gradients).
__device__ __forceinline__ float stream_shift(uint32_t stream, uint32_t k0, uint32_t k1) {
    uint32_t w[4];
    philox4x32_10(0u, 0u, stream, 0u, k0, k1, w);
    return (float)(w[0] >> 8) * 0x1p-24f - 0.5f;
}

// ---------------------------------------------------------------------------------------
// Cross-lane min/max over aligned groups of G lanes (G a power of two, 2..64), all lanes of
// the group end with the result. DPP inside a 16-lane row, gfx950 row/half swaps across rows.
// ---------------------------------------------------------------------------------------
template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
    // every lane has a valid source for the controls used here, so the previous value of the
    // destination is irrelevant and the move can fold into the min/max that consumes it
    return __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(v), CTRL, 0xF, 0xF, true));
}

__device__ __forceinline__ void swap16(float v, float& a, float& b) {
    auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    a = __uint_as_float(r[0]);
    b = __uint_as_float(r[1]);
}

__device__ __forceinline__ void swap32(float v, float& a, float& b) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    a = __uint_as_float(r[0]);
    b = __uint_as_float(r[1]);
}

template <int G>
__device__ __forceinline__ float group_min(float v) {
    if (G >= 2) v = fminf(v, dpp_move<0xB1>(v));   // quad_perm [1,0,3,2]
    if (G >= 4) v = fminf(v, dpp_move<0x4E>(v));   // quad_perm [2,3,0,1]
    if (G >= 8) v = fminf(v, dpp_move<0x141>(v));  // row_half_mirror
    if (G >= 16) v = fminf(v, dpp_move<0x140>(v)); // row_mirror
    if (G >= 32) { float a, b; swap16(v, a, b); v = fminf(a, b); }
    if (G >= 64) { float a, b; swap32(v, a, b); v = fminf(a, b); }
    return v;
}

template <int G>
__device__ __forceinline__ float group_max(float v) {
    if (G >= 2) v = fmaxf(v, dpp_move<0xB1>(v));
    if (G >= 4) v = fmaxf(v, dpp_move<0x4E>(v));
    if (G >= 8) v = fmaxf(v, dpp_move<0x141>(v));
    if (G >= 16) v = fmaxf(v, dpp_move<0x140>(v));
    if (G >= 32) { float a, b; swap16(v, a, b); v = fmaxf(a, b); }
    if (G >= 64) { float a, b; swap32(v, a, b); v = fmaxf(a, b); }
    return v;
}

// ---------------------------------------------------------------------------------------
// Per-bucket grids
// ---------------------------------------------------------------------------------------
struct MinMaxGrid {
    float lo, scale, inv;
};

__device__ __forceinline__ MinMaxGrid make_minmax_grid(float lo, float hi, float Lf, bool symmetric) {
    lo = lo + 0.0f;  // -0 -> +0: one bit pattern for the stored base
    hi = hi + 0.0f;
    if (symmetric) {  // grid over [-a, a], a = max |v|
        const float a = fmaxf(fabsf(lo), fabsf(hi));
        lo = -a + 0.0f;
        hi = a;
    }
    const float range = hi - lo;
    const float inv = Lf / range;
    const float scale = range / Lf;
    const bool ok = (range > 0.0f) && (range < __builtin_inff()) && (inv < __builtin_inff());
    MinMaxGrid g;
    g.lo = lo;
    g.scale = ok ? scale : 0.0f;
    g.inv = ok ? inv : 0.0f;
    return g;
}

// x / delta, as a multiplication when 1/delta is exact (delta a power of two): the product
// and the quotient are then roundings of the same real number.
struct Divider {
    float delta, inv_delta;
    bool pow2;
};

__device__ __forceinline__ float div_delta(float v, const Divider& d) {
    return d.pow2 ? v * d.inv_delta : v / d.delta;
}

// Coin-flip code of one gradient element: floor(t) + [u < frac(t)], t clamped to [0, L]
// (t >= 0 always; the upper clamp catches (hi - lo) * inv rounding above L). v_med3 is the
// clamp and v_fract is t - floor(t), exactly, for finite t >= 0. h = u * 2^16.
__device__ __forceinline__ float grad_position(float g, const MinMaxGrid& grid, float Lf) {
    const float t = (g - grid.lo) * grid.inv;
    return __builtin_amdgcn_fmed3f(t, 0.0f, Lf);
}

// ... as a float (for decoding in registers)
__device__ __forceinline__ float grad_code(float g, const MinMaxGrid& grid, float Lf, float h) {
    const float t = grad_position(g, grid, Lf);
    const float frac = __builtin_amdgcn_fractf(t);
    const float u = h * 0x1p-16f;
    return floorf(t) + ((u < frac) ? 1.0f : 0.0f);
}

// ... as an integer (for packing): truncation is floor for t >= 0
__device__ __forceinline__ uint32_t grad_code_int(float g, const MinMaxGrid& grid, float Lf, float h) {
    const float t = grad_position(g, grid, Lf);
    const float frac = __builtin_amdgcn_fractf(t);
    const float u = h * 0x1p-16f;
    return (uint32_t)t + ((u < frac) ? 1u : 0u);
}

__device__ __forceinline__ float weight_code_minmax(float x, const MinMaxGrid& grid, float Lf,
                                                    float xi) {
    const float t = (x - grid.lo) * grid.inv;
    const float k = rintf(t - xi);
    return __builtin_amdgcn_fmed3f(k, 0.0f, Lf);
}

__device__ __forceinline__ float weight_code_lattice(float x, const Divider& d, float xi, float k0,
                                                     float Lf, uint32_t& saturated) {
    const float k = rintf(div_delta(x, d) - xi);
    float c = k - k0;
    if (c > Lf) {
        c = Lf;
        saturated += 1u;
    }
    return c;
}

// Nearest of the K = 2^BITS ascending levels `lv` (in LDS) to z; ties and equal levels resolve
// to the lowest index. Branch-free lower bound over the power-of-two table, then the closer of
// the two neighbours.
template <int BITS>
__device__ __forceinline__ int nearest_level(float z, const float* lv) {
    constexpr int K = 1 << BITS;
    int j = 0;  // ends as the number of levels < z among the first K-1, i.e. a lower bound
#pragma unroll
    for (int step = K / 2; step >= 1; step >>= 1)
        if (lv[j + step - 1] < z) j += step;
    // levels[j-1] < z <= levels[j] (with j in [0, K-1]; if all of the first K-1 are < z, j = K-1)
    const int lo_idx = j > 0 ? j - 1 : 0;
    const float d_lo = fabsf(z - lv[lo_idx]);
    const float d_hi = fabsf(z - lv[j]);
    int c = d_hi < d_lo ? j : lo_idx;
    while (c > 0 && lv[c - 1] == lv[c]) --c;  // first among equal levels (rare)
    return c;
}

// The same search without control flow per element: `first[k]` = the lowest index whose level
// equals lv[k] (fill_first_equal), looked up instead of walked to. The encoder's 16 independent
// searches of a lane then interleave freely; with the loop above each of them is a basic block.
template <int BITS>
__device__ __forceinline__ int nearest_level(float z, const float* lv, const int* first) {
    constexpr int K = 1 << BITS;
    int j = 0;
#pragma unroll
    for (int step = K / 2; step >= 1; step >>= 1)
        if (lv[j + step - 1] < z) j += step;
    const int lo_idx = j > 0 ? j - 1 : 0;
    const float d_lo = fabsf(z - lv[lo_idx]);
    const float d_hi = fabsf(z - lv[j]);
    return first[d_hi < d_lo ? j : lo_idx];
}

// first[k] for k = k0, k0 + stride, ... < K (lv complete and visible to the caller's threads)
__device__ __forceinline__ void fill_first_equal(const float* lv, int* first, int K, int k0, int stride) {
    for (int k = k0; k < K; k += stride) {
        int j = k;
        while (j > 0 && lv[j - 1] == lv[j]) --j;
        first[k] = j;
    }
}

// Unbiased rounding of z onto the two of the K = 2^BITS ascending levels `lv` (in LDS) that
// enclose it: with i the largest index such that lv[i] <= z, code = i + [h * 2^-16 < p],
// p = (z - lv[i]) / (lv[i+1] - lv[i]); z below the first level gives 0, at or above the last K-1.
// h is the 16-bit rounding uniform as a float (exact), so h < p * 2^16 is the same comparison.
template <int BITS>
__device__ __forceinline__ int stochastic_level(float z, float h, const float* lv) {
    constexpr int K = 1 << BITS;
    int cnt = 0;  // number of levels <= z among the first K-1 (branch-free search), then the last one
#pragma unroll
    for (int step = K / 2; step >= 1; step >>= 1)
        if (lv[cnt + step - 1] <= z) cnt += step;
    if (cnt == K - 1 && lv[K - 1] <= z) cnt = K;
    if (cnt == 0) return 0;
    if (cnt == K) return K - 1;
    const int i = cnt - 1;
    const float p = (z - lv[i]) / (lv[i + 1] - lv[i]);
    return i + (h < p * 65536.0f ? 1 : 0);
}

// ---------------------------------------------------------------------------------------
// Packing: 4 consecutive codes of a lane, 8 consecutive codes (a chunk) = BITS bytes
// ---------------------------------------------------------------------------------------
template <int BITS>
__device__ __forceinline__ uint32_t pack4(const uint32_t (&c)[4]) {
    uint32_t acc = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) acc |= c[i] << (i * BITS);
    return acc;
}

template <int BITS>
__device__ __forceinline__ uint32_t pack4(const float (&c)[4]) {
    uint32_t acc = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) acc |= (uint32_t)c[i] << (i * BITS);
    return acc;
}

// Store the BITS bytes of a packed chunk at byte address p in LDS (p is a multiple of BITS
// bytes from a 16-byte aligned base, so the widest naturally aligned pieces are used).
template <int BITS>
__device__ __forceinline__ void store_chunk(uint8_t* p, uint64_t v) {
    if (BITS == 8) {
        u2 w = {(uint32_t)v, (uint32_t)(v >> 32)};
        *reinterpret_cast<u2*>(p) = w;
    } else if (BITS == 4) {
        *reinterpret_cast<uint32_t*>(p) = (uint32_t)v;
    } else if (BITS == 2) {
        *reinterpret_cast<uint16_t*>(p) = (uint16_t)v;
    } else if (BITS == 6) {
        uint16_t* q = reinterpret_cast<uint16_t*>(p);
        q[0] = (uint16_t)v; q[1] = (uint16_t)(v >> 16); q[2] = (uint16_t)(v >> 32);
    } else {
#pragma unroll
        for (int i = 0; i < BITS; ++i) p[i] = (uint8_t)(v >> (8 * i));
    }
}

template <int BITS>
__device__ __forceinline__ uint64_t load_chunk(const uint8_t* p) {
    if (BITS == 8) {
        u2 w = *reinterpret_cast<const u2*>(p);
        return (uint64_t)w[0] | ((uint64_t)w[1] << 32);
    } else if (BITS == 4) {
        return *reinterpret_cast<const uint32_t*>(p);
    } else if (BITS == 2) {
        return *reinterpret_cast<const uint16_t*>(p);
    } else if (BITS == 6) {
        const uint16_t* q = reinterpret_cast<const uint16_t*>(p);
        return (uint64_t)q[0] | ((uint64_t)q[1] << 16) | ((uint64_t)q[2] << 32);
    } else {
        uint64_t v = 0;
#pragma unroll
        for (int i = 0; i < BITS; ++i) v |= (uint64_t)p[i] << (8 * i);
        return v;
    }
}

// binary32 -> bfloat16 bits, round to nearest even (finite inputs)
__device__ __forceinline__ uint32_t bf16_bits(float v) {
    uint32_t b = __float_as_uint(v);
    b += 0x7FFFu + ((b >> 16) & 1u);
    return b >> 16;
}

// binary32 -> IEEE binary16 bits: the hardware conversion (round to nearest even, subnormal
// results kept, overflow to infinity)
__device__ __forceinline__ uint32_t f16_bits(float v) {
    return (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)v);
}

// the 2-byte output formats of the decoders
__device__ __forceinline__ uint32_t half_bits(float v, bool f16) { return f16 ? f16_bits(v) : bf16_bits(v); }

}  // namespace qsdp
