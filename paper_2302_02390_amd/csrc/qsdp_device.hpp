// Device-side building blocks of the QSDP codec for gfx950 (wave64).
//
// Arithmetic contract (binary32, round to nearest even, no contraction; this file is
// compiled with -ffp-contract=off, fused multiply-adds are written as fmaf):
//   bucket grid   lo = min + 0.0f, hi = max + 0.0f, range = hi - lo,
//                 scale = range / L, inv = L / range (0, 0 for a degenerate bucket: range 0, not
//                 finite, or inv * 2^16 not finite)
//   Q^g           ti = min(trunc(fma(g - lo, inv * 2^16, 1/2)), L * 2^16); code = (ti + h) >> 16, h the
//                 element's 16-bit uniform
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

// Rounding uniforms of a row pair: the 16-bit integers h of the lane's eight elements, still packed
// two to a word (low half first). Lane l holds elements (r*G + l)*4 .. +3 of rows r = 2c and 2c+1.
// A Philox block (8 elements) spans the lane pair (l even, l+1) of one row: the even lane computes
// the block of row 2c, the odd lane that of row 2c+1, and the pair swaps the halves the other needs.
// w[0..1] serve row 2c, w[2..3] row 2c+1. bucket_block = index of the bucket's first block.
template <int G>
__device__ __forceinline__ void grad_uniforms_rows(uint64_t bucket_block, int c, int l, uint32_t k0,
                                                   uint32_t k1, uint32_t (&h)[4]) {
    const int odd = l & 1;
    const uint64_t block = bucket_block + (uint64_t)(((2 * c + odd) * G + (l - odd)) >> 1);
    uint32_t w[4];
    philox4x32_10((uint32_t)block, (uint32_t)(block >> 32), 0u, 0u, k0, k1, w);
    const uint32_t send0 = odd ? w[0] : w[2];
    const uint32_t send1 = odd ? w[1] : w[3];
    // every lane has a partner, so the destination's previous value never shows
    const uint32_t recv0 = (uint32_t)__builtin_amdgcn_mov_dpp((int)send0, 0xB1, 0xF, 0xF, true);
    const uint32_t recv1 = (uint32_t)__builtin_amdgcn_mov_dpp((int)send1, 0xB1, 0xF, 0xF, true);
    h[0] = odd ? recv0 : w[0]; h[1] = odd ? recv1 : w[1];  // row 2c
    h[2] = odd ? w[2] : recv0; h[3] = odd ? w[3] : recv1;  // row 2c+1
}

// The 16-bit uniform of element i (0..7) of a row pair out of the packed words above.
__device__ __forceinline__ uint32_t uniform16(const uint32_t (&h)[4], int i) {
    return (i & 1) ? (h[i >> 1] >> 16) : (h[i >> 1] & 0xFFFFu);
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
    const bool ok = (range > 0.0f) && (range < __builtin_inff()) && (inv * 65536.0f < __builtin_inff());
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

// Coin-flip code of one gradient element, decided in integers: the position in the bucket's grid
// in units of 2^-16 of a cell, ti = min(trunc(fma(g - lo, inv * 2^16, 1/2)), L * 2^16) (the
// conversion saturates, so a non-finite input cannot fault), plus the 16-bit uniform h; the code is
// the sum's bits 16 and up: floor(t) + 1 for exactly (ti mod 2^16) of the 2^16 values of h.
__device__ __forceinline__ uint32_t grad_sum16(float g, const MinMaxGrid& grid, uint32_t top16, uint32_t h) {
    const float t16 = fmaf(g - grid.lo, grid.inv * 65536.0f, 0.5f);
    const uint32_t ti = (uint32_t)t16;
    return (ti < top16 ? ti : top16) + h;
}

// ... as a float (for decoding in registers): byte 2 of the sum (the code is at most 255)
__device__ __forceinline__ float grad_code(float g, const MinMaxGrid& grid, uint32_t top16, uint32_t h) {
    return (float)((grad_sum16(g, grid, top16, h) >> 16) & 0xFFu);
}

// ... as an integer (for packing)
__device__ __forceinline__ uint32_t grad_code_int(float g, const MinMaxGrid& grid, uint32_t top16, uint32_t h) {
    return (grad_sum16(g, grid, top16, h) >> 16) & 0xFFu;
}

__device__ __forceinline__ float weight_code_minmax(float x, const MinMaxGrid& grid, float Lf,
                                                    float xi) {
    const float t = (x - grid.lo) * grid.inv;
    const float k = rintf(t - xi);
    return __builtin_amdgcn_fmed3f(k, 0.0f, Lf);
}

// The position of x in the grid before rounding: weight_code_minmax is clamp(rint(this), 0, L).
__device__ __forceinline__ float weight_position_minmax(float x, const MinMaxGrid& grid, float xi) {
    const float t = (x - grid.lo) * grid.inv;
    return t - xi;
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

// ---------------------------------------------------------------------------------------
// Learned levels: K = 2^BITS ascending levels in [0, 1]. The encoders work in "cell units": every
// level and every normalised value is scaled by kLevelCells (a power of two, so all comparisons,
// differences and products below are the unscaled ones times an exact power of two and give the
// same decisions bit for bit). An encoder first counts the levels below (or at) the value, then
// fetches what it needs about that landing place with one LDS read from a table built once per
// workgroup (or per wave, where every tensor has its own levels).
//   * Counting by cell: the unit interval is cut into kLevelCells cells; a table holds for each cell
//     how many levels lie below its start and the next level. If no cell holds two levels, the count
//     for a value is the cell's count plus one comparison with that next level: one LDS read.
//   * Counting by search (a table with two levels in one cell): branch-free binary search whose
//     first two pivots are wave-uniform and held in scalar registers.
// ---------------------------------------------------------------------------------------
constexpr int kLevelCells = 256;
constexpr float kLevelCellsF = 256.0f;

struct LevelCell {
    float next;  // the first level not below (LE: not at or below) the cell's start, +inf if none
    int count;   // levels below (LE: at or below) the cell's start
};

// Entries c = c0, c0 + stride, ... <= kLevelCells of the cell table over the first `kc` scaled levels
// lv (cell c is [c, c+1) in cell units; the last entry serves a value of exactly 1). Returns whether
// one of these cells holds two levels, in which case the table must not be used.
template <bool LE>
__device__ __forceinline__ bool fill_level_cells(const float* lv, LevelCell* cells, int kc, int c0, int stride) {
    bool crowded = false;
    for (int c = c0; c <= kLevelCells; c += stride) {
        const float start = (float)c;
        int lo = 0, hi = kc;  // lv[k] below start for k < lo, not below for k >= hi
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (LE ? lv[mid] <= start : lv[mid] < start) lo = mid + 1; else hi = mid;
        }
        LevelCell e = {lo < kc ? lv[lo] : __builtin_inff(), lo};
        cells[c] = e;
        crowded = crowded || (lo + 1 < kc && lv[lo + 1] < start + 1.0f);
    }
    return crowded;
}

// The cell table's count for a value zc (in cell units; the conversion saturates, the index is
// clamped, so a non-finite value cannot read outside the table).
template <bool LE>
__device__ __forceinline__ int count_levels_by_cell(float zc, const LevelCell* cells) {
    const uint32_t c = (uint32_t)zc;
    const LevelCell e = cells[c < (uint32_t)kLevelCells ? c : (uint32_t)kLevelCells];
    return e.count + ((LE ? e.next <= zc : e.next < zc) ? 1 : 0);
}

struct LevelPivots {
    float mid, lower, upper, last;  // lv[K/2-1], lv[K/4-1], lv[3K/4-1], lv[K-1]
};

// All lanes read the same addresses, so the values are wave-uniform and can live in SGPRs.
template <int BITS>
__device__ __forceinline__ LevelPivots load_level_pivots(const float* lv) {
    constexpr int K = 1 << BITS;
    auto uniform = [](float v) { return __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(v))); };
    LevelPivots pv;
    pv.mid = uniform(lv[K / 2 - 1]);
    pv.lower = uniform(lv[BITS >= 2 ? K / 4 - 1 : 0]);
    pv.upper = uniform(lv[BITS >= 2 ? 3 * K / 4 - 1 : 0]);
    pv.last = uniform(lv[K - 1]);
    return pv;
}

// How many of the first K-1 levels are < z (LE: <= z): a lower (upper) bound over the power-of-two table.
template <int BITS, bool LE>
__device__ __forceinline__ int count_levels_by_search(float z, const float* lv, const LevelPivots& pv) {
    constexpr int K = 1 << BITS;
    auto below = [](float q, float zz) { return LE ? q <= zz : q < zz; };
    int j = below(pv.mid, z) ? K / 2 : 0;
    if (BITS >= 2) j += below(j ? pv.upper : pv.lower, z) ? K / 4 : 0;
#pragma unroll
    for (int step = K / 8; step >= 1; step >>= 1)
        if (below(lv[j + step - 1], z)) j += step;
    return j;
}

// What the nearest-level encoder needs at landing place j (lv[j-1] < z <= lv[j]): the two candidate
// levels and the code of the lower one, which is the lowest index whose level equals it (ties and
// equal levels resolve to the lowest index).
struct LevelNear {
    float lo, hi;
    int first_lo, unused;
};

// Entries k = k0, k0 + stride, ... < K of that table (lv complete and visible to the caller's threads).
__device__ __forceinline__ void fill_level_near(const float* lv, LevelNear* near, int K, int k0, int stride) {
    for (int k = k0; k < K; k += stride) {
        int f = k > 0 ? k - 1 : 0;
        const float lo = lv[f];
        while (f > 0 && lv[f - 1] == lo) --f;
        LevelNear e = {lo, lv[k], f, 0};
        near[k] = e;
    }
}

// Nearest of the levels to z (both in cell units); ties and equal levels resolve to the lowest index.
// by_cell (wave-uniform): the cell table may be used.
template <int BITS>
__device__ __forceinline__ uint32_t nearest_level(float z, const float* lv, const LevelCell* cells, const LevelNear* near,
                                                  const LevelPivots& pv, bool by_cell) {
    // the number of levels < z among the first K-1: j in [0, K-1]
    const int j = by_cell ? count_levels_by_cell<false>(z, cells) : count_levels_by_search<BITS, false>(z, lv, pv);
    const LevelNear e = near[j];
    return (uint32_t)(fabsf(z - e.hi) < fabsf(z - e.lo) ? j : e.first_lo);
}

// The same by the plain definition over an (unscaled) table in LDS (level fit: one value per thread at a time).
template <int BITS>
__device__ __forceinline__ int nearest_level(float z, const float* lv) {
    constexpr int K = 1 << BITS;
    int j = 0;  // ends as the number of levels < z among the first K-1, i.e. a lower bound
#pragma unroll
    for (int step = K / 2; step >= 1; step >>= 1)
        if (lv[j + step - 1] < z) j += step;
    const int lo_idx = j > 0 ? j - 1 : 0;
    const float d_lo = fabsf(z - lv[lo_idx]);
    const float d_hi = fabsf(z - lv[j]);
    int c = d_hi < d_lo ? j : lo_idx;
    while (c > 0 && lv[c - 1] == lv[c]) --c;  // first among equal levels (rare)
    return c;
}

// What the coin-flip encoder needs at level i: the level (cell units) and the reciprocal of the gap
// to the next one (per cell unit; 0 for the last level: nothing to round up to).
struct LevelCoin {
    float q, rgap;
};

// lv: the scaled levels. The reciprocal of a scaled gap is the unscaled reciprocal divided by
// kLevelCells, exactly, so (z - q) * rgap in cell units is the unscaled product bit for bit.
__device__ __forceinline__ void fill_level_coin(const float* lv, LevelCoin* coin, int K, int k0, int stride) {
    for (int k = k0; k < K; k += stride) {
        LevelCoin e = {lv[k], k + 1 < K ? 1.0f / (lv[k + 1] - lv[k]) : 0.0f};
        coin[k] = e;
    }
}

// Unbiased rounding of z onto the two levels that enclose it: with i the largest index such that
// lv[i] <= z and p = (z - lv[i]) * (1 / (lv[i+1] - lv[i])), code = i + [2^16 - (h + 1/2) < p * 2^16]: up
// for the round(p * 2^16) largest of the 2^16 values of the uniform h (given as a float, exact). z
// below the first level gives 0 (p < 0 there), at or above the last K-1 (its reciprocal gap is 0).
// z and the tables are in cell units; p comes out unscaled.
template <int BITS>
__device__ __forceinline__ uint32_t stochastic_level(float z, float h, const float* lv, const LevelCell* cells,
                                                     const LevelCoin* coin, const LevelPivots& pv, bool by_cell) {
    constexpr int K = 1 << BITS;
    int cnt;  // levels <= z
    if (by_cell) {
        cnt = count_levels_by_cell<true>(z, cells);
    } else {
        cnt = count_levels_by_search<BITS, true>(z, lv, pv);  // among the first K-1 ...
        cnt += (cnt == K - 1 && pv.last <= z) ? 1 : 0;         // ... and the last one
    }
    const int i = cnt > 0 ? cnt - 1 : 0;
    const LevelCoin e = coin[i];
    const float p = (z - e.q) * e.rgap;
    return (uint32_t)i + ((65535.5f - h) < p * 65536.0f ? 1u : 0u);
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

// Codes given as floats. At 8 bits one instruction per code converts and places it: the conversion to a
// byte rounds to nearest even and saturates to [0, 255], so it also accepts the unrounded grid position
// of weight_position_minmax and then yields clamp(rint(position), 0, 255), the code itself.
template <int BITS>
__device__ __forceinline__ uint32_t pack4(const float (&c)[4]) {
    uint32_t acc = 0;
    if constexpr (BITS == 8) {
#pragma unroll
        for (int i = 0; i < 4; ++i) acc = __builtin_amdgcn_cvt_pk_u8_f32(c[i], (uint32_t)i, acc);
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) acc |= (uint32_t)c[i] << (i * BITS);
    }
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
