/*
 * qsdp_ref.c -- CPU oracle for the QSDP codec and quantized SGD step.
 *
 * TEST INFRASTRUCTURE ONLY (see qsdp_ref.h). Plain C, one element at a time,
 * no blocking, no SIMD intrinsics, no code shared with the GPU library.
 * Build: gcc -O2 -std=c11 -ffp-contract=off -fno-fast-math -fopenmp -shared -fPIC
 *
 * Notation (per bucket): m elements v_0..v_{m-1}; b bits; L = 2^b - 1;
 * lo = min v, hi = max v; scale = (hi-lo)/L is the grid spacing the paper calls
 * delta, inv = L/(hi-lo); code in [0, L].
 */
#include "qsdp_ref.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

#define MAX_BUCKET 8192

static int g_threads = 1;

int qsdp_ref_set_threads(int threads) {
    if (threads >= 1) g_threads = threads;
    return g_threads;
}

/* ------------------------------------------------------------------------- */
/* Random numbers. The paper only asks for one random scalar per vector (Def. 1)*/
/* and independent coin flips (coin-flip definition); the generator is ours:   */
/* Philox4x32-10, counter-based, so that any shard of a vector can be          */
/* quantized alone and give the bytes the whole vector would give.             */
/* ------------------------------------------------------------------------- */

void qsdp_ref_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = (uint64_t)0xD2511F53u * (uint64_t)c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
        uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
        uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
        uint32_t n0 = hi1 ^ c1 ^ k0;
        uint32_t n1 = lo1;
        uint32_t n2 = hi0 ^ c3 ^ k1;
        uint32_t n3 = lo0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* Gradient stream (stream id 0): one Philox block serves the 8 elements with
 * the same e/8; element e takes the 16 bits h of word (e%8)/2, low half first. */
uint32_t qsdp_ref_grad_uniform16(uint64_t seed, uint64_t e) {
    uint64_t block = e / 8u;
    uint32_t ctr[4] = {(uint32_t)block, (uint32_t)(block >> 32), 0u, 0u};
    uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    uint32_t out[4];
    qsdp_ref_philox4x32_10(ctr, key, out);
    unsigned j = (unsigned)(e % 8u);
    uint32_t w = out[j / 2u];
    return (j % 2u) ? (w >> 16) : (w & 0xFFFFu);
}

/* The same as a real number: u = h * 2^-16 is exact in binary32 and lies in [0,1). */
float qsdp_ref_grad_uniform(uint64_t seed, uint64_t e) {
    return (float)qsdp_ref_grad_uniform16(seed, e) * 0x1p-16f;
}

/* Weight stream (stream id 1): one draw per call, whatever the shard.
 * xi = (top 24 bits of word 0) * 2^-24 - 1/2, exact, in [-1/2, 1/2). */
float qsdp_ref_weight_shift(uint64_t seed) {
    uint32_t ctr[4] = {0u, 0u, 1u, 0u};
    uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    uint32_t out[4];
    qsdp_ref_philox4x32_10(ctr, key, out);
    return (float)(out[0] >> 8) * 0x1p-24f - 0.5f;
}

/* Shift of the shared-shift gradient quantizer (stream id 2), same construction. */
float qsdp_ref_grad_shift(uint64_t seed) {
    uint32_t ctr[4] = {0u, 0u, 2u, 0u};
    uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    uint32_t out[4];
    qsdp_ref_philox4x32_10(ctr, key, out);
    return (float)(out[0] >> 8) * 0x1p-24f - 0.5f;
}

/* ------------------------------------------------------------------------- */
/* Sizes and argument checks                                                   */
/* ------------------------------------------------------------------------- */

static int args_ok(uint64_t n, int bits, int bucket) {
    return n >= 1 && bits >= 1 && bits <= 8 && bucket >= 32 && bucket <= MAX_BUCKET &&
           bucket % 32 == 0;
}

static uint64_t num_buckets(uint64_t n, int bucket) {
    return (n + (uint64_t)bucket - 1u) / (uint64_t)bucket;
}

size_t qsdp_ref_codes_bytes(uint64_t n, int bits, int bucket) {
    if (!args_ok(n, bits, bucket)) return 0;
    return (size_t)(num_buckets(n, bucket) * (uint64_t)bucket * (uint64_t)bits / 8u);
}

size_t qsdp_ref_meta_bytes(uint64_t n, int bucket) {
    if (!args_ok(n, 8, bucket)) return 0;
    return (size_t)(num_buckets(n, bucket) * 2u * sizeof(float));
}

/* ------------------------------------------------------------------------- */
/* One bucket                                                                  */
/* ------------------------------------------------------------------------- */

/* Min-max statistics of a bucket (Section 5.1: each bucket is scaled by its
 * own min and max). Signed zeros are canonicalised to +0 so that the stored
 * meta-data has one bit pattern. A bucket whose range is zero, not finite, or
 * so small that 2^16 * L/range overflows (the coin flip works in units of 2^-16
 * of a cell) is treated as constant: scale = inv = 0. */
static void bucket_stats(const float* v, int m, float Lf, int symmetric, float* lo_out,
                         float* hi_out, float* scale_out, float* inv_out) {
    float lo = v[0], hi = v[0];
    for (int i = 1; i < m; ++i) {
        if (v[i] < lo) lo = v[i];
        if (v[i] > hi) hi = v[i];
    }
    lo = lo + 0.0f;
    hi = hi + 0.0f;
    if (symmetric) { /* grid over [-a, a], a = max |v| (the scaling of Section 3.2) */
        float a = fmaxf(fabsf(lo), fabsf(hi));
        lo = -a + 0.0f;
        hi = a;
    }
    float range = hi - lo;
    float scale = 0.0f, inv = 0.0f;
    if (range > 0.0f && isfinite(range)) {
        float inv_try = Lf / range;
        if (isfinite(inv_try * 65536.0f)) {
            scale = range / Lf;
            inv = inv_try;
        }
    }
    *lo_out = lo; *hi_out = hi; *scale_out = scale; *inv_out = inv;
}

/* Coin-flip quantizer in bucket coordinates t = (g - lo)/scale in [0, L]: floor(t) with
 * probability 1 - frac(t), floor(t)+1 with probability frac(t). The coin is a 16-bit uniform
 * integer h, so the decision is taken in integers: the position is expressed in units of 2^-16
 * of a cell and rounded to the nearest unit (one fused multiply-add, then truncation),
 *     ti = min(floor(fma(g - lo, inv * 2^16, 1/2)), L * 2^16),
 * and the code is floor((ti + h) / 2^16): that is floor(t) + 1 for exactly (ti mod 2^16) of the
 * 2^16 values of h, the largest ones. The rounding of frac(t) to 16 bits is to nearest, so what it
 * adds to E[Q(g)] - g has no preferred sign (at most scale * 2^-17 either way). u[i] in [0,1)
 * carries h as h * 2^-16. */
static uint32_t grid_position16(float d, float inv16, uint32_t top16) {
    float t16 = fmaf(d, inv16, 0.5f);
    if (!(t16 >= 0.0f)) return 0u; /* cannot happen for finite input: d >= 0, inv16 >= 0 */
    if (t16 >= (float)top16) return top16;
    return (uint32_t)t16;
}

static void grad_bucket(const float* g, const float* u, int m, int bits, int symmetric,
                        uint8_t* code, float* base_out, float* scale_out) {
    float Lf = (float)((1 << bits) - 1);
    float lo, hi, scale, inv;
    bucket_stats(g, m, Lf, symmetric, &lo, &hi, &scale, &inv);
    uint32_t top16 = (uint32_t)((1 << bits) - 1) << 16;
    float inv16 = inv * 65536.0f;
    for (int i = 0; i < m; ++i) {
        uint32_t h = (uint32_t)(u[i] * 65536.0f);
        uint32_t ti = grid_position16(g[i] - lo, inv16, top16);
        code[i] = (uint8_t)((ti + h) >> 16);
    }
    *base_out = lo;
    *scale_out = scale;
}

/* Random-shift quantizer (Def. 1), per-bucket grid: with delta := scale and the
 * shift r := lo + xi*scale, the nearest point of delta*Z + r to x is
 * r + scale*round((x - lo)/scale - xi). The clamp to [0, L] only acts on the
 * binary32 rounding of t - xi near L + 1/2 and on the tie at xi = -1/2. */
static void weight_bucket_minmax(const float* x, int m, int bits, float xi, int symmetric,
                                 uint8_t* code, float* base_out, float* scale_out) {
    float Lf = (float)((1 << bits) - 1);
    float lo, hi, scale, inv;
    bucket_stats(x, m, Lf, symmetric, &lo, &hi, &scale, &inv);
    for (int i = 0; i < m; ++i) {
        float t = (x[i] - lo) * inv;
        float k = rintf(t - xi);
        k = fminf(fmaxf(k, 0.0f), Lf);
        code[i] = (uint8_t)(int)k;
    }
    *base_out = fmaf(xi, scale, lo);
    *scale_out = scale;
}

/* Random-shift quantizer (Def. 1), explicit grid delta*(Z + xi): lattice
 * coordinate k = round(x/delta - xi). A bucket stores k relative to the
 * coordinate k0 of its smallest element, in b bits; a coordinate further than
 * L from k0 is clamped and counted. */
static void weight_bucket_lattice(const float* x, int m, int bits, float delta, float xi,
                                  uint8_t* code, float* base_out, float* scale_out,
                                  uint64_t* sat) {
    float Lf = (float)((1 << bits) - 1);
    float lo = x[0];
    for (int i = 1; i < m; ++i)
        if (x[i] < lo) lo = x[i];
    lo = lo + 0.0f;
    float k0 = rintf(lo / delta - xi);
    for (int i = 0; i < m; ++i) {
        float k = rintf(x[i] / delta - xi);
        float c = k - k0;
        if (c > Lf) {
            c = Lf;
            *sat += 1u;
        }
        code[i] = (uint8_t)(int)c;
    }
    *base_out = (k0 + xi) * delta;
    *scale_out = delta;
}

static void weight_bucket(const float* x, int m, int bits, float delta, float xi, int symmetric,
                          uint8_t* code, float* base, float* scale, uint64_t* sat) {
    if (delta > 0.0f)
        weight_bucket_lattice(x, m, bits, delta, xi, code, base, scale, sat);
    else
        weight_bucket_minmax(x, m, bits, xi, symmetric, code, base, scale);
}

/* The variants of the two quantizers (flags of the *_ex entry points). */
static int is_symmetric(uint32_t flags) { return (flags & QSDP_REF_FLAG_SYMMETRIC) != 0; }

static float weight_shift_for(uint64_t seed, uint32_t flags) {
    return (flags & QSDP_REF_FLAG_NO_SHIFT) ? 0.0f : qsdp_ref_weight_shift(seed);
}

static float grad_shift_for(uint64_t seed, uint32_t flags) {
    return (flags & QSDP_REF_FLAG_NO_SHIFT) ? 0.0f : qsdp_ref_grad_shift(seed);
}

/* Gradient bucket under the flags: coin flips with the element uniforms u, or, with
 * GRAD_SHIFT, the random-shift quantizer itself (the appendix notes that it is an unbiased
 * quantizer in the sense required of Q^g), which draws nothing per element. */
static void grad_bucket_flags(const float* g, const float* u, int m, int bits, uint32_t flags,
                              float xi_g, uint8_t* code, float* base, float* scale) {
    if (flags & QSDP_REF_FLAG_GRAD_SHIFT)
        weight_bucket_minmax(g, m, bits, xi_g, is_symmetric(flags), code, base, scale);
    else
        grad_bucket(g, u, m, bits, is_symmetric(flags), code, base, scale);
}

/* Decoding: lattice point -> value, one fused multiply-add. */
static void dequant_bucket(const uint8_t* code, int m, float base, float scale, float* out) {
    for (int i = 0; i < m; ++i) out[i] = fmaf((float)code[i], scale, base);
}

/* Wire format of one bucket: the codes of its `bucket` slots (slots past the
 * end of a short last bucket hold 0) form a little-endian bit stream, element
 * i in bits [i*b, (i+1)*b); bit p of the stream is bit p%32 of word p/32. */
static void pack_bucket(const uint8_t* code, int m, int bits, int bucket, uint32_t* words) {
    int nwords = bucket * bits / 32;
    for (int w = 0; w < nwords; ++w) words[w] = 0u;
    for (int i = 0; i < m; ++i) {
        for (int q = 0; q < bits; ++q) {
            if ((code[i] >> q) & 1u) {
                int p = i * bits + q;
                words[p / 32] |= (uint32_t)1u << (p % 32);
            }
        }
    }
}

static void unpack_bucket(const uint32_t* words, int m, int bits, uint8_t* code) {
    for (int i = 0; i < m; ++i) {
        unsigned c = 0;
        for (int q = 0; q < bits; ++q) {
            int p = i * bits + q;
            c |= ((words[p / 32] >> (p % 32)) & 1u) << q;
        }
        code[i] = (uint8_t)c;
    }
}

/* binary32 -> bfloat16, round to nearest even (finite inputs). */
uint16_t qsdp_ref_f32_to_bf16(float v) {
    uint32_t bitsv;
    memcpy(&bitsv, &v, sizeof bitsv);
    bitsv += 0x7FFFu + ((bitsv >> 16) & 1u);
    return (uint16_t)(bitsv >> 16);
}

/* binary32 -> IEEE binary16, round to nearest even: subnormal results kept, values beyond the
 * largest finite half (65504 + half an ulp) become infinity. The half-precision format of the
 * paper's mixed-precision setting (Section 6, experimental setup). */
uint16_t qsdp_ref_f32_to_f16(float v) {
    uint32_t b;
    memcpy(&b, &v, sizeof b);
    uint32_t sign = (b >> 16) & 0x8000u;
    uint32_t mag = b & 0x7FFFFFFFu;
    if (mag > 0x7F800000u) return (uint16_t)(sign | 0x7E00u); /* NaN */
    if (mag == 0x7F800000u) return (uint16_t)(sign | 0x7C00u);
    int e = (int)(mag >> 23);
    if (e == 0) return (uint16_t)sign;            /* below 2^-126: far under half the smallest half subnormal */
    uint32_t m = (mag & 0x7FFFFFu) | 0x800000u;   /* |v| = m * 2^(e-150), m has 24 bits */
    int he = e - 127 + 15;                        /* biased half exponent if the result is normal */
    int drop = he >= 1 ? 13 : 13 + (1 - he);      /* low bits of m that do not fit (subnormals lose more) */
    if (drop > 24) return (uint16_t)sign;         /* |v| < 2^-25: rounds to zero */
    uint32_t q = m >> drop;
    uint32_t rem = m & ((1u << drop) - 1u);
    uint32_t half = 1u << (drop - 1);
    if (rem > half || (rem == half && (q & 1u))) q += 1u;
    /* normal: q carries the implicit one in bit 10, so adding it to (he-1)<<10 also lets a
     * rounding carry move into the exponent; subnormal: q is the result (0x400 = smallest normal) */
    uint32_t h = he >= 1 ? ((uint32_t)(he - 1) << 10) + q : q;
    if (h >= 0x7C00u) h = 0x7C00u;
    return (uint16_t)(sign | h);
}

static uint16_t to_half_format(float v, int out_dtype) {
    return out_dtype == QSDP_REF_F16 ? qsdp_ref_f32_to_f16(v) : qsdp_ref_f32_to_bf16(v);
}

static int out_dtype_ok(int out_dtype) {
    return out_dtype == QSDP_REF_F32 || out_dtype == QSDP_REF_BF16 || out_dtype == QSDP_REF_F16;
}

static int bucket_len(uint64_t n, int bucket, uint64_t j) {
    uint64_t start = j * (uint64_t)bucket;
    uint64_t rest = n - start;
    return rest < (uint64_t)bucket ? (int)rest : bucket;
}

/* ------------------------------------------------------------------------- */
/* Cores with the randomness passed in                                         */
/* ------------------------------------------------------------------------- */

int qsdp_ref_quantize_grad_u(const float* g, uint64_t n, int bits, int bucket, const float* u,
                             uint8_t* codes, float* meta) {
    return qsdp_ref_quantize_grad_u_ex(g, n, bits, bucket, u, 0u, codes, meta);
}

int qsdp_ref_quantize_grad_u_ex(const float* g, uint64_t n, int bits, int bucket, const float* u,
                                uint32_t flags, uint8_t* codes, float* meta) {
    if (!g || !u || !codes || !meta || !args_ok(n, bits, bucket)) return QSDP_REF_EINVAL;
    if (flags & QSDP_REF_FLAG_GRAD_SHIFT) return QSDP_REF_EINVAL; /* no uniforms in that variant */
    int64_t nb = (int64_t)num_buckets(n, bucket);
#pragma omp parallel for schedule(static) num_threads(g_threads)
    for (int64_t j = 0; j < nb; ++j) {
        uint64_t s = (uint64_t)j * (uint64_t)bucket;
        int m = bucket_len(n, bucket, (uint64_t)j);
        grad_bucket(g + s, u + s, m, bits, is_symmetric(flags), codes + s, &meta[2 * j],
                    &meta[2 * j + 1]);
    }
    return QSDP_REF_OK;
}

int qsdp_ref_quantize_weight_xi(const float* x, uint64_t n, int bits, int bucket, float delta,
                                float xi, uint8_t* codes, float* meta, uint64_t* n_saturated) {
    return qsdp_ref_quantize_weight_xi_ex(x, n, bits, bucket, delta, xi, 0u, codes, meta,
                                          n_saturated);
}

int qsdp_ref_quantize_weight_xi_ex(const float* x, uint64_t n, int bits, int bucket, float delta,
                                   float xi, uint32_t flags, uint8_t* codes, float* meta,
                                   uint64_t* n_saturated) {
    if (!x || !codes || !meta || !args_ok(n, bits, bucket)) return QSDP_REF_EINVAL;
    if (!(delta >= 0.0f) || !isfinite(delta)) return QSDP_REF_EINVAL;
    int64_t nb = (int64_t)num_buckets(n, bucket);
    uint64_t sat = 0;
#pragma omp parallel for schedule(static) num_threads(g_threads) reduction(+ : sat)
    for (int64_t j = 0; j < nb; ++j) {
        uint64_t s = (uint64_t)j * (uint64_t)bucket;
        int m = bucket_len(n, bucket, (uint64_t)j);
        uint64_t local = 0;
        weight_bucket(x + s, m, bits, delta, xi, is_symmetric(flags), codes + s, &meta[2 * j],
                      &meta[2 * j + 1], &local);
        sat += local;
    }
    if (n_saturated) *n_saturated += sat;
    return QSDP_REF_OK;
}

void qsdp_ref_pack(const uint8_t* codes, uint64_t n, int bits, int bucket, uint32_t* words) {
    int64_t nb = (int64_t)num_buckets(n, bucket);
    int wpb = bucket * bits / 32;
    for (int64_t j = 0; j < nb; ++j)
        pack_bucket(codes + (uint64_t)j * (uint64_t)bucket, bucket_len(n, bucket, (uint64_t)j),
                    bits, bucket, words + (uint64_t)j * (uint64_t)wpb);
}

void qsdp_ref_unpack(const uint32_t* words, uint64_t n, int bits, int bucket, uint8_t* codes) {
    int64_t nb = (int64_t)num_buckets(n, bucket);
    int wpb = bucket * bits / 32;
    for (int64_t j = 0; j < nb; ++j)
        unpack_bucket(words + (uint64_t)j * (uint64_t)wpb, bucket_len(n, bucket, (uint64_t)j),
                      bits, codes + (uint64_t)j * (uint64_t)bucket);
}

/* ------------------------------------------------------------------------- */
/* The four operations                                                         */
/* ------------------------------------------------------------------------- */

int qsdp_ref_quantize_grad(const float* g, uint64_t n, int bits, int bucket, uint64_t seed,
                           uint64_t index_offset, uint32_t* codes, float* meta) {
    return qsdp_ref_quantize_grad_ex(g, n, bits, bucket, seed, index_offset, 0u, codes, meta);
}

int qsdp_ref_quantize_grad_ex(const float* g, uint64_t n, int bits, int bucket, uint64_t seed,
                              uint64_t index_offset, uint32_t flags, uint32_t* codes, float* meta) {
    if (!g || !codes || !meta || !args_ok(n, bits, bucket)) return QSDP_REF_EINVAL;
    if (index_offset % 8u != 0u || (flags & ~QSDP_REF_FLAG_ALL)) return QSDP_REF_EINVAL;
    float xi_g = grad_shift_for(seed, flags);
    int64_t nb = (int64_t)num_buckets(n, bucket);
    int wpb = bucket * bits / 32;
#pragma omp parallel for schedule(static) num_threads(g_threads)
    for (int64_t j = 0; j < nb; ++j) {
        uint64_t s = (uint64_t)j * (uint64_t)bucket;
        int m = bucket_len(n, bucket, (uint64_t)j);
        float u[MAX_BUCKET];
        uint8_t code[MAX_BUCKET];
        for (int i = 0; i < m; ++i) u[i] = qsdp_ref_grad_uniform(seed, index_offset + s + (uint64_t)i);
        grad_bucket_flags(g + s, u, m, bits, flags, xi_g, code, &meta[2 * j], &meta[2 * j + 1]);
        pack_bucket(code, m, bits, bucket, codes + (uint64_t)j * (uint64_t)wpb);
    }
    return QSDP_REF_OK;
}

int qsdp_ref_quantize_weight(const float* x, uint64_t n, int bits, int bucket, float delta,
                             uint64_t seed, uint32_t* codes, float* meta,
                             uint64_t* n_saturated) {
    return qsdp_ref_quantize_weight_ex(x, n, bits, bucket, delta, seed, 0u, codes, meta,
                                       n_saturated);
}

int qsdp_ref_quantize_weight_ex(const float* x, uint64_t n, int bits, int bucket, float delta,
                                uint64_t seed, uint32_t flags, uint32_t* codes, float* meta,
                                uint64_t* n_saturated) {
    if (!x || !codes || !meta || !args_ok(n, bits, bucket)) return QSDP_REF_EINVAL;
    if (!(delta >= 0.0f) || !isfinite(delta) || (flags & ~QSDP_REF_FLAG_ALL)) return QSDP_REF_EINVAL;
    float xi = weight_shift_for(seed, flags);
    int64_t nb = (int64_t)num_buckets(n, bucket);
    int wpb = bucket * bits / 32;
    uint64_t sat = 0;
#pragma omp parallel for schedule(static) num_threads(g_threads) reduction(+ : sat)
    for (int64_t j = 0; j < nb; ++j) {
        uint64_t s = (uint64_t)j * (uint64_t)bucket;
        int m = bucket_len(n, bucket, (uint64_t)j);
        uint8_t code[MAX_BUCKET];
        uint64_t local = 0;
        weight_bucket(x + s, m, bits, delta, xi, is_symmetric(flags), code, &meta[2 * j],
                      &meta[2 * j + 1], &local);
        pack_bucket(code, m, bits, bucket, codes + (uint64_t)j * (uint64_t)wpb);
        sat += local;
    }
    if (n_saturated) *n_saturated += sat;
    return QSDP_REF_OK;
}

int qsdp_ref_dequantize(const uint32_t* codes, const float* meta, uint64_t n, int bits,
                        int bucket, int out_dtype, void* out) {
    if (!codes || !meta || !out || !args_ok(n, bits, bucket)) return QSDP_REF_EINVAL;
    if (!out_dtype_ok(out_dtype)) return QSDP_REF_EINVAL;
    int64_t nb = (int64_t)num_buckets(n, bucket);
    int wpb = bucket * bits / 32;
#pragma omp parallel for schedule(static) num_threads(g_threads)
    for (int64_t j = 0; j < nb; ++j) {
        uint64_t s = (uint64_t)j * (uint64_t)bucket;
        int m = bucket_len(n, bucket, (uint64_t)j);
        uint8_t code[MAX_BUCKET];
        float val[MAX_BUCKET];
        unpack_bucket(codes + (uint64_t)j * (uint64_t)wpb, m, bits, code);
        dequant_bucket(code, m, meta[2 * j], meta[2 * j + 1], val);
        if (out_dtype == QSDP_REF_F32) {
            for (int i = 0; i < m; ++i) ((float*)out)[s + (uint64_t)i] = val[i];
        } else {
            for (int i = 0; i < m; ++i) ((uint16_t*)out)[s + (uint64_t)i] = to_half_format(val[i], out_dtype);
        }
    }
    return QSDP_REF_OK;
}

/* Decode the slices of all peers and add them up in peer order, then scale. */
int qsdp_ref_dequantize_add(const uint32_t* codes, uint64_t codes_stride_words, const float* meta,
                            uint64_t meta_stride_floats, int npeers, uint64_t n, int bits,
                            int bucket, float alpha, float* out) {
    if (!codes || !meta || !out || npeers < 1 || !args_ok(n, bits, bucket) || !isfinite(alpha))
        return QSDP_REF_EINVAL;
    int64_t nb = (int64_t)num_buckets(n, bucket);
    int wpb = bucket * bits / 32;
#pragma omp parallel for schedule(static) num_threads(g_threads)
    for (int64_t j = 0; j < nb; ++j) {
        uint64_t s = (uint64_t)j * (uint64_t)bucket;
        int m = bucket_len(n, bucket, (uint64_t)j);
        uint8_t code[MAX_BUCKET];
        float val[MAX_BUCKET], sum[MAX_BUCKET];
        for (int p = 0; p < npeers; ++p) {
            const uint32_t* pc = codes + (uint64_t)p * codes_stride_words;
            const float* pm = meta + (uint64_t)p * meta_stride_floats;
            unpack_bucket(pc + (uint64_t)j * (uint64_t)wpb, m, bits, code);
            dequant_bucket(code, m, pm[2 * j], pm[2 * j + 1], val);
            for (int i = 0; i < m; ++i) sum[i] = (p == 0) ? val[i] : sum[i] + val[i];
        }
        for (int i = 0; i < m; ++i) out[s + (uint64_t)i] = alpha * sum[i];
    }
    return QSDP_REF_OK;
}

/* x <- Q^w(x - lr * Q^g(g)): per bucket, quantize the gradient, decode it,
 * take the step, quantize the result, decode it (the iterate lives on the
 * quantization grid). The same seed drives both random streams. */
int qsdp_ref_fused_step(float* x, const float* g, uint64_t n, float lr, int wbits, int gbits,
                        int bucket, float delta, uint64_t seed, uint64_t index_offset,
                        uint32_t* wcodes, float* wmeta, uint64_t* n_saturated) {
    return qsdp_ref_fused_step_ex(x, g, n, lr, wbits, gbits, bucket, delta, seed, index_offset, 0u,
                                  wcodes, wmeta, n_saturated);
}

int qsdp_ref_fused_step_ex(float* x, const float* g, uint64_t n, float lr, int wbits, int gbits,
                           int bucket, float delta, uint64_t seed, uint64_t index_offset,
                           uint32_t flags, uint32_t* wcodes, float* wmeta, uint64_t* n_saturated) {
    if (!x || !g || !args_ok(n, wbits, bucket) || !args_ok(n, gbits, bucket) ||
        (flags & ~(QSDP_REF_FLAG_ALL | QSDP_REF_FLAG_KEEP_MASTER)))
        return QSDP_REF_EINVAL;
    if (!(delta >= 0.0f) || !isfinite(delta) || !isfinite(lr)) return QSDP_REF_EINVAL;
    if ((wcodes == NULL) != (wmeta == NULL)) return QSDP_REF_EINVAL;
    if (index_offset % 8u != 0u) return QSDP_REF_EINVAL;
    int keep_master = (flags & QSDP_REF_FLAG_KEEP_MASTER) != 0;
    float xi = weight_shift_for(seed, flags);
    float xi_g = grad_shift_for(seed, flags);
    int64_t nb = (int64_t)num_buckets(n, bucket);
    int wpb = bucket * wbits / 32;
    uint64_t sat = 0;
#pragma omp parallel for schedule(static) num_threads(g_threads) reduction(+ : sat)
    for (int64_t j = 0; j < nb; ++j) {
        uint64_t s = (uint64_t)j * (uint64_t)bucket;
        int m = bucket_len(n, bucket, (uint64_t)j);
        float u[MAX_BUCKET], ghat[MAX_BUCKET], y[MAX_BUCKET];
        uint8_t gcode[MAX_BUCKET], wcode[MAX_BUCKET];
        float gbase, gscale, wbase, wscale;
        uint64_t local = 0;
        for (int i = 0; i < m; ++i) u[i] = qsdp_ref_grad_uniform(seed, index_offset + s + (uint64_t)i);
        grad_bucket_flags(g + s, u, m, gbits, flags, xi_g, gcode, &gbase, &gscale);
        dequant_bucket(gcode, m, gbase, gscale, ghat);
        for (int i = 0; i < m; ++i) y[i] = fmaf(-lr, ghat[i], x[s + (uint64_t)i]);
        weight_bucket(y, m, wbits, delta, xi, is_symmetric(flags), wcode, &wbase, &wscale, &local);
        if (keep_master) {
            for (int i = 0; i < m; ++i) x[s + (uint64_t)i] = y[i]; /* the partition stays unquantized */
        } else {
            dequant_bucket(wcode, m, wbase, wscale, x + s);
        }
        if (wcodes) {
            pack_bucket(wcode, m, wbits, bucket, wcodes + (uint64_t)j * (uint64_t)wpb);
            wmeta[2 * j] = wbase;
            wmeta[2 * j + 1] = wscale;
        }
        sat += local;
    }
    if (n_saturated) *n_saturated += sat;
    return QSDP_REF_OK;
}

int qsdp_ref_fused_step_codes(uint32_t* wcodes, float* wmeta, const float* g, uint64_t n, float lr,
                              int wbits, int gbits, int bucket, float delta, uint64_t seed,
                              uint64_t index_offset, uint32_t flags, uint64_t* n_saturated) {
    if (!wcodes || !wmeta || !g || !args_ok(n, wbits, bucket) || (flags & ~QSDP_REF_FLAG_ALL))
        return QSDP_REF_EINVAL; /* KEEP_MASTER: there is no full-precision partition here */
    float* x = (float*)malloc((size_t)n * sizeof(float));
    if (!x) return QSDP_REF_EINVAL;
    int rc = qsdp_ref_dequantize(wcodes, wmeta, n, wbits, bucket, QSDP_REF_F32, x);
    if (rc == QSDP_REF_OK)
        rc = qsdp_ref_fused_step_ex(x, g, n, lr, wbits, gbits, bucket, delta, seed, index_offset, flags,
                                    wcodes, wmeta, n_saturated);
    free(x);
    return rc;
}

/* The shard owner's update in Algorithm 2 with P workers: the quantized gradient slices of all
 * peers are decoded and averaged (as qsdp_ref_dequantize_add does, peers in order), the SGD step
 * is taken with that average, and the new weights are quantized by Q^w (what the next weight
 * gather transmits) and decoded:
 *   ghat = alpha * (((d_0 + d_1) + d_2) + ...);  y = fma(-lr, ghat, x);  x <- decode(Q^w(y)).
 * No Q^g is applied here: the gradients arrive already quantized by their senders. */
int qsdp_ref_recv_step(float* x, const uint32_t* gcodes, uint64_t codes_stride_words, const float* gmeta,
                       uint64_t meta_stride_floats, int npeers, uint64_t n, float alpha, float lr,
                       int wbits, int gbits, int bucket, float delta, uint64_t seed, uint32_t flags,
                       uint32_t* wcodes, float* wmeta, uint64_t* n_saturated) {
    if (!x || !args_ok(n, wbits, bucket) ||
        (flags & ~(QSDP_REF_FLAG_NO_SHIFT | QSDP_REF_FLAG_SYMMETRIC | QSDP_REF_FLAG_KEEP_MASTER)))
        return QSDP_REF_EINVAL;
    if (!isfinite(lr) || (wcodes == NULL) != (wmeta == NULL)) return QSDP_REF_EINVAL;
    float* ghat = (float*)malloc((size_t)n * sizeof(float));
    uint32_t* codes = wcodes ? wcodes : (uint32_t*)malloc(qsdp_ref_codes_bytes(n, wbits, bucket));
    float* meta = wmeta ? wmeta : (float*)malloc(qsdp_ref_meta_bytes(n, bucket));
    int rc = (ghat && codes && meta) ? QSDP_REF_OK : QSDP_REF_EINVAL;
    if (rc == QSDP_REF_OK)
        rc = qsdp_ref_dequantize_add(gcodes, codes_stride_words, gmeta, meta_stride_floats, npeers, n, gbits,
                                     bucket, alpha, ghat);
    if (rc == QSDP_REF_OK) {
        for (uint64_t i = 0; i < n; ++i) ghat[i] = fmaf(-lr, ghat[i], x[i]); /* y, in place */
        rc = qsdp_ref_quantize_weight_ex(ghat, n, wbits, bucket, delta, seed,
                                         flags & ~(uint32_t)QSDP_REF_FLAG_KEEP_MASTER, codes, meta, n_saturated);
    }
    if (rc == QSDP_REF_OK) {
        if (flags & QSDP_REF_FLAG_KEEP_MASTER)
            memcpy(x, ghat, (size_t)n * sizeof(float)); /* x <- y: the partition stays unquantized */
        else
            rc = qsdp_ref_dequantize(codes, meta, n, wbits, bucket, QSDP_REF_F32, x);
    }
    free(ghat);
    if (!wcodes) free(codes);
    if (!wmeta) free(meta);
    return rc;
}

/* ------------------------------------------------------------------------- */
/* Learned quantization levels (Section 5.2, Algorithm 1)                      */
/* ------------------------------------------------------------------------- */

int qsdp_ref_levels_uniform(int bits, float* levels) {
    if (bits < 1 || bits > 8 || !levels) return QSDP_REF_EINVAL;
    int K = 1 << bits;
    for (int k = 0; k < K; ++k) levels[k] = (float)k / (float)(K - 1);
    return QSDP_REF_OK;
}

static int levels_ok(const float* levels, int bits) {
    int K = 1 << bits;
    for (int k = 0; k < K; ++k) {
        if (!(levels[k] >= 0.0f && levels[k] <= 1.0f)) return 0;
        if (k > 0 && levels[k] < levels[k - 1]) return 0;
    }
    return 1;
}

/* Bucket-wise normalisation: z = (v - lo) * (1 / (hi - lo)); a degenerate bucket maps to 0. */
static void normalize_bucket(const float* v, int m, float* z, float* lo_out, float* range_out) {
    float lo, hi, scale_unused, inv_unused;
    bucket_stats(v, m, 1.0f, 0, &lo, &hi, &scale_unused, &inv_unused);
    float range = hi - lo;
    float inv = 0.0f;
    if (range > 0.0f && isfinite(range)) {
        float t = 1.0f / range;
        if (isfinite(t * 65536.0f)) inv = t; else range = 0.0f; /* the rule of bucket_stats */
    } else {
        range = 0.0f;
    }
    for (int i = 0; i < m; ++i) z[i] = (v[i] - lo) * inv;
    *lo_out = lo;
    *range_out = range;
}

/* Nearest level by the plain definition: smallest |z - q_k|, first index on ties. */
static int closest_level(float z, const float* levels, int K) {
    int best = 0;
    float best_d = fabsf(z - levels[0]);
    for (int k = 1; k < K; ++k) {
        float d = fabsf(z - levels[k]);
        if (d < best_d) {
            best_d = d;
            best = k;
        }
    }
    return best;
}

int qsdp_ref_quantize_levels(const float* v, uint64_t n, int bits, int bucket, const float* levels,
                             uint32_t* codes, float* meta) {
    if (!v || !levels || !codes || !meta || !args_ok(n, bits, bucket) || !levels_ok(levels, bits))
        return QSDP_REF_EINVAL;
    int64_t nb = (int64_t)num_buckets(n, bucket);
    int wpb = bucket * bits / 32;
    int K = 1 << bits;
#pragma omp parallel for schedule(static) num_threads(g_threads)
    for (int64_t j = 0; j < nb; ++j) {
        uint64_t s = (uint64_t)j * (uint64_t)bucket;
        int m = bucket_len(n, bucket, (uint64_t)j);
        float z[MAX_BUCKET];
        uint8_t code[MAX_BUCKET];
        normalize_bucket(v + s, m, z, &meta[2 * j], &meta[2 * j + 1]);
        for (int i = 0; i < m; ++i) code[i] = (uint8_t)closest_level(z[i], levels, K);
        pack_bucket(code, m, bits, bucket, codes + (uint64_t)j * (uint64_t)wpb);
    }
    return QSDP_REF_OK;
}

/* Unbiased rounding onto non-uniform levels: the coin-flip quantizer of the appendix between the
 * two levels that enclose z. With i the largest index such that q_i <= z and q_{i+1} the next
 * level (so q_i <= z < q_{i+1}) and p = (z - q_i) * (1 / (q_{i+1} - q_i)), the reciprocal of the gap
 * rounded to binary32 first: code = i + [1 - 2^-17 - u < p],
 * i.e. with u = h * 2^-16 the level above is taken for the round(p * 2^16) largest values of h
 * (p is rounded to 16 bits to nearest and large h rounds up, as in the uniform coin flip). z below the first level
 * gives code 0, z at or above the last gives K-1: no pair of levels encloses those, so the
 * quantizer is unbiased exactly on [q_0, q_{K-1}]. */
static int stochastic_level(float z, float u, const float* levels, int K) {
    if (!(z >= levels[0])) return 0;
    int i = 0;
    for (int k = 1; k < K; ++k)
        if (levels[k] <= z) i = k;
    if (i == K - 1) return K - 1;
    float gap = levels[i + 1] - levels[i]; /* > 0 by the choice of i */
    float r = 1.0f / gap;                  /* a property of the table: one division per level, not per value */
    float p = (z - levels[i]) * r;
    /* 2^16 - (h + 1/2) < p * 2^16: up for the round(p * 2^16) largest values of h (both sides exact) */
    return i + ((1.0f - 0x1p-17f) - u < p ? 1 : 0);
}

int qsdp_ref_quantize_levels_stochastic(const float* v, uint64_t n, int bits, int bucket, const float* levels,
                                        uint64_t seed, uint64_t index_offset, uint32_t* codes, float* meta) {
    if (!v || !levels || !codes || !meta || !args_ok(n, bits, bucket) || !levels_ok(levels, bits))
        return QSDP_REF_EINVAL;
    if (index_offset % 8u != 0u) return QSDP_REF_EINVAL;
    int64_t nb = (int64_t)num_buckets(n, bucket);
    int wpb = bucket * bits / 32;
    int K = 1 << bits;
#pragma omp parallel for schedule(static) num_threads(g_threads)
    for (int64_t j = 0; j < nb; ++j) {
        uint64_t s = (uint64_t)j * (uint64_t)bucket;
        int m = bucket_len(n, bucket, (uint64_t)j);
        float z[MAX_BUCKET];
        uint8_t code[MAX_BUCKET];
        normalize_bucket(v + s, m, z, &meta[2 * j], &meta[2 * j + 1]);
        for (int i = 0; i < m; ++i) {
            float u = qsdp_ref_grad_uniform(seed, index_offset + s + (uint64_t)i);
            code[i] = (uint8_t)stochastic_level(z[i], u, levels, K);
        }
        pack_bucket(code, m, bits, bucket, codes + (uint64_t)j * (uint64_t)wpb);
    }
    return QSDP_REF_OK;
}

/* The same with the uniform of every element given by the caller (for exhaustive tests). */
int qsdp_ref_quantize_levels_u(const float* v, uint64_t n, int bits, int bucket, const float* levels,
                               const float* u, uint8_t* codes, float* meta) {
    if (!v || !levels || !u || !codes || !meta || !args_ok(n, bits, bucket) || !levels_ok(levels, bits))
        return QSDP_REF_EINVAL;
    int64_t nb = (int64_t)num_buckets(n, bucket);
    int K = 1 << bits;
    for (int64_t j = 0; j < nb; ++j) {
        uint64_t s = (uint64_t)j * (uint64_t)bucket;
        int m = bucket_len(n, bucket, (uint64_t)j);
        float z[MAX_BUCKET];
        normalize_bucket(v + s, m, z, &meta[2 * j], &meta[2 * j + 1]);
        for (int i = 0; i < m; ++i) codes[s + (uint64_t)i] = (uint8_t)stochastic_level(z[i], u[s + (uint64_t)i], levels, K);
    }
    return QSDP_REF_OK;
}

int qsdp_ref_dequantize_levels(const uint32_t* codes, const float* meta, uint64_t n, int bits,
                               int bucket, const float* levels, int out_dtype, void* out) {
    if (!codes || !meta || !levels || !out || !args_ok(n, bits, bucket)) return QSDP_REF_EINVAL;
    if (!out_dtype_ok(out_dtype)) return QSDP_REF_EINVAL;
    int64_t nb = (int64_t)num_buckets(n, bucket);
    int wpb = bucket * bits / 32;
#pragma omp parallel for schedule(static) num_threads(g_threads)
    for (int64_t j = 0; j < nb; ++j) {
        uint64_t s = (uint64_t)j * (uint64_t)bucket;
        int m = bucket_len(n, bucket, (uint64_t)j);
        uint8_t code[MAX_BUCKET];
        unpack_bucket(codes + (uint64_t)j * (uint64_t)wpb, m, bits, code);
        for (int i = 0; i < m; ++i) {
            float val = fmaf(levels[code[i]], meta[2 * j + 1], meta[2 * j]);
            if (out_dtype == QSDP_REF_F32) ((float*)out)[s + (uint64_t)i] = val;
            else ((uint16_t*)out)[s + (uint64_t)i] = to_half_format(val, out_dtype);
        }
    }
    return QSDP_REF_OK;
}

int qsdp_ref_fit_levels(const float* v, uint64_t n, int bits, int bucket, float lr,
                        uint64_t max_batches, float* levels) {
    if (!v || !levels || !args_ok(n, bits, bucket) || !levels_ok(levels, bits)) return QSDP_REF_EINVAL;
    if (!(lr > 0.0f && lr < 1.0f)) return QSDP_REF_EINVAL;
    uint64_t nb = num_buckets(n, bucket);
    if (max_batches > 0 && max_batches < nb) nb = max_batches;
    int K = 1 << bits;
    /* keep[c] = (1 - lr)^c by repeated multiplication */
    static double keep[MAX_BUCKET + 1];
    double one_minus = 1.0 - (double)lr;
    keep[0] = 1.0;
    for (int c = 1; c <= bucket; ++c) keep[c] = keep[c - 1] * one_minus;
    for (uint64_t j = 0; j < nb; ++j) {
        uint64_t s = j * (uint64_t)bucket;
        int m = bucket_len(n, bucket, j);
        float z[MAX_BUCKET];
        float lo, range;
        normalize_bucket(v + s, m, z, &lo, &range);
        int64_t sum[256];
        uint32_t count[256];
        for (int k = 0; k < K; ++k) { sum[k] = 0; count[k] = 0; }
        for (int i = 0; i < m; ++i) {
            int k = closest_level(z[i], levels, K);
            sum[k] += (int64_t)(z[i] * 4294967296.0f); /* exact scaling, truncation */
            count[k] += 1u;
        }
        for (int k = 0; k < K; ++k) {
            if (count[k] == 0) continue;
            double mean = ((double)sum[k] / (double)count[k]) * (1.0 / 4294967296.0);
            double q = (double)levels[k];
            levels[k] = (float)(q - (1.0 - keep[count[k]]) * (q - mean));
        }
    }
    return QSDP_REF_OK;
}

/* Algorithm 1 exactly as Section 5.2 prints it: after the bucket-wise normalisation the values
 * are visited one by one, in storage order; each value picks the level closest to it in the
 * table AS IT STANDS at that moment, and that one level takes one gradient step of rate lr
 * towards the value, q <- q - lr*(q - v), before the next value is looked at. No batching: the
 * batch size of Appendix C does not enter. The table is carried in binary64 (the step is a
 * convex combination, so a level never leaves its cell and the table stays ascending) and
 * rounded to binary32 once, at the end. qsdp_ref_fit_levels above is the parallel reading of
 * the same algorithm that the GPU library implements; the tests measure one against the other. */
int qsdp_ref_fit_levels_sequential(const float* v, uint64_t n, int bits, int bucket, float lr,
                                   uint64_t max_batches, float* levels) {
    if (!v || !levels || !args_ok(n, bits, bucket) || !levels_ok(levels, bits)) return QSDP_REF_EINVAL;
    if (!(lr > 0.0f && lr < 1.0f)) return QSDP_REF_EINVAL;
    uint64_t nb = num_buckets(n, bucket);
    if (max_batches > 0 && max_batches < nb) nb = max_batches;
    int K = 1 << bits;
    double q[256];
    for (int k = 0; k < K; ++k) q[k] = (double)levels[k];
    for (uint64_t j = 0; j < nb; ++j) {
        uint64_t s = j * (uint64_t)bucket;
        int m = bucket_len(n, bucket, j);
        float z[MAX_BUCKET];
        float lo, range;
        normalize_bucket(v + s, m, z, &lo, &range);
        for (int i = 0; i < m; ++i) {
            double zi = (double)z[i];
            int best = 0; /* find_closest against the current table, first index on ties */
            double best_d = fabs(zi - q[0]);
            for (int k = 1; k < K; ++k) {
                double d = fabs(zi - q[k]);
                if (d < best_d) {
                    best_d = d;
                    best = k;
                }
            }
            q[best] = q[best] - (double)lr * (q[best] - zi);
        }
    }
    for (int k = 0; k < K; ++k) levels[k] = (float)q[k];
    return QSDP_REF_OK;
}

/* ------------------------------------------------------------------------- */
/* AdamW inside the quantized iteration (Appendix A names the optimizer)       */
/* ------------------------------------------------------------------------- */

/* One element of AdamW with decoupled weight decay, in binary32 and in this order:
 *   m <- fma(beta1, m, (1-beta1) g);  v <- fma(beta2, v, ((1-beta2) g) g);
 *   u = (m / bias1) / (sqrt(v / bias2) + eps);  returns y = fma(-lr, fma(wd, x, u), x). */
static float adamw_element(float x, float ghat, float* mom, float* var, float lr, float beta1, float beta2,
                           float omb1, float omb2, float eps, float weight_decay, float bias1, float bias2) {
    float mi = fmaf(beta1, *mom, omb1 * ghat);
    float vi = fmaf(beta2, *var, (omb2 * ghat) * ghat);
    *mom = mi;
    *var = vi;
    float upd = (mi / bias1) / (sqrtf(vi / bias2) + eps);
    return fmaf(-lr, fmaf(weight_decay, x, upd), x);
}

int qsdp_ref_fused_adamw_step(float* x, const float* g, float* mom, float* var, uint64_t n, float lr,
                              float beta1, float beta2, float eps, float weight_decay, float bias1,
                              float bias2, int wbits, int gbits, int bucket, float delta,
                              uint64_t seed, uint64_t index_offset, uint32_t flags,
                              uint32_t* wcodes, float* wmeta, uint64_t* n_saturated) {
    if (!x || !g || !mom || !var || !args_ok(n, wbits, bucket) || !args_ok(n, gbits, bucket) ||
        (flags & ~(QSDP_REF_FLAG_ALL | QSDP_REF_FLAG_KEEP_MASTER)))
        return QSDP_REF_EINVAL;
    if (!(delta >= 0.0f) || !isfinite(delta) || !isfinite(lr)) return QSDP_REF_EINVAL;
    if (!(beta1 >= 0.0f && beta1 < 1.0f && beta2 >= 0.0f && beta2 < 1.0f && eps > 0.0f && bias1 > 0.0f &&
          bias2 > 0.0f && isfinite(weight_decay)))
        return QSDP_REF_EINVAL;
    if ((wcodes == NULL) != (wmeta == NULL) || index_offset % 8u != 0u) return QSDP_REF_EINVAL;
    float xi = weight_shift_for(seed, flags);
    float xi_g = grad_shift_for(seed, flags);
    float omb1 = 1.0f - beta1, omb2 = 1.0f - beta2;
    int64_t nb = (int64_t)num_buckets(n, bucket);
    int wpb = bucket * wbits / 32;
    uint64_t sat = 0;
#pragma omp parallel for schedule(static) num_threads(g_threads) reduction(+ : sat)
    for (int64_t j = 0; j < nb; ++j) {
        uint64_t s = (uint64_t)j * (uint64_t)bucket;
        int m = bucket_len(n, bucket, (uint64_t)j);
        float u[MAX_BUCKET], ghat[MAX_BUCKET], y[MAX_BUCKET];
        uint8_t gcode[MAX_BUCKET], wcode[MAX_BUCKET];
        float gbase, gscale, wbase, wscale;
        uint64_t local = 0;
        for (int i = 0; i < m; ++i) u[i] = qsdp_ref_grad_uniform(seed, index_offset + s + (uint64_t)i);
        grad_bucket_flags(g + s, u, m, gbits, flags, xi_g, gcode, &gbase, &gscale);
        dequant_bucket(gcode, m, gbase, gscale, ghat);
        for (int i = 0; i < m; ++i) {
            uint64_t e = s + (uint64_t)i;
            y[i] = adamw_element(x[e], ghat[i], &mom[e], &var[e], lr, beta1, beta2, omb1, omb2, eps, weight_decay,
                                 bias1, bias2);
        }
        weight_bucket(y, m, wbits, delta, xi, is_symmetric(flags), wcode, &wbase, &wscale, &local);
        if (flags & QSDP_REF_FLAG_KEEP_MASTER) {
            for (int i = 0; i < m; ++i) x[s + (uint64_t)i] = y[i]; /* the partition stays unquantized */
        } else {
            dequant_bucket(wcode, m, wbase, wscale, x + s);
        }
        if (wcodes) {
            pack_bucket(wcode, m, wbits, bucket, wcodes + (uint64_t)j * (uint64_t)wpb);
            wmeta[2 * j] = wbase;
            wmeta[2 * j + 1] = wscale;
        }
        sat += local;
    }
    if (n_saturated) *n_saturated += sat;
    return QSDP_REF_OK;
}

/* The shard owner's update with P workers and AdamW (what the paper's experiments run:
 * Algorithm 2 with the optimizer of Appendix A): ghat = the scaled sum of the decoded peer slices
 * as in qsdp_ref_recv_step, then adamw_element per element, then Q^w of the result; x receives
 * its decode, or the value itself with KEEP_MASTER. */
int qsdp_ref_recv_adamw_step(float* x, float* mom, float* var, const uint32_t* gcodes,
                             uint64_t codes_stride_words, const float* gmeta, uint64_t meta_stride_floats,
                             int npeers, uint64_t n, float alpha, float lr, float beta1, float beta2, float eps,
                             float weight_decay, float bias1, float bias2, int wbits, int gbits, int bucket,
                             float delta, uint64_t seed, uint32_t flags, uint32_t* wcodes, float* wmeta,
                             uint64_t* n_saturated) {
    if (!x || !mom || !var || !args_ok(n, wbits, bucket) ||
        (flags & ~(QSDP_REF_FLAG_NO_SHIFT | QSDP_REF_FLAG_SYMMETRIC | QSDP_REF_FLAG_KEEP_MASTER)))
        return QSDP_REF_EINVAL;
    if (!isfinite(lr) || (wcodes == NULL) != (wmeta == NULL)) return QSDP_REF_EINVAL;
    if (!(beta1 >= 0.0f && beta1 < 1.0f && beta2 >= 0.0f && beta2 < 1.0f && eps > 0.0f && bias1 > 0.0f &&
          bias2 > 0.0f && isfinite(weight_decay)))
        return QSDP_REF_EINVAL;
    float* y = (float*)malloc((size_t)n * sizeof(float));
    uint32_t* codes = wcodes ? wcodes : (uint32_t*)malloc(qsdp_ref_codes_bytes(n, wbits, bucket));
    float* meta = wmeta ? wmeta : (float*)malloc(qsdp_ref_meta_bytes(n, bucket));
    int rc = (y && codes && meta) ? QSDP_REF_OK : QSDP_REF_EINVAL;
    if (rc == QSDP_REF_OK)
        rc = qsdp_ref_dequantize_add(gcodes, codes_stride_words, gmeta, meta_stride_floats, npeers, n, gbits,
                                     bucket, alpha, y); /* y holds ghat for now */
    if (rc == QSDP_REF_OK) {
        float omb1 = 1.0f - beta1, omb2 = 1.0f - beta2;
        for (uint64_t i = 0; i < n; ++i)
            y[i] = adamw_element(x[i], y[i], &mom[i], &var[i], lr, beta1, beta2, omb1, omb2, eps, weight_decay,
                                 bias1, bias2);
        rc = qsdp_ref_quantize_weight_ex(y, n, wbits, bucket, delta, seed,
                                         flags & ~(uint32_t)QSDP_REF_FLAG_KEEP_MASTER, codes, meta, n_saturated);
    }
    if (rc == QSDP_REF_OK) {
        if (flags & QSDP_REF_FLAG_KEEP_MASTER)
            memcpy(x, y, (size_t)n * sizeof(float));
        else
            rc = qsdp_ref_dequantize(codes, meta, n, wbits, bucket, QSDP_REF_F32, x);
    }
    free(y);
    if (!wcodes) free(codes);
    if (!wmeta) free(meta);
    return rc;
}
