// Kernels of the QSDP codec for gfx950.
//
// Two families share the element arithmetic of qsdp_device.hpp:
//   * wave kernels: a bucket is owned by an aligned group of G lanes of one wave and never
//     leaves registers: one pass over HBM, no LDS, no barrier. Lane l of the group holds P
//     chunks of 8 consecutive elements: chunk c covers elements (c*G + l)*8 .. +7 of the
//     bucket (two 16-byte loads), which is exactly one Philox block and BITS bytes of codes.
//     Bucket size B = 8*G*P. A wave handles 64/G buckets at a time, waves stride over the
//     full buckets of the vector.
//   * block kernel: one 256-thread workgroup per bucket, staged in LDS; any bucket size, any
//     bits, short last bucket. Used for the shapes the wave kernels do not cover.
#pragma once

#include "qsdp_device.hpp"

namespace qsdp {

enum Mode { MODE_GRAD = 0, MODE_WEIGHT = 1, MODE_FUSED = 2 };

struct Params {
    // tensors
    const float* g;      // GRAD, FUSED: gradient
    float* x;            // FUSED: in/out weights
    const float* xin;    // WEIGHT: weights to quantize
    uint32_t* codes;     // packed output (nullable in FUSED)
    float* meta;         // {base, scale} per bucket (nullable iff codes is)
    unsigned long long* n_saturated;  // nullable
    // problem
    uint64_t n;             // elements
    uint64_t first_bucket;  // first bucket this launch handles
    uint64_t num_buckets;   // buckets this launch handles
    uint64_t block0;        // index_offset / 8
    int bucket;
    int gbits, wbits;
    float lr;
    float delta, inv_delta;  // lattice mode when delta > 0
    int delta_pow2;
    uint32_t key0, key1;
};

// ---------------------------------------------------------------------------------------
// Wave kernels
// ---------------------------------------------------------------------------------------
template <int G, int P>
struct Tile {
    static constexpr int kBucket = 8 * G * P;
    static constexpr int kBucketsPerWave = 64 / G;
    float v[P][8];
};

template <int G, int P>
__device__ __forceinline__ void load_tile(const float* base, int l, float (&v)[P][8]) {
#pragma unroll
    for (int c = 0; c < P; ++c) {
        const f4* p = reinterpret_cast<const f4*>(base + (size_t)(c * G + l) * 8);
        const f4 a = __builtin_nontemporal_load(p);
        const f4 b = __builtin_nontemporal_load(p + 1);
        v[c][0] = a[0]; v[c][1] = a[1]; v[c][2] = a[2]; v[c][3] = a[3];
        v[c][4] = b[0]; v[c][5] = b[1]; v[c][6] = b[2]; v[c][7] = b[3];
    }
}

template <int G, int P>
__device__ __forceinline__ void store_tile(float* base, int l, const float (&v)[P][8]) {
#pragma unroll
    for (int c = 0; c < P; ++c) {
        f4* p = reinterpret_cast<f4*>(base + (size_t)(c * G + l) * 8);
        const f4 a = {v[c][0], v[c][1], v[c][2], v[c][3]};
        const f4 b = {v[c][4], v[c][5], v[c][6], v[c][7]};
        __builtin_nontemporal_store(a, p);
        __builtin_nontemporal_store(b, p + 1);
    }
}

template <int G, int P>
__device__ __forceinline__ void tile_minmax(const float (&v)[P][8], float& lo, float& hi) {
    lo = v[0][0];
    hi = v[0][0];
#pragma unroll
    for (int c = 0; c < P; ++c)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            lo = fminf(lo, v[c][i]);
            hi = fmaxf(hi, v[c][i]);
        }
    lo = group_min<G>(lo);
    hi = group_max<G>(hi);
}

// MODE_GRAD / MODE_WEIGHT / MODE_FUSED over full buckets. BITS is the width of the codes
// that are stored (0: FUSED without code output). delta > 0 selects the explicit grid (a
// wave-uniform branch).
template <int MODE, int G, int P, int BITS>
__global__ void __launch_bounds__(256) wave_kernel(const Params p) {
    constexpr int B = 8 * G * P;
    constexpr int BPW = 64 / G;
    const int lane = threadIdx.x & 63;
    const int sub = lane / G;
    const int l = lane % G;
    const uint32_t wave_in_block = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint64_t waves_per_block = blockDim.x >> 6;
    const uint64_t wave0 = (uint64_t)blockIdx.x * waves_per_block + wave_in_block;
    const uint64_t nwaves = (uint64_t)gridDim.x * waves_per_block;
    const uint64_t ngroups = (p.num_buckets + BPW - 1) / BPW;

    const float Lg = (float)((1 << p.gbits) - 1);
    const float Lw = (float)((1 << p.wbits) - 1);
    const Divider div = {p.delta, p.inv_delta, p.delta_pow2 != 0};
    const bool lattice = p.delta > 0.0f;
    float xi = 0.0f;
    if (MODE != MODE_GRAD) xi = weight_shift(p.key0, p.key1);
    uint32_t saturated = 0;

    for (uint64_t q = wave0; q < ngroups; q += nwaves) {
        const uint64_t rel = q * BPW + sub;          // bucket within this launch
        const bool active = rel < p.num_buckets;
        const uint64_t bucket = p.first_bucket + (active ? rel : 0);
        const uint64_t e0 = bucket * (uint64_t)B;    // first element of the bucket

        float w[P][8];  // the values that get weight-quantized (x, or y = x - lr*ghat)
        float base = 0.0f, scale = 0.0f;

        if (MODE == MODE_GRAD || MODE == MODE_FUSED) {
            float gv[P][8];
            load_tile<G, P>(p.g + e0, l, gv);
            if (MODE == MODE_FUSED) load_tile<G, P>(p.x + e0, l, w);
            float lo, hi;
            tile_minmax<G, P>(gv, lo, hi);
            const MinMaxGrid grid = make_minmax_grid(lo, hi, Lg);
#pragma unroll
            for (int c = 0; c < P; ++c) {
                float h[8];
                grad_uniforms_x65536(p.block0 + (e0 >> 3) + (uint64_t)(c * G + l), p.key0, p.key1, h);
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const float code = grad_code(gv[c][i], grid, Lg, h[i]);
                    if (MODE == MODE_GRAD) {
                        gv[c][i] = code;
                    } else {
                        const float ghat = fmaf(code, grid.scale, grid.lo);
                        w[c][i] = fmaf(-p.lr, ghat, w[c][i]);
                    }
                }
            }
            if (MODE == MODE_GRAD) {
                if (active) {
                    uint8_t* cb = reinterpret_cast<uint8_t*>(p.codes) + (e0 >> 3) * BITS;
#pragma unroll
                    for (int c = 0; c < P; ++c)
                        store_chunk<BITS>(cb + (size_t)(c * G + l) * BITS, pack8<BITS>(gv[c]));
                    if (l == 0) {
                        p.meta[2 * bucket] = grid.lo;
                        p.meta[2 * bucket + 1] = grid.scale;
                    }
                }
                continue;
            }
        } else {
            load_tile<G, P>(p.xin + e0, l, w);
        }

        // weight quantization of w
        if (lattice) {
            float lo = w[0][0];
#pragma unroll
            for (int c = 0; c < P; ++c)
#pragma unroll
                for (int i = 0; i < 8; ++i) lo = fminf(lo, w[c][i]);
            lo = group_min<G>(lo) + 0.0f;
            const float k0 = rintf(div_delta(lo, div) - xi);
            base = (k0 + xi) * p.delta;
            scale = p.delta;
            uint32_t sat_here = 0;
#pragma unroll
            for (int c = 0; c < P; ++c)
#pragma unroll
                for (int i = 0; i < 8; ++i) w[c][i] = weight_code_lattice(w[c][i], div, xi, k0, Lw, sat_here);
            if (active) saturated += sat_here;
        } else {
            float lo, hi;
            tile_minmax<G, P>(w, lo, hi);
            const MinMaxGrid grid = make_minmax_grid(lo, hi, Lw);
            base = fmaf(xi, grid.scale, grid.lo);
            scale = grid.scale;
#pragma unroll
            for (int c = 0; c < P; ++c)
#pragma unroll
                for (int i = 0; i < 8; ++i) w[c][i] = weight_code_minmax(w[c][i], grid, Lw, xi);
        }

        if (active) {
            if (BITS != 0) {
                uint8_t* cb = reinterpret_cast<uint8_t*>(p.codes) + (e0 >> 3) * BITS;
#pragma unroll
                for (int c = 0; c < P; ++c)
                    store_chunk<(BITS ? BITS : 8)>(cb + (size_t)(c * G + l) * BITS,
                                                   pack8<(BITS ? BITS : 8)>(w[c]));
                if (l == 0) {
                    p.meta[2 * bucket] = base;
                    p.meta[2 * bucket + 1] = scale;
                }
            }
            if (MODE == MODE_FUSED) {
#pragma unroll
                for (int c = 0; c < P; ++c)
#pragma unroll
                    for (int i = 0; i < 8; ++i) w[c][i] = fmaf(w[c][i], scale, base);
                store_tile<G, P>(p.x + e0, l, w);
            }
        }
    }

    if (MODE != MODE_GRAD && p.n_saturated != nullptr) {
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) saturated += __shfl_down(saturated, off, 64);
        if (lane == 0 && saturated != 0) atomicAdd(p.n_saturated, (unsigned long long)saturated);
    }
}

// ---------------------------------------------------------------------------------------
// Block kernel: one workgroup per bucket, bucket staged in LDS.
// ---------------------------------------------------------------------------------------
constexpr int kMaxBucket = 8192;

__device__ __forceinline__ void block_minmax(float& lo, float& hi, float* red /* 8 floats */) {
    lo = group_min<64>(lo);
    hi = group_max<64>(hi);
    const int wave = threadIdx.x >> 6;
    __syncthreads();  // red may still be read from a previous use
    if ((threadIdx.x & 63) == 0) {
        red[wave] = lo;
        red[4 + wave] = hi;
    }
    __syncthreads();
    lo = fminf(fminf(red[0], red[1]), fminf(red[2], red[3]));
    hi = fmaxf(fmaxf(red[4], red[5]), fmaxf(red[6], red[7]));
}

template <int MODE>
__global__ void __launch_bounds__(256) block_kernel(const Params p) {
    __shared__ float val[kMaxBucket];
    __shared__ uint8_t code[kMaxBucket];
    __shared__ float red[8];
    __shared__ unsigned int sat_block;

    const int tid = threadIdx.x;
    const int B = p.bucket;
    const float Lg = (float)((1 << p.gbits) - 1);
    const float Lw = (float)((1 << p.wbits) - 1);
    const Divider div = {p.delta, p.inv_delta, p.delta_pow2 != 0};
    const bool lattice = p.delta > 0.0f;
    float xi = 0.0f;
    if (MODE != MODE_GRAD) xi = weight_shift(p.key0, p.key1);
    if (tid == 0) sat_block = 0;

    for (uint64_t rel = blockIdx.x; rel < p.num_buckets; rel += gridDim.x) {
        const uint64_t bucket = p.first_bucket + rel;
        const uint64_t e0 = bucket * (uint64_t)B;
        const int m = (int)((p.n - e0 < (uint64_t)B) ? (p.n - e0) : (uint64_t)B);
        __syncthreads();  // previous bucket's LDS contents are dead
        float base = 0.0f, scale = 0.0f;
        int bits = (MODE == MODE_GRAD) ? p.gbits : p.wbits;

        if (MODE == MODE_GRAD || MODE == MODE_FUSED) {
            float lo = __builtin_inff(), hi = -__builtin_inff();
            for (int i = tid; i < m; i += 256) {
                const float v = p.g[e0 + i];
                val[i] = v;
                lo = fminf(lo, v);
                hi = fmaxf(hi, v);
            }
            block_minmax(lo, hi, red);
            const MinMaxGrid grid = make_minmax_grid(lo, hi, Lg);
            for (int i = tid; i < m; i += 256) {
                const uint64_t e = (p.block0 << 3) + e0 + (uint64_t)i;
                uint32_t w[4];
                const uint64_t blk = e >> 3;
                philox4x32_10((uint32_t)blk, (uint32_t)(blk >> 32), 0u, 0u, p.key0, p.key1, w);
                const uint32_t j = (uint32_t)(e & 7u);
                const uint32_t word = w[j >> 1];
                const float h = (float)((j & 1u) ? (word >> 16) : (word & 0xFFFFu));
                const float c = grad_code(val[i], grid, Lg, h);
                if (MODE == MODE_GRAD) {
                    code[i] = (uint8_t)(uint32_t)c;
                } else {
                    const float ghat = fmaf(c, grid.scale, grid.lo);
                    val[i] = fmaf(-p.lr, ghat, p.x[e0 + i]);
                }
            }
            base = grid.lo;
            scale = grid.scale;
        } else {
            for (int i = tid; i < m; i += 256) val[i] = p.xin[e0 + i];
        }

        if (MODE != MODE_GRAD) {
            // each thread re-reads only the val[] entries it wrote: no barrier needed here
            float lo = __builtin_inff(), hi = -__builtin_inff();
            for (int i = tid; i < m; i += 256) {
                lo = fminf(lo, val[i]);
                hi = fmaxf(hi, val[i]);
            }
            block_minmax(lo, hi, red);
            unsigned int sat_here = 0;
            if (lattice) {
                lo = lo + 0.0f;
                const float k0 = rintf(div_delta(lo, div) - xi);
                base = (k0 + xi) * p.delta;
                scale = p.delta;
                for (int i = tid; i < m; i += 256) {
                    const float c = weight_code_lattice(val[i], div, xi, k0, Lw, sat_here);
                    code[i] = (uint8_t)(uint32_t)c;
                    if (MODE == MODE_FUSED) p.x[e0 + i] = fmaf(c, scale, base);
                }
                if (sat_here) atomicAdd(&sat_block, sat_here);
            } else {
                const MinMaxGrid grid = make_minmax_grid(lo, hi, Lw);
                base = fmaf(xi, grid.scale, grid.lo);
                scale = grid.scale;
                for (int i = tid; i < m; i += 256) {
                    const float c = weight_code_minmax(val[i], grid, Lw, xi);
                    code[i] = (uint8_t)(uint32_t)c;
                    if (MODE == MODE_FUSED) p.x[e0 + i] = fmaf(c, scale, base);
                }
            }
        }

        if (p.codes != nullptr) {
            __syncthreads();  // code[] complete
            const int wpb = B * bits / 32;
            uint32_t* out = p.codes + bucket * (uint64_t)wpb;
            for (int w = tid; w < wpb; w += 256) {
                const int first = (32 * w) / bits;
                int last = (32 * w + 31) / bits;
                if (last > B - 1) last = B - 1;
                uint32_t word = 0;
                for (int e = first; e <= last; ++e) {
                    const uint32_t c = (e < m) ? (uint32_t)code[e] : 0u;
                    const int sh = e * bits - 32 * w;
                    word |= (sh >= 0) ? (c << sh) : (c >> (-sh));
                }
                out[w] = word;
            }
            if (tid == 0) {
                p.meta[2 * bucket] = base;
                p.meta[2 * bucket + 1] = scale;
            }
        }
    }

    if (MODE != MODE_GRAD && p.n_saturated != nullptr) {
        __syncthreads();
        if (tid == 0 && sat_block != 0) atomicAdd(p.n_saturated, (unsigned long long)sat_block);
    }
}

// ---------------------------------------------------------------------------------------
// Decoding: elementwise, a lane per chunk of 8 elements (BITS bytes in, 16 or 32 bytes out).
// ---------------------------------------------------------------------------------------
struct DequantParams {
    const uint32_t* codes;
    const float* meta;
    void* out;
    uint64_t n;
    uint64_t nchunks;  // ceil(n / 8)
    int bucket;
};

template <int BITS, bool BF16>
__global__ void __launch_bounds__(256) dequant_kernel(const DequantParams p) {
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    const uint8_t* cb = reinterpret_cast<const uint8_t*>(p.codes);
    const uint32_t chunks_per_bucket = (uint32_t)p.bucket >> 3;
    for (uint64_t ch = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; ch < p.nchunks; ch += stride) {
        const uint64_t v = load_chunk<BITS>(cb + ch * BITS);
        const uint64_t bucket = ch / chunks_per_bucket;
        const float base = p.meta[2 * bucket];
        const float scale = p.meta[2 * bucket + 1];
        float o[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const uint32_t c = (uint32_t)(v >> (i * BITS)) & ((1u << BITS) - 1u);
            o[i] = fmaf((float)c, scale, base);
        }
        const uint64_t e = ch * 8;
        if (e + 8 <= p.n) {
            if (BF16) {
                u4 w;
#pragma unroll
                for (int i = 0; i < 4; ++i) w[i] = bf16_bits(o[2 * i]) | (bf16_bits(o[2 * i + 1]) << 16);
                __builtin_nontemporal_store(w, reinterpret_cast<u4*>(static_cast<uint16_t*>(p.out) + e));
            } else {
                f4* q = reinterpret_cast<f4*>(static_cast<float*>(p.out) + e);
                const f4 a = {o[0], o[1], o[2], o[3]};
                const f4 b = {o[4], o[5], o[6], o[7]};
                __builtin_nontemporal_store(a, q);
                __builtin_nontemporal_store(b, q + 1);
            }
        } else {
            for (int i = 0; i < 8; ++i) {
                if (e + i < p.n) {
                    if (BF16) static_cast<uint16_t*>(p.out)[e + i] = (uint16_t)bf16_bits(o[i]);
                    else static_cast<float*>(p.out)[e + i] = o[i];
                }
            }
        }
    }
}

}  // namespace qsdp
