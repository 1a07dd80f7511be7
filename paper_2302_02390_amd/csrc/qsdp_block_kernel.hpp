// Block kernel: one 256-thread workgroup per bucket, staged in LDS; any bucket size and code
// width. Serves the bucket sizes the wave kernels are not instantiated for.
#pragma once

#include "qsdp_params.hpp"

namespace qsdp {

// ---------------------------------------------------------------------------------------
// Block kernel: one workgroup per bucket, bucket staged in LDS.
// ---------------------------------------------------------------------------------------
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
__global__ void __launch_bounds__(256) block_kernel(const Params p, const Segment* __restrict__ segs) {
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
    const bool symmetric = (p.flags & FLAG_SYMMETRIC) != 0;
    const bool grad_shift = (p.flags & FLAG_GRAD_SHIFT) != 0;
    const bool keep_master = (p.flags & FLAG_KEEP_MASTER) != 0;
    const PhiloxKey key = launch_key(p);
    const Shifts shifts = draw_shifts(p, key, MODE != MODE_GRAD && MODE != MODE_LEVELS);
    const float xi = shifts.xi;
    if (tid == 0) sat_block = 0;

    for (uint64_t rel = blockIdx.x; rel < p.num_buckets; rel += gridDim.x) {
        const uint64_t bucket = p.first_bucket + rel;
        const BucketRef ref = locate_bucket(p, segs, bucket, bucket, (uint32_t)B);
        const uint64_t e0 = ref.e0;
        const int m = (int)ref.m;
        __syncthreads();  // previous bucket's LDS contents are dead
        float base = 0.0f, scale = 0.0f;
        int bits = (MODE == MODE_GRAD) ? p.gbits : p.wbits;

        // code-resident weights: the old iterate is decoded from the bucket's codes and meta
        const int wpb_in = B * p.wbits / 32;
        const uint32_t* old_words = mode_codes_resident(MODE) ? p.codes + bucket * (uint64_t)wpb_in : nullptr;
        const float old_base = mode_codes_resident(MODE) ? p.meta[2 * bucket] : 0.0f;
        const float old_scale = mode_codes_resident(MODE) ? p.meta[2 * bucket + 1] : 0.0f;

        if (mode_local_gradient(MODE)) {
            float lo = __builtin_inff(), hi = -__builtin_inff();
            for (int i = tid; i < m; i += 256) {
                const uint16_t* g16 = reinterpret_cast<const uint16_t*>(p.g);
                const float v = p.g_half == 1 ? widen16<true>(g16[e0 + i])
                                : p.g_half == 2 ? widen16<false>(g16[e0 + i]) : p.g[e0 + i];
                val[i] = v;
                lo = fminf(lo, v);
                hi = fmaxf(hi, v);
            }
            block_minmax(lo, hi, red);
            const MinMaxGrid grid = make_minmax_grid(lo, hi, Lg, symmetric);
            const float gbase = grad_shift ? fmaf(shifts.xi_g, grid.scale, grid.lo) : grid.lo;
            for (int i = tid; i < m; i += 256) {
                float c;
                if (grad_shift) {
                    c = weight_code_minmax(val[i], grid, Lg, shifts.xi_g);
                } else {
                    const uint64_t e = (p.block0 << 3) + e0 + (uint64_t)i;
                    uint32_t w[4];
                    const uint64_t blk = e >> 3;
                    philox4x32_10((uint32_t)blk, (uint32_t)(blk >> 32), 0u, 0u, key.k0, key.k1, w);
                    const uint32_t j = (uint32_t)(e & 7u);
                    const uint32_t word = w[j >> 1];
                    const uint32_t h = (j & 1u) ? (word >> 16) : (word & 0xFFFFu);
                    c = grad_code(val[i], grid, (uint32_t)Lg << 16, h);
                }
                if (MODE == MODE_GRAD) {
                    code[i] = (uint8_t)(uint32_t)c;
                } else {
                    const float ghat = fmaf(c, grid.scale, gbase);
                    float xold;
                    if (mode_codes_resident(MODE)) {
                        const int bit = i * p.wbits;
                        uint64_t two = old_words[bit >> 5];
                        if ((bit >> 5) + 1 < wpb_in) two |= (uint64_t)old_words[(bit >> 5) + 1] << 32;
                        const uint32_t cw = (uint32_t)(two >> (bit & 31)) & ((1u << p.wbits) - 1u);
                        xold = fmaf((float)cw, old_scale, old_base);
                    } else {
                        xold = p.x[e0 + i];
                    }
                    float mom = 0.0f, var = 0.0f;
                    if (mode_local_adamw(MODE)) {
                        mom = p.mom[e0 + i];
                        var = p.var[e0 + i];
                    }
                    val[i] = step_value<MODE>(p, xold, ghat, mom, var);
                    if (mode_local_adamw(MODE)) {
                        p.mom[e0 + i] = mom;
                        p.var[e0 + i] = var;
                    }
                }
            }
            base = gbase;
            scale = grid.scale;
        } else if (mode_is_recv(MODE)) {
            const int wpb_g = B * p.gbits / 32;
            const int bit_mask = (1 << p.gbits) - 1;
            for (int i = tid; i < m; i += 256) {
                const int bit = i * p.gbits;
                float sum = 0.0f;
                for (int peer = 0; peer < p.npeers; ++peer) {
                    const uint32_t* words = p.peer_codes + (uint64_t)peer * p.peer_codes_stride_words +
                                            bucket * (uint64_t)wpb_g;
                    const float* pm = p.peer_meta + (uint64_t)peer * p.peer_meta_stride_floats;
                    uint64_t two = words[bit >> 5];
                    if ((bit >> 5) + 1 < wpb_g) two |= (uint64_t)words[(bit >> 5) + 1] << 32;
                    const uint32_t c = (uint32_t)(two >> (bit & 31)) & (uint32_t)bit_mask;
                    const float d = fmaf((float)c, pm[2 * bucket + 1], pm[2 * bucket]);
                    sum = (peer == 0) ? d : sum + d;
                }
                float mom = 0.0f, var = 0.0f;
                if (MODE == MODE_RECV_ADAMW) {
                    mom = p.mom[e0 + i];
                    var = p.var[e0 + i];
                }
                val[i] = step_value<MODE>(p, p.x[e0 + i], p.alpha * sum, mom, var);
                if (MODE == MODE_RECV_ADAMW) {
                    p.mom[e0 + i] = mom;
                    p.var[e0 + i] = var;
                }
            }
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
            if (MODE == MODE_LEVELS) {
                const MinMaxGrid grid = make_minmax_grid(lo, hi, 1.0f, false);
                base = grid.lo;
                scale = grid.scale;
                const int K = 1 << p.wbits;
                const bool stochastic = (p.flags & FLAG_LEVELS_STOCHASTIC) != 0;
                const float* levels = p.levels + (p.levels_per_tensor != 0 ? (uint64_t)ref.tensor * K : 0);
                for (int i = tid; i < m; i += 256) {
                    const float z = (val[i] - grid.lo) * grid.inv;
                    if (stochastic) {
                        // plain scan for the largest index whose level is <= z, then the coin flip
                        const uint64_t e = (p.block0 << 3) + e0 + (uint64_t)i;
                        uint32_t w[4];
                        const uint64_t blk = e >> 3;
                        philox4x32_10((uint32_t)blk, (uint32_t)(blk >> 32), 0u, 0u, key.k0, key.k1, w);
                        const uint32_t j = (uint32_t)(e & 7u);
                        const uint32_t word = w[j >> 1];
                        const float h = (float)((j & 1u) ? (word >> 16) : (word & 0xFFFFu));
                        int c = 0;
                        if (z >= levels[0]) {
                            int lower = 0;
                            for (int k = 1; k < K; ++k)
                                if (levels[k] <= z) lower = k;
                            c = lower;
                            if (lower < K - 1) {
                                const float q0 = levels[lower];
                                const float prob = (z - q0) * (1.0f / (levels[lower + 1] - q0));
                                c = lower + ((65535.5f - h) < prob * 65536.0f ? 1 : 0);
                            }
                        }
                        code[i] = (uint8_t)c;
                        continue;
                    }
                    // plain scan: nearest level, first index on ties (the table is in global memory)
                    int best = 0;
                    float best_d = fabsf(z - levels[0]);
                    for (int k = 1; k < K; ++k) {
                        const float d = fabsf(z - levels[k]);
                        if (d < best_d) {
                            best_d = d;
                            best = k;
                        }
                    }
                    code[i] = (uint8_t)best;
                }
            } else if (lattice) {
                lo = lo + 0.0f;
                const float k0 = rintf(div_delta(lo, div) - xi);
                base = (k0 + xi) * p.delta;
                scale = p.delta;
                for (int i = tid; i < m; i += 256) {
                    const float c = weight_code_lattice(val[i], div, xi, k0, Lw, sat_here);
                    code[i] = (uint8_t)(uint32_t)c;
                    if (MODE == MODE_FUSED || MODE == MODE_ADAMW || mode_is_recv(MODE))
                        p.x[e0 + i] = keep_master ? val[i] : fmaf(c, scale, base);
                    if ((MODE == MODE_FUSED || MODE == MODE_ADAMW) && p.x16 != nullptr)
                        static_cast<uint16_t*>(p.x16)[e0 + i] = (uint16_t)half_bits(fmaf(c, scale, base), p.x16_f16 != 0);
                }
                if (sat_here) atomicAdd(&sat_block, sat_here);
            } else {
                const MinMaxGrid grid = make_minmax_grid(lo, hi, Lw, symmetric);
                base = fmaf(xi, grid.scale, grid.lo);
                scale = grid.scale;
                for (int i = tid; i < m; i += 256) {
                    const float c = weight_code_minmax(val[i], grid, Lw, xi);
                    code[i] = (uint8_t)(uint32_t)c;
                    if (MODE == MODE_FUSED || MODE == MODE_ADAMW || mode_is_recv(MODE))
                        p.x[e0 + i] = keep_master ? val[i] : fmaf(c, scale, base);
                    if ((MODE == MODE_FUSED || MODE == MODE_ADAMW) && p.x16 != nullptr)
                        static_cast<uint16_t*>(p.x16)[e0 + i] = (uint16_t)half_bits(fmaf(c, scale, base), p.x16_f16 != 0);
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

}  // namespace qsdp
