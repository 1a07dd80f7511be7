// Level fitting (Algorithm 1 in batched form).
#pragma once

#include "qsdp_block_kernel.hpp"  // block_minmax
#include "qsdp_params.hpp"

namespace qsdp {

// ---------------------------------------------------------------------------------------
// Level fitting (Algorithm 1 in batched form): ONE workgroup walks the buckets in order, since
// every batch starts from the levels the previous one left. Per bucket: stage the values in
// LDS, block min/max, assign every value to its nearest level (levels frozen), accumulate
// exact 32.32 fixed-point sums and counts per level with LDS atomics (order independent, so the
// result is reproducible), then level k takes its count_k steps of rate lr towards the mean
// of its values at once, in binary64: q <- q - (1 - (1-lr)^c)(q - mean). The chain of batches is
// kept short: the next batch's values are fetched while the current one is processed, the
// powers (1-lr)^c come from an LDS table filled once by repeated multiplication (the order in
// which single steps compound), and small level tables are accumulated per wave.
// ---------------------------------------------------------------------------------------
struct FitParams {
    const float* v;
    float* levels;  // in/out, 2^bits floats (one table per tensor when segs is given)
    uint64_t n;
    uint64_t num_batches;  // with segs: the cap on the batches of every tensor (0 = none)
    const Segment* segs;   // multi-tensor fit: workgroup t fits tensor t on its own table
    int bucket;
    int bits;
    float lr;
};

template <int BITS>
__global__ void __launch_bounds__(256) fit_levels_kernel(const FitParams p) {
    constexpr int K = 1 << BITS;
    constexpr int kCopies = K <= 16 ? 4 : 1;  // small tables: one accumulator set per wave (fewer atomic collisions)
    constexpr int kKeepMax = 2048;            // (1 - lr)^c is tabulated up to this count
    constexpr int kPre = 8;                   // values per thread fetched one batch ahead (buckets up to 2048)
    __shared__ float val[kMaxBucket];
    __shared__ float lv[K];
    __shared__ long long sum[kCopies][K];
    __shared__ unsigned int count[kCopies][K];
    __shared__ double keep_tab[kKeepMax + 1];
    __shared__ float red[8];
    const int tid = threadIdx.x;
    const int copy = kCopies == 1 ? 0 : (tid >> 6);
    const int B = p.bucket;
    const bool prefetch = B <= 256 * kPre;
    // this workgroup's tensor: the whole vector, or tensor blockIdx.x of a multi-tensor fit
    const float* v = p.v;
    float* levels = p.levels;
    uint64_t n = p.n, num_batches = p.num_batches;
    if (p.segs != nullptr) {
        const Segment seg = p.segs[blockIdx.x];
        v += seg.offset;
        levels += (uint64_t)blockIdx.x * K;
        n = seg.n;
        num_batches = (n + (uint64_t)B - 1) / (uint64_t)B;
        if (p.num_batches > 0 && p.num_batches < num_batches) num_batches = p.num_batches;
    }
    for (int k = tid; k < K; k += 256) lv[k] = levels[k];
    const double one_minus = 1.0 - (double)p.lr;
    if (tid == 0) {
        // (1 - lr)^c by repeated multiplication, the order in which c single steps compound
        double keep = 1.0;
        keep_tab[0] = 1.0;
        const int top = B < kKeepMax ? B : kKeepMax;
        for (int c = 1; c <= top; ++c) {
            keep *= one_minus;
            keep_tab[c] = keep;
        }
    }
    float nxt[kPre];
    auto fetch = [&](uint64_t j) {
        const uint64_t e0 = j * (uint64_t)B;
        const int m = (int)((n - e0 < (uint64_t)B) ? (n - e0) : (uint64_t)B);
#pragma unroll
        for (int q = 0; q < kPre; ++q) {
            const int i = tid + 256 * q;
            nxt[q] = i < m ? v[e0 + i] : 0.0f;
        }
    };
    if (prefetch && num_batches > 0) fetch(0);
    for (uint64_t j = 0; j < num_batches; ++j) {
        const uint64_t e0 = j * (uint64_t)B;
        const int m = (int)((n - e0 < (uint64_t)B) ? (n - e0) : (uint64_t)B);
        __syncthreads();  // previous batch's level update and LDS reads are complete (and keep_tab is written)
        float lo = __builtin_inff(), hi = -__builtin_inff();
        if (prefetch) {
#pragma unroll
            for (int q = 0; q < kPre; ++q) {
                const int i = tid + 256 * q;
                if (i < m) {
                    val[i] = nxt[q];
                    lo = fminf(lo, nxt[q]);
                    hi = fmaxf(hi, nxt[q]);
                }
            }
            if (j + 1 < num_batches) fetch(j + 1);  // in flight while this batch is processed
        } else {
            for (int i = tid; i < m; i += 256) {
                const float x = v[e0 + i];
                val[i] = x;
                lo = fminf(lo, x);
                hi = fmaxf(hi, x);
            }
        }
        for (int k = tid; k < kCopies * K; k += 256) {
            (&sum[0][0])[k] = 0;
            (&count[0][0])[k] = 0u;
        }
        block_minmax(lo, hi, red);  // contains the barriers that publish sum/count = 0 too
        const MinMaxGrid grid = make_minmax_grid(lo, hi, 1.0f, false);
        for (int i = tid; i < m; i += 256) {
            const float z = (val[i] - grid.lo) * grid.inv;
            const int k = nearest_level<BITS>(z, lv);
            atomicAdd(reinterpret_cast<unsigned long long*>(&sum[copy][k]),
                      (unsigned long long)(long long)(z * 4294967296.0f));
            atomicAdd(&count[copy][k], 1u);
        }
        __syncthreads();
        for (int k = tid; k < K; k += 256) {
            unsigned int c = 0;
            long long total = 0;  // exact integer sums: any order of accumulation gives the same value
#pragma unroll
            for (int w = 0; w < kCopies; ++w) {
                c += count[w][k];
                total += sum[w][k];
            }
            if (c != 0u) {
                double keep = keep_tab[c < (unsigned)kKeepMax ? c : (unsigned)kKeepMax];
                for (unsigned int t = kKeepMax; t < c; ++t) keep *= one_minus;
                const double mean = ((double)total / (double)c) * (1.0 / 4294967296.0);
                const double q = (double)lv[k];
                lv[k] = (float)(q - (1.0 - keep) * (q - mean));
            }
        }
    }
    __syncthreads();
    for (int k = tid; k < K; k += 256) levels[k] = lv[k];
}

}  // namespace qsdp
