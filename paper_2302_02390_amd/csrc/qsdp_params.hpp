// Launch parameters shared by the encoder kernels (wave and block kernels): the modes, the
// parameter block, the Philox key of a launch, the step arithmetic between the two quantizers,
// and the lookup of a bucket's tensor in a multi-tensor call.
#pragma once

#include "qsdp_device.hpp"

namespace qsdp {

// Largest bucket any kernel accepts (the block kernel and the level fit stage one bucket in LDS).
constexpr int kMaxBucket = 8192;

// What one launch of an encoder kernel does:
// MODE_GRAD: Q^g of a gradient vector: coin-flip (or shared-shift) rounding onto the bucket's
// min-max grid, packed codes + meta out (Section 3.2, the appendix definition).
// MODE_WEIGHT: Q^w of a weight vector: random-shift rounding onto the bucket's min-max grid or onto
// the explicit lattice delta, packed codes + meta out (Definition 1).
// MODE_FUSED: x <- Q^w(x - lr * Q^g(g)) in one pass, x updated in place, codes + meta of the new x
// optionally emitted (the iteration of Sections 3.3 / 4.1).
// MODE_FUSED_CODES: the fused step with the weights resident as packed codes + meta (the
// iterate always lies on its bucket grids, so codes + meta hold it exactly): decode, step,
// re-quantize, write codes + meta back in place; no fp32 copy of x is read or written.
// MODE_LEVELS: nearest-level encoding against a table of learned (non-uniform) levels in
// bucket-normalised coordinates.
// MODE_ADAMW: the fused step with AdamW (moments m, v in fp32, updated in place) between the
// two quantizers instead of the plain SGD update.
// MODE_RECV: the shard owner's step with P workers: the gradient is the scaled sum of the
// decoded slices of all peers (no Q^g here), then the SGD step and Q^w as in MODE_FUSED.
// MODE_RECV_ADAMW: the same with the AdamW update of MODE_ADAMW in place of the SGD step.
// MODE_ADAMW_CODES: MODE_ADAMW on code-resident weights (x_t decoded from codes + meta as in
// MODE_FUSED_CODES, the moments in fp32).
// MODE_SUM: only the first half of MODE_RECV: out = alpha * (sum of the decoded peer slices).
// MODE_LEVELS_COIN: MODE_LEVELS with the unbiased coin flip between the two enclosing levels
// instead of the nearest level (wave kernels only: a kernel of its own so that the nearest-level
// encoder does not carry the registers of the rounding uniforms; the block kernel takes
// MODE_LEVELS with FLAG_LEVELS_STOCHASTIC).
enum Mode { MODE_GRAD = 0, MODE_WEIGHT = 1, MODE_FUSED = 2, MODE_FUSED_CODES = 3, MODE_LEVELS = 4,
            MODE_ADAMW = 5, MODE_RECV = 6, MODE_RECV_ADAMW = 7, MODE_SUM = 8, MODE_LEVELS_COIN = 9,
            MODE_ADAMW_CODES = 10 };

constexpr bool mode_is_levels(int mode) { return mode == MODE_LEVELS || mode == MODE_LEVELS_COIN; }

constexpr bool mode_is_recv(int mode) { return mode == MODE_RECV || mode == MODE_RECV_ADAMW; }
constexpr bool mode_reads_peers(int mode) { return mode_is_recv(mode) || mode == MODE_SUM; }
constexpr bool mode_is_adamw(int mode) {
    return mode == MODE_ADAMW || mode == MODE_RECV_ADAMW || mode == MODE_ADAMW_CODES;
}
// the weights live as packed codes + meta (decoded in registers, overwritten by the new codes)
constexpr bool mode_codes_resident(int mode) { return mode == MODE_FUSED_CODES || mode == MODE_ADAMW_CODES; }
// the gradient is a local fp32 (or 16-bit) vector that goes through Q^g inside the kernel
constexpr bool mode_local_gradient(int mode) {
    return mode == MODE_GRAD || mode == MODE_FUSED || mode == MODE_FUSED_CODES || mode == MODE_ADAMW ||
           mode == MODE_ADAMW_CODES;
}
// modes that take the gradient in 16 bits and can write a 16-bit copy of the new weights
constexpr bool mode_mixed_precision(int mode) { return mode == MODE_GRAD || mode == MODE_FUSED || mode == MODE_ADAMW; }
// the AdamW moments are read and written next to a local gradient
constexpr bool mode_local_adamw(int mode) { return mode == MODE_ADAMW || mode == MODE_ADAMW_CODES; }

// One tensor of a multi-tensor ("segmented") call: `n` elements at element offset `offset` of
// the flat buffers; its buckets are numbered first_bucket .. first_bucket + ceil(n/B) - 1.
struct Segment {
    uint64_t offset;
    uint64_t n;
    uint64_t first_bucket;
};

struct Params {
    // tensors
    const float* g;      // GRAD, FUSED: gradient (2-byte values when g_half != 0)
    float* x;            // FUSED: in/out weights
    void* x16;           // FUSED, optional: the new quantized weights once more as bf16 / binary16 values
    const float* xin;    // WEIGHT, LEVELS: values to quantize
    const float* levels; // LEVELS: 2^wbits ascending levels in [0, 1]; segmented calls with
                         // levels_per_tensor: one such table per tensor, back to back
    float* mom;          // ADAMW: first moment, in/out
    float* var;          // ADAMW: second moment, in/out
    float beta1, beta2, omb1, omb2, eps, weight_decay, bias1, bias2;  // ADAMW
    uint32_t* codes;     // packed output (nullable in FUSED)
    float* meta;         // {base, scale} per bucket (nullable iff codes is)
    unsigned long long* n_saturated;  // nullable
    const Segment* segs;  // device table of nseg tensors, or nullptr: one tensor of n elements
    // RECV: peer k's packed gradient codes (gbits wide) start k * peer_codes_stride_words after
    // peer_codes, its meta k * peer_meta_stride_floats after peer_meta; ghat = alpha * sum
    const uint32_t* peer_codes;
    const float* peer_meta;
    uint64_t peer_codes_stride_words, peer_meta_stride_floats;
    int npeers;
    float alpha;
    // problem
    uint64_t n;             // elements (single tensor)
    uint64_t first_bucket;  // first bucket this launch handles
    uint64_t num_buckets;   // buckets this launch handles
    uint64_t block0;        // index_offset / 8
    uint32_t nseg;
    uint32_t x16_f16;  // x16 holds IEEE binary16 instead of bf16
    uint32_t g_half;  // 0: binary32 gradient; 1: bf16, 2: binary16, widened to binary32 (exactly) on load
    uint32_t levels_per_tensor;  // LEVELS with segs: table of tensor t at levels + t * 2^wbits
    uint32_t flags;  // FLAG_* variants
    int bucket;
    int gbits, wbits;
    float lr;
    float delta, inv_delta;  // lattice mode when delta > 0
    int delta_pow2;
    uint32_t key0, key1;
    // optional device-resident seed increment (8-byte aligned): the Philox key is taken from
    // seed + *seed_dev, read when the kernel starts, so that a captured launch can be replayed
    // with a seed that other work in the graph advances
    const unsigned long long* seed_dev;
};

struct PhiloxKey {
    uint32_t k0, k1;
};

__device__ __forceinline__ PhiloxKey launch_key(const Params& p) {
    PhiloxKey k = {p.key0, p.key1};
    if (p.seed_dev != nullptr) {
        const unsigned long long s = (((unsigned long long)p.key1 << 32) | p.key0) + *p.seed_dev;
        k.k0 = (uint32_t)s;
        k.k1 = (uint32_t)(s >> 32);
    }
    return k;
}

// The value that gets weight-quantized: x - lr * ghat, or the AdamW update (binary32, in the
// order m <- fma(b1, m, (1-b1) g); v <- fma(b2, v, ((1-b2) g) g); u = (m/c1) / (sqrt(v/c2) + eps);
// y = fma(-lr, fma(wd, x, u), x)).
template <int MODE>
__device__ __forceinline__ float step_value(const Params& p, float x, float ghat, float& mom, float& var) {
    if constexpr (mode_is_adamw(MODE)) {
        mom = fmaf(p.beta1, mom, p.omb1 * ghat);
        var = fmaf(p.beta2, var, (p.omb2 * ghat) * ghat);
        const float upd = (mom / p.bias1) / (sqrtf(var / p.bias2) + p.eps);
        return fmaf(-p.lr, fmaf(p.weight_decay, x, upd), x);
    } else {
        return fmaf(-p.lr, ghat, x);
    }
}

// Quantizer variants (same values as the QSDP_FLAG_* of the C header)
// FLAG_KEEP_MASTER (step modes): x receives the updated value itself, the codes still Q^w of it
// FLAG_LEVELS_STOCHASTIC (internal, MODE_LEVELS): coin-flip rounding between the enclosing levels
enum : uint32_t { FLAG_GRAD_SHIFT = 1u, FLAG_NO_SHIFT = 2u, FLAG_SYMMETRIC = 4u, FLAG_KEEP_MASTER = 8u,
                  FLAG_LEVELS_STOCHASTIC = 0x100u };

struct Shifts {
    float xi;    // weight shift
    float xi_g;  // gradient shift (FLAG_GRAD_SHIFT)
};

__device__ __forceinline__ Shifts draw_shifts(const Params& p, PhiloxKey key, bool weights) {
    Shifts s = {0.0f, 0.0f};
    if (!(p.flags & FLAG_NO_SHIFT)) {
        if (weights) s.xi = stream_shift(1u, key.k0, key.k1);
        if (p.flags & FLAG_GRAD_SHIFT) s.xi_g = stream_shift(2u, key.k0, key.k1);
    }
    return s;
}

// The tensor of a segmented call that owns bucket `gb`, given a WAVE-UNIFORM bucket gb0 <= gb
// (the first bucket the wave works on): binary search for gb0, then a per-lane walk forward that
// is taken only where the wave's buckets straddle tensors. The table is a __restrict__ kernel
// argument so that the uniform search compiles to scalar loads; through the vector memory path
// every probe would cost a round trip behind the streaming traffic.
__device__ __forceinline__ Segment find_segment(const Segment* __restrict__ segs, uint32_t nseg, uint64_t gb0,
                                                uint64_t gb, uint32_t* index = nullptr) {
    uint32_t lo = 0, hi = nseg;  // segs[lo].first_bucket <= gb0 < segs[hi].first_bucket
    while (hi - lo > 1) {
        const uint32_t mid = (lo + hi) >> 1;
        if (segs[mid].first_bucket <= gb0) lo = mid; else hi = mid;
    }
    Segment seg = segs[lo];
    uint64_t next_first = lo + 1 < nseg ? segs[lo + 1].first_bucket : ~0ull;
    uint32_t idx = lo;
    while (gb >= next_first) {
        ++idx;
        seg = segs[idx];
        next_first = idx + 1 < nseg ? segs[idx + 1].first_bucket : ~0ull;
    }
    if (index != nullptr) *index = idx;
    return seg;
}

// Where a bucket starts in the flat buffers (element index) and how many of its B slots hold
// elements. gb0: a wave-uniform bucket <= gb (see find_segment).
struct BucketRef {
    uint64_t e0;
    uint32_t m;
    uint32_t tensor;  // index in the segment table (0 for a single tensor)
};

__device__ __forceinline__ BucketRef locate_bucket(const Params& p, const Segment* __restrict__ segs, uint64_t gb0,
                                                   uint64_t gb, uint32_t B) {
    BucketRef ref;
    uint64_t left;
    ref.tensor = 0;
    if (segs != nullptr) {
        const Segment seg = find_segment(segs, p.nseg, gb0, gb, &ref.tensor);
        const uint64_t local = (gb - seg.first_bucket) * B;
        ref.e0 = seg.offset + local;
        left = seg.n - local;
    } else {
        ref.e0 = gb * B;
        left = p.n - ref.e0;
    }
    ref.m = left < B ? (uint32_t)left : B;
    return ref;
}

}  // namespace qsdp
