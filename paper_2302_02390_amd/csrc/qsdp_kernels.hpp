// Kernels of the QSDP codec for gfx950.
//
// Two families share the element arithmetic of qsdp_device.hpp:
//   * wave kernels: a bucket is owned by an aligned group of G lanes of one wave and its values
//     never leave registers: one pass over HBM, no barrier (LDS only stages the packed codes so
//     that they are written with 16-byte stores). The bucket is cut into R rows
//     of 4*G elements; lane l of the group holds elements (r*G + l)*4 .. +3 of every row r, so
//     each load/store instruction of a wave touches whole contiguous 16*G-byte segments.
//     Bucket size B = 4*G*R, R even. A Philox block (8 elements) and a packed code chunk
//     (8 codes = BITS bytes) span the lane pair (l even, l+1) of one row: for each row pair
//     (2c, 2c+1) the even lane owns the block/chunk of row 2c and the odd lane that of row
//     2c+1, and the pair swaps halves with one DPP quad permute. A wave handles 64/G buckets
//     at a time, one wave per such group (waves stride only past 2^20 workgroups); a short last
//     bucket takes a guarded element-wise path of the same kernel. Buckets larger than one
//     wave's tile are shared by the W waves of a workgroup (B = 4*G*R*W, G = 64): each wave
//     owns a contiguous 1/W of the bucket and the waves combine their min/max through LDS.
//   * block kernel: one 256-thread workgroup per bucket, staged in LDS; any bucket size, any
//     bits. Used for the bucket sizes the wave kernels are not instantiated for (several times
//     slower: the values make a round trip through LDS and the codes are packed bit by bit).
// Decoders, the decode-and-sum kernel and the level-fitting kernel follow at the end.
#pragma once

#include "qsdp_device.hpp"

namespace qsdp {

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
// MODE_SUM: only the first half of MODE_RECV: out = alpha * (sum of the decoded peer slices).
// MODE_LEVELS_COIN: MODE_LEVELS with the unbiased coin flip between the two enclosing levels
// instead of the nearest level (wave kernels only: a kernel of its own so that the nearest-level
// encoder does not carry the registers of the rounding uniforms; the block kernel takes
// MODE_LEVELS with FLAG_LEVELS_STOCHASTIC).
enum Mode { MODE_GRAD = 0, MODE_WEIGHT = 1, MODE_FUSED = 2, MODE_FUSED_CODES = 3, MODE_LEVELS = 4,
            MODE_ADAMW = 5, MODE_RECV = 6, MODE_RECV_ADAMW = 7, MODE_SUM = 8, MODE_LEVELS_COIN = 9 };

constexpr bool mode_is_levels(int mode) { return mode == MODE_LEVELS || mode == MODE_LEVELS_COIN; }

constexpr bool mode_is_recv(int mode) { return mode == MODE_RECV || mode == MODE_RECV_ADAMW; }
constexpr bool mode_reads_peers(int mode) { return mode_is_recv(mode) || mode == MODE_SUM; }
constexpr bool mode_is_adamw(int mode) { return mode == MODE_ADAMW || mode == MODE_RECV_ADAMW; }

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

// ---------------------------------------------------------------------------------------
// Wave kernels
// ---------------------------------------------------------------------------------------
// Lane l's rows of a tile of 4*G*R elements at `base`. `m` = how many of the tile's elements
// exist; `partial` (wave-uniform) selects the guarded element-wise path for a short bucket.
template <int G, int R>
__device__ __forceinline__ void load_rows(const float* base, int l, int m, bool partial, float (&v)[R][4]) {
    if (!partial) {
        const f4* p = reinterpret_cast<const f4*>(base) + l;
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const f4 a = __builtin_nontemporal_load(p + r * G);
            v[r][0] = a[0]; v[r][1] = a[1]; v[r][2] = a[2]; v[r][3] = a[3];
        }
    } else {
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int idx = (r * G + l) * 4 + i;
                v[r][i] = idx < m ? base[idx] : 0.0f;
            }
    }
}

// A 2-byte floating-point value widened to binary32 (exact in both formats): bf16 is the upper
// half of the binary32 pattern, binary16 goes through the hardware conversion.
template <bool BF16>
__device__ __forceinline__ float widen16(uint32_t h) {
    if (BF16) return __builtin_bit_cast(float, h << 16);
    return (float)__builtin_bit_cast(_Float16, (uint16_t)h);
}

// The same tile read from 2-byte values, 8 bytes per lane and row.
template <int G, int R, bool BF16>
__device__ __forceinline__ void load_rows_half(const uint16_t* base, int l, int m, bool partial, float (&v)[R][4]) {
    if (!partial) {
        const u2* p = reinterpret_cast<const u2*>(base) + l;
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const u2 a = __builtin_nontemporal_load(p + r * G);
            v[r][0] = widen16<BF16>(a[0] & 0xFFFFu);
            v[r][1] = widen16<BF16>(a[0] >> 16);
            v[r][2] = widen16<BF16>(a[1] & 0xFFFFu);
            v[r][3] = widen16<BF16>(a[1] >> 16);
        }
    } else {
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int idx = (r * G + l) * 4 + i;
                v[r][i] = idx < m ? widen16<BF16>(base[idx]) : 0.0f;
            }
    }
}

template <int G, int R>
__device__ __forceinline__ void store_rows(float* base, int l, int m, bool partial, const float (&v)[R][4]) {
    if (!partial) {
        f4* p = reinterpret_cast<f4*>(base) + l;
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const f4 a = {v[r][0], v[r][1], v[r][2], v[r][3]};
            __builtin_nontemporal_store(a, p + r * G);
        }
    } else {
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int idx = (r * G + l) * 4 + i;
                if (idx < m) base[idx] = v[r][i];
            }
    }
}

// min and max over the bucket (the group's G lanes); slots at or past m do not take part
template <int G, int R>
__device__ __forceinline__ void rows_minmax(const float (&v)[R][4], int l, int m, bool partial, float& lo,
                                            float& hi) {
    if (!partial) {
        lo = v[0][0];
        hi = v[0][0];
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                lo = fminf(lo, v[r][i]);
                hi = fmaxf(hi, v[r][i]);
            }
    } else {
        lo = __builtin_inff();
        hi = -__builtin_inff();
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const bool valid = (r * G + l) * 4 + i < m;
                lo = valid ? fminf(lo, v[r][i]) : lo;
                hi = valid ? fmaxf(hi, v[r][i]) : hi;
            }
    }
    lo = group_min<G>(lo);
    hi = group_max<G>(hi);
}

// Slots at or past m (a short bucket) carry code 0. Only called on the guarded path.
template <int G, int R, typename CodeT>
__device__ __forceinline__ void zero_slots_past_end(CodeT (&c)[R][4], int l, int m) {
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if ((r * G + l) * 4 + i >= m) c[r][i] = CodeT(0);
}

// Pack the codes of all rows and stage them in LDS in wire order, then write the wave's code
// tile (its 64/G buckets are consecutive, so the tile is 32*R*BITS contiguous bytes) with
// 16-byte stores, one contiguous run per instruction. c[r][i] are the codes of this lane's
// elements; `stage` is this wave's LDS tile; `tile_out` the tile's place in the code buffer;
// buckets at or past `active_buckets` of the wave's 64/G are not written.
template <int G, int R, int BITS, typename CodeT>
__device__ __forceinline__ void store_codes(uint8_t* stage, u4* tile_out, int lane, int active_buckets,
                                            const CodeT (&c)[R][4]) {
    constexpr int kBucketBytes = 4 * G * R * BITS / 8;
    constexpr int kPieces = 2 * R * BITS;  // 16-byte pieces in the tile
    const int l = lane % G;
    const int sub = lane / G;
    const int odd = l & 1;
#pragma unroll
    for (int cp = 0; cp < R / 2; ++cp) {
        const uint32_t q0 = pack4<BITS>(c[2 * cp]);      // this lane's 4 codes of row 2cp
        const uint32_t q1 = pack4<BITS>(c[2 * cp + 1]);  // ... of row 2cp+1
        const uint32_t recv = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(odd ? q0 : q1), 0xB1, 0xF,
                                                                    0xF, false);
        // even lane: chunk of row 2cp = own q0 (low half) | partner's q0; odd lane: chunk of
        // row 2cp+1 = partner's q1 (low half) | own q1
        const uint64_t chunk = odd ? ((uint64_t)recv | ((uint64_t)q1 << (4 * BITS)))
                                   : ((uint64_t)q0 | ((uint64_t)recv << (4 * BITS)));
        const int chunk_index = ((2 * cp + odd) * G + (l - odd)) >> 1;
        store_chunk<BITS>(stage + sub * kBucketBytes + chunk_index * BITS, chunk);
    }
    // LDS traffic of one wave is processed in order; keep the compiler from reordering it
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const u4* staged = reinterpret_cast<const u4*>(stage);
#pragma unroll
    for (int k0 = 0; k0 < kPieces; k0 += 64) {
        const int k = k0 + lane;
        if (k < kPieces && (k * 16) / kBucketBytes < active_buckets)
            __builtin_nontemporal_store(staged[k], tile_out + k);
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// The reverse of store_codes, in two phases so that several tiles can be in flight: fetch the
// wave's code tile with 16-byte loads (one piece per lane: 2*R*BITS <= 64 pieces), then stage
// it in LDS and give every lane the codes of its own elements (as floats). The even lane reads
// the chunk of row 2cp (its own 4 codes, then its partner's), the odd lane that of row 2cp+1
// (its partner's 4 codes, then its own); one DPP quad permute hands each lane the half it lacks.
template <int G, int R, int BITS>
__device__ __forceinline__ u4 fetch_code_tile(const u4* tile_in, int lane, int active_buckets) {
    constexpr int kBucketBytes = 4 * G * R * BITS / 8;
    constexpr int kPieces = 2 * R * BITS;
    static_assert(kPieces <= 64, "one 16-byte piece per lane");
    u4 piece = {0u, 0u, 0u, 0u};
    if (lane < kPieces && (lane * 16) / kBucketBytes < active_buckets) piece = __builtin_nontemporal_load(tile_in + lane);
    return piece;
}

template <int G, int R, int BITS>
__device__ __forceinline__ void unstage_codes(uint8_t* stage, u4 piece, int lane, float (&c)[R][4]) {
    constexpr int kBucketBytes = 4 * G * R * BITS / 8;
    constexpr int kPieces = 2 * R * BITS;
    constexpr uint32_t kHalfMask = (BITS == 8) ? 0xFFFFFFFFu : ((1u << (4 * BITS)) - 1u);
    const int l = lane % G;
    const int sub = lane / G;
    const int odd = l & 1;
    if (lane < kPieces) reinterpret_cast<u4*>(stage)[lane] = piece;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
    for (int cp = 0; cp < R / 2; ++cp) {
        const int chunk_index = ((2 * cp + odd) * G + (l - odd)) >> 1;
        const uint64_t chunk = load_chunk<BITS>(stage + sub * kBucketBytes + chunk_index * BITS);
        const uint32_t lo4 = (uint32_t)chunk & kHalfMask;
        const uint32_t hi4 = (uint32_t)(chunk >> (4 * BITS)) & kHalfMask;
        const uint32_t recv = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(odd ? lo4 : hi4), 0xB1, 0xF, 0xF,
                                                                    false);
        const uint32_t q0 = odd ? recv : lo4;  // this lane's 4 codes of row 2cp
        const uint32_t q1 = odd ? hi4 : recv;  // ... of row 2cp+1
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            c[2 * cp][i] = (float)((q0 >> (i * BITS)) & ((1u << BITS) - 1u));
            c[2 * cp + 1][i] = (float)((q1 >> (i * BITS)) & ((1u << BITS) - 1u));
        }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

template <int G, int R, int BITS>
__device__ __forceinline__ void load_codes(uint8_t* stage, const u4* tile_in, int lane, int active_buckets,
                                           float (&c)[R][4]) {
    unstage_codes<G, R, BITS>(stage, fetch_code_tile<G, R, BITS>(tile_in, lane, active_buckets), lane, c);
}

// The same two phases for a code width known only at run time (the peers' gradient codes of the
// receive-side modes; wave-uniform `gb` in 1..8), so that those modes are not instantiated per
// width. The tile (32*R*gb bytes) is staged as it is; lane l then cuts the 4*gb bits of its four
// consecutive elements of a row out of the two staged words that hold them (the stage has a
// spare word past the tile for the last lane's second read).
template <int G, int R>
__device__ __forceinline__ u4 fetch_code_tile_rt(const u4* tile_in, int lane, int active_buckets, int gb) {
    const int pieces = 2 * R * gb;            // 16-byte pieces in the tile
    const int bucket_bytes = G * R * gb / 2;  // 4*G*R codes of gb bits
    u4 piece = {0u, 0u, 0u, 0u};
    if (lane < pieces && lane * 16 < active_buckets * bucket_bytes) piece = __builtin_nontemporal_load(tile_in + lane);
    return piece;
}

template <int G, int R>
__device__ __forceinline__ void unstage_codes_rt(uint8_t* stage, u4 piece, int lane, int gb, float (&c)[R][4]) {
    const int l = lane % G;
    const int sub = lane / G;
    if (lane < 2 * R * gb) reinterpret_cast<u4*>(stage)[lane] = piece;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const uint32_t* words = reinterpret_cast<const uint32_t*>(stage);
    const uint32_t mask = (1u << gb) - 1u;
    const uint32_t bit0 = (uint32_t)((sub * G * R + l) * 4 * gb);  // this lane's first code of row 0
    const uint32_t row_bits = (uint32_t)(G * 4 * gb);             // wave-uniform
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const uint32_t bit = bit0 + (uint32_t)r * row_bits;
        const uint32_t w = bit >> 5;
        // the 32 bits that start at `bit` (the 4*gb <= 32 bits of interest are its low part); a 64-bit
        // shift measured 4 % faster here than v_alignbit_b32
        const uint64_t two = (uint64_t)words[w] | ((uint64_t)words[w + 1] << 32);
        const uint32_t q = (uint32_t)(two >> (bit & 31u));
#pragma unroll
        for (int i = 0; i < 4; ++i) c[r][i] = (float)((q >> (i * gb)) & mask);
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// Combine per-wave (lo, hi) across the W waves of a workgroup that share a bucket. `slot` is a
// [2][W] LDS array that no other reduction uses; callers alternate two slots between loop
// iterations so that a fast wave's next write cannot overtake a slow wave's read.
template <int W>
__device__ __forceinline__ void block_combine_minmax(float& lo, float& hi, float* slot, uint32_t wave) {
    if (W > 1) {
        if ((threadIdx.x & 63) == 0) {
            slot[wave] = lo;
            slot[W + wave] = hi;
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < W; ++i) {
            lo = fminf(lo, slot[i]);
            hi = fmaxf(hi, slot[W + i]);
        }
    }
}

// ghat-sum of the receive-side modes for the wave's tile: sum = ((d_0 + d_1) + d_2) + ..., d_k the
// decoded slice of peer k. The tiles of up to kPeerGroup peers are in flight before the first is
// unpacked. The peers' code width p.gbits is a run-time value here (compile-time unpacking of the
// common widths next to the generic one, chosen by a wave-uniform branch, measured 15 % slower
// than the generic path alone: three inlined copies of the loop cost registers).
template <int G, int R>
__device__ __forceinline__ void sum_peer_slices(const Params& p, uint8_t* stage, uint64_t tile_slot0,
                                                uint64_t bucket, int lane, int active_buckets,
                                                float (&sum)[R][4]) {
    constexpr int kPeerGroup = 4;
    const int gb = p.gbits;
    const u4* gtile = reinterpret_cast<const u4*>(reinterpret_cast<const uint8_t*>(p.peer_codes) +
                                                  (tile_slot0 >> 3) * (uint64_t)gb);
    const uint64_t stride_u4 = p.peer_codes_stride_words >> 2;
    for (int peer0 = 0; peer0 < p.npeers; peer0 += kPeerGroup) {
        u4 piece[kPeerGroup];
        float gbase[kPeerGroup], gscale[kPeerGroup];
#pragma unroll
        for (int k = 0; k < kPeerGroup; ++k) {
            // past the last peer: re-read the last one (in bounds), its values are not used
            const uint64_t peer = peer0 + k < p.npeers ? peer0 + k : p.npeers - 1;
            piece[k] = fetch_code_tile_rt<G, R>(gtile + peer * stride_u4, lane, active_buckets, gb);
            const float* pm = p.peer_meta + peer * p.peer_meta_stride_floats;
            gbase[k] = pm[2 * bucket];
            gscale[k] = pm[2 * bucket + 1];
        }
#pragma unroll
        for (int k = 0; k < kPeerGroup; ++k) {
            if (peer0 + k < p.npeers) {  // wave-uniform
                float c[R][4];
                unstage_codes_rt<G, R>(stage, piece[k], lane, gb, c);
#pragma unroll
                for (int r = 0; r < R; ++r)
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const float d = fmaf(c[r][i], gscale[k], gbase[k]);
                        sum[r][i] = (peer0 + k == 0) ? d : sum[r][i] + d;
                    }
            }
        }
    }
}

// Every mode over the buckets first_bucket .. +num_buckets-1 (the last bucket of a tensor may
// be short). BITS is the width of the codes that are stored (0: a step without code output, or
// MODE_SUM). W = waves per bucket (W > 1: the workgroup has exactly W waves and owns one bucket
// per iteration). delta > 0 selects the explicit grid, p.flags the quantizer variants (both
// wave-uniform branches).
template <int MODE, int G, int R, int BITS, int W>
__global__ void __launch_bounds__(256) wave_kernel(const Params p, const Segment* __restrict__ segs) {
    static_assert(R % 2 == 0 && G >= 2 && G <= 64, "shape");
    static_assert(W == 1 || (G == 64 && W <= 4), "shared buckets use whole waves");
    constexpr int T = 4 * G * R;  // elements of a bucket one wave holds
    constexpr int B = T * W;
    constexpr int BPW = 64 / G;
    constexpr int SB = BITS ? BITS : 8;  // only used when BITS != 0
    const int lane = threadIdx.x & 63;
    const int sub = lane / G;
    const int l = lane % G;
    const uint32_t wave_in_block = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint64_t waves_per_block = blockDim.x >> 6;
    // W == 1: a wave strides over groups of BPW buckets; W > 1: a workgroup strides over buckets
    const uint64_t unit0 = W == 1 ? (uint64_t)blockIdx.x * waves_per_block + wave_in_block : blockIdx.x;
    const uint64_t unit_stride = W == 1 ? (uint64_t)gridDim.x * waves_per_block : gridDim.x;
    const uint64_t nunits = (p.num_buckets + BPW - 1) / BPW;

    // LDS staging tile of the packed codes (stored, or read from the peers): 32*R*bits bytes per
    // wave, up to 4 waves per block (the peers' tiles are at most 8 bits wide and take one spare
    // 16-byte piece, see unstage_codes_rt)
    constexpr bool kStaged = BITS != 0 || mode_reads_peers(MODE);
    constexpr int kTileBytes = mode_reads_peers(MODE) ? 32 * R * 8 + 16 : 32 * R * SB;
    __shared__ u4 stage_all[kStaged ? 4 * kTileBytes / 16 : 1];
    uint8_t* stage = reinterpret_cast<uint8_t*>(stage_all) + (kStaged ? wave_in_block * kTileBytes : 0);
    __shared__ float red_all[W > 1 ? 2 * 2 * 2 * W : 1];  // [parity][g or w][lo/hi][wave]
    uint32_t parity = 0;
    // MODE_LEVELS: the level table in LDS. One table for the whole call is loaded once per
    // workgroup; with one table per tensor every wave keeps the table of the tensor it works on
    // in a slot of its own and reloads it when its buckets move on to another tensor.
    __shared__ float level_tables[mode_is_levels(MODE) ? 4 * (1 << SB) : 1];
    const bool levels_per_tensor = mode_is_levels(MODE) && p.levels_per_tensor != 0 && segs != nullptr;
    const float* level_table = level_tables + (levels_per_tensor ? wave_in_block * (1u << SB) : 0u);
    uint32_t loaded_tensor = ~0u;  // wave-uniform: whose table the wave's slot holds
    if constexpr (mode_is_levels(MODE)) {
        if (!levels_per_tensor) {
            for (int k = threadIdx.x; k < (1 << SB); k += blockDim.x) level_tables[k] = p.levels[k];
            __syncthreads();
        }
    }

    const float Lg = (float)((1 << p.gbits) - 1);
    const float Lw = (float)((1 << p.wbits) - 1);
    const Divider div = {p.delta, p.inv_delta, p.delta_pow2 != 0};
    const bool lattice = p.delta > 0.0f;
    const bool symmetric = (p.flags & FLAG_SYMMETRIC) != 0;
    const bool grad_shift = (p.flags & FLAG_GRAD_SHIFT) != 0;
    constexpr bool kWritesX = MODE == MODE_FUSED || MODE == MODE_ADAMW || mode_is_recv(MODE);
    const bool keep_master = kWritesX && (p.flags & FLAG_KEEP_MASTER) != 0;
    const PhiloxKey key = launch_key(p);
    const Shifts shifts = draw_shifts(p, key, MODE != MODE_GRAD && !mode_is_levels(MODE) && MODE != MODE_SUM);
    const float xi = shifts.xi;
    uint32_t saturated = 0;

    for (uint64_t q = unit0; q < nunits; q += unit_stride, parity ^= 1u) {
        const uint64_t rel = q * BPW + sub;          // bucket within this launch
        const bool active = rel < p.num_buckets;
        const uint64_t left = p.num_buckets - q * BPW;
        const int active_buckets = left < (uint64_t)BPW ? (int)left : BPW;
        const uint64_t bucket0 = p.first_bucket + q * BPW;  // wave-uniform
        const uint64_t bucket = active ? p.first_bucket + rel : bucket0;
        const BucketRef ref = locate_bucket(p, segs, bucket0, bucket, B);
        // this wave's tile of the bucket: all of it, or the wave's 1/W
        const uint32_t part0 = W > 1 ? wave_in_block * (uint32_t)T : 0u;
        const uint64_t e0 = ref.e0 + part0;
        const int m = ref.m > part0 ? (int)(ref.m - part0 < (uint32_t)T ? ref.m - part0 : (uint32_t)T) : 0;
        const bool partial = __builtin_amdgcn_ballot_w64(m < T) != 0;
        // Philox block of the tile's first element; the tile's place in the code buffer (the
        // code stream is indexed by bucket number, every bucket padded to B slots)
        const uint64_t block_e0 = p.block0 + (e0 >> 3);
        const uint64_t tile_slot0 = (W == 1 ? (p.first_bucket + q * BPW) * (uint64_t)B
                                            : bucket * (uint64_t)B + part0);
        u4* tile_out = reinterpret_cast<u4*>(reinterpret_cast<uint8_t*>(p.codes) + (tile_slot0 >> 3) * SB);
        float* red_g = red_all + (W > 1 ? parity * 4 * W : 0);
        float* red_w = red_g + (W > 1 ? 2 * W : 0);
        const bool writes_meta = active && l == 0 && (W == 1 || wave_in_block == 0);

        float w[R][4];  // the values that get weight-quantized (x, or y = x - lr*ghat)
        float base = 0.0f, scale = 0.0f;

        if (MODE == MODE_GRAD || MODE == MODE_FUSED || MODE == MODE_FUSED_CODES || MODE == MODE_ADAMW) {
            float gv[R][4];
            uint32_t gcode[R][4];  // MODE_GRAD only
            float mom[R][4], var[R][4];  // MODE_ADAMW only
            if ((MODE == MODE_GRAD || MODE == MODE_FUSED) && p.g_half == 1)
                load_rows_half<G, R, true>(reinterpret_cast<const uint16_t*>(p.g) + e0, l, m, partial, gv);
            else if ((MODE == MODE_GRAD || MODE == MODE_FUSED) && p.g_half == 2)
                load_rows_half<G, R, false>(reinterpret_cast<const uint16_t*>(p.g) + e0, l, m, partial, gv);
            else
                load_rows<G, R>(p.g + e0, l, m, partial, gv);
            if (MODE == MODE_FUSED || MODE == MODE_ADAMW) load_rows<G, R>(p.x + e0, l, m, partial, w);
            if constexpr (MODE == MODE_ADAMW) {
                load_rows<G, R>(p.mom + e0, l, m, partial, mom);
                load_rows<G, R>(p.var + e0, l, m, partial, var);
            }
            if constexpr (MODE == MODE_FUSED_CODES) {
                // x = decode(codes, meta) in registers
                load_codes<G, R, SB>(stage, tile_out, lane, active_buckets, w);
                const float xbase = p.meta[2 * bucket];
                const float xscale = p.meta[2 * bucket + 1];
#pragma unroll
                for (int r = 0; r < R; ++r)
#pragma unroll
                    for (int i = 0; i < 4; ++i) w[r][i] = fmaf(w[r][i], xscale, xbase);
            }
            float lo, hi;
            rows_minmax<G, R>(gv, l, m, partial, lo, hi);
            block_combine_minmax<W>(lo, hi, red_g, wave_in_block);
            const MinMaxGrid grid = make_minmax_grid(lo, hi, Lg, symmetric);
            // base of the decoded gradient: lo, or lo + xi_g * scale for the shared-shift variant
            const float gbase = grad_shift ? fmaf(shifts.xi_g, grid.scale, grid.lo) : grid.lo;
            if (grad_shift) {
                // random-shift quantizer on the gradient: nothing is drawn per element
#pragma unroll
                for (int r = 0; r < R; ++r)
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const float code = weight_code_minmax(gv[r][i], grid, Lg, shifts.xi_g);
                        if constexpr (MODE == MODE_GRAD) {
                            gcode[r][i] = (uint32_t)code;
                        } else {
                            const float ghat = fmaf(code, grid.scale, gbase);
                            w[r][i] = step_value<MODE>(p, w[r][i], ghat, mom[r][i], var[r][i]);
                        }
                    }
            } else {
#pragma unroll
                for (int cp = 0; cp < R / 2; ++cp) {
                    float h[8];
                    grad_uniforms_rows<G>(block_e0, cp, l, key.k0, key.k1, h);
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        const int r = 2 * cp + (i >> 2);
                        if constexpr (MODE == MODE_GRAD) {
                            gcode[r][i & 3] = grad_code_int(gv[r][i & 3], grid, Lg, h[i]);
                        } else {
                            const float code = grad_code(gv[r][i & 3], grid, Lg, h[i]);
                            const float ghat = fmaf(code, grid.scale, grid.lo);
                            w[r][i & 3] = step_value<MODE>(p, w[r][i & 3], ghat, mom[r][i & 3], var[r][i & 3]);
                        }
                    }
                }
            }
            if constexpr (MODE == MODE_ADAMW) {
                if (active) {
                    store_rows<G, R>(p.mom + e0, l, m, partial, mom);
                    store_rows<G, R>(p.var + e0, l, m, partial, var);
                }
            }
            if constexpr (MODE == MODE_GRAD) {
                if (partial) zero_slots_past_end<G, R>(gcode, l, m);
                store_codes<G, R, SB>(stage, tile_out, lane, active_buckets, gcode);
                if (writes_meta) {
                    p.meta[2 * bucket] = gbase;
                    p.meta[2 * bucket + 1] = grid.scale;
                }
                continue;
            }
        } else if constexpr (MODE == MODE_SUM) {
            // out (passed in p.x) = alpha * (((d_0 + d_1) + d_2) + ...), d_k = decoded slice of peer k
            sum_peer_slices<G, R>(p, stage, tile_slot0, bucket, lane, active_buckets, w);
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int i = 0; i < 4; ++i) w[r][i] = p.alpha * w[r][i];
            if (active) store_rows<G, R>(p.x + e0, l, m, partial, w);
            continue;
        } else if constexpr (mode_is_recv(MODE)) {
            // ghat = alpha * (((d_0 + d_1) + d_2) + ...), d_k = decoded slice of peer k
            load_rows<G, R>(p.x + e0, l, m, partial, w);
            float mom[R][4], var[R][4];  // MODE_RECV_ADAMW only
            if constexpr (MODE == MODE_RECV_ADAMW) {
                load_rows<G, R>(p.mom + e0, l, m, partial, mom);
                load_rows<G, R>(p.var + e0, l, m, partial, var);
            }
            float sum[R][4];
            sum_peer_slices<G, R>(p, stage, tile_slot0, bucket, lane, active_buckets, sum);
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    w[r][i] = step_value<MODE>(p, w[r][i], p.alpha * sum[r][i], mom[r][i], var[r][i]);
            if constexpr (MODE == MODE_RECV_ADAMW) {
                if (active) {
                    store_rows<G, R>(p.mom + e0, l, m, partial, mom);
                    store_rows<G, R>(p.var + e0, l, m, partial, var);
                }
            }
        } else {
            load_rows<G, R>(p.xin + e0, l, m, partial, w);
        }

        // the full-precision partition keeps the updated value itself (stored before w turns into codes)
        if (kWritesX && keep_master && active) store_rows<G, R>(p.x + e0, l, m, partial, w);

        // weight quantization of w
        if constexpr (mode_is_levels(MODE)) {
            float lo, hi;
            rows_minmax<G, R>(w, l, m, partial, lo, hi);
            block_combine_minmax<W>(lo, hi, red_w, wave_in_block);
            const MinMaxGrid grid = make_minmax_grid(lo, hi, 1.0f, false);  // scale = hi - lo, inv = 1/(hi - lo)
            base = grid.lo;
            scale = grid.scale;
            // One pass per distinct tensor among the wave's buckets (one pass, unless the buckets
            // straddle tensors): every lane computes, the lanes of the pass's tensor replace their
            // values by the codes (a lane belongs to exactly one pass; what it computes in the others,
            // from values or from codes, is dropped). All lanes stay converged (the uniforms are
            // exchanged between lanes).
            uint64_t pending = ~0ull;
            do {
                bool mine = true;
                if (levels_per_tensor) {
                    const uint32_t cur = (uint32_t)__builtin_amdgcn_readlane((int)ref.tensor, __builtin_ctzll(pending));
                    mine = ref.tensor == cur;
                    if (cur != loaded_tensor) {
                        float* slot = level_tables + wave_in_block * (1u << SB);
                        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");  // earlier reads of the slot are done
                        __builtin_amdgcn_wave_barrier();
                        for (int k = lane; k < (1 << SB); k += 64) slot[k] = p.levels[(uint64_t)cur * (1u << SB) + k];
                        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                        __builtin_amdgcn_wave_barrier();
                        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                        loaded_tensor = cur;
                    }
                }
                if constexpr (MODE == MODE_LEVELS_COIN) {
#pragma unroll
                    for (int cp = 0; cp < R / 2; ++cp) {
                        float h[8];
                        grad_uniforms_rows<G>(block_e0, cp, l, key.k0, key.k1, h);
#pragma unroll
                        for (int i = 0; i < 8; ++i) {
                            const int r = 2 * cp + (i >> 2);
                            const float z = (w[r][i & 3] - grid.lo) * grid.inv;
                            const float c = (float)stochastic_level<SB>(z, h[i], level_table);
                            w[r][i & 3] = mine ? c : w[r][i & 3];
                        }
                    }
                } else {
#pragma unroll
                    for (int r = 0; r < R; ++r)
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const float z = (w[r][i] - grid.lo) * grid.inv;
                            const float c = (float)nearest_level<SB>(z, level_table);
                            w[r][i] = mine ? c : w[r][i];
                        }
                }
                pending &= ~__builtin_amdgcn_ballot_w64(mine);
            } while (pending != 0);
        } else if (lattice) {
            float lo, unused_hi;
            rows_minmax<G, R>(w, l, m, partial, lo, unused_hi);
            block_combine_minmax<W>(lo, unused_hi, red_w, wave_in_block);
            lo = lo + 0.0f;
            const float k0 = rintf(div_delta(lo, div) - xi);
            base = (k0 + xi) * p.delta;
            scale = p.delta;
            uint32_t sat_here = 0;
            if (!partial) {
#pragma unroll
                for (int r = 0; r < R; ++r)
#pragma unroll
                    for (int i = 0; i < 4; ++i) w[r][i] = weight_code_lattice(w[r][i], div, xi, k0, Lw, sat_here);
            } else {  // short bucket: slots past the end neither count as saturated nor carry a code
#pragma unroll
                for (int r = 0; r < R; ++r)
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        uint32_t sat_one = 0;
                        const float c = weight_code_lattice(w[r][i], div, xi, k0, Lw, sat_one);
                        const bool valid = (r * G + l) * 4 + i < m;
                        w[r][i] = valid ? c : 0.0f;
                        sat_here += valid ? sat_one : 0u;
                    }
            }
            if (active) saturated += sat_here;
        } else {
            float lo, hi;
            rows_minmax<G, R>(w, l, m, partial, lo, hi);
            block_combine_minmax<W>(lo, hi, red_w, wave_in_block);
            const MinMaxGrid grid = make_minmax_grid(lo, hi, Lw, symmetric);
            base = fmaf(xi, grid.scale, grid.lo);
            scale = grid.scale;
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int i = 0; i < 4; ++i) w[r][i] = weight_code_minmax(w[r][i], grid, Lw, xi);
        }
        if (partial && BITS != 0) zero_slots_past_end<G, R>(w, l, m);

        if (BITS != 0) {
            store_codes<G, R, SB>(stage, tile_out, lane, active_buckets, w);
            if (writes_meta) {
                p.meta[2 * bucket] = base;
                p.meta[2 * bucket + 1] = scale;
            }
        }
        if (active && !keep_master) {
            if (kWritesX) {
#pragma unroll
                for (int r = 0; r < R; ++r)
#pragma unroll
                    for (int i = 0; i < 4; ++i) w[r][i] = fmaf(w[r][i], scale, base);
                store_rows<G, R>(p.x + e0, l, m, partial, w);
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

        // MODE_FUSED_CODES: the old iterate is decoded from the bucket's codes and meta
        const int wpb_in = B * p.wbits / 32;
        const uint32_t* old_words = (MODE == MODE_FUSED_CODES) ? p.codes + bucket * (uint64_t)wpb_in : nullptr;
        const float old_base = (MODE == MODE_FUSED_CODES) ? p.meta[2 * bucket] : 0.0f;
        const float old_scale = (MODE == MODE_FUSED_CODES) ? p.meta[2 * bucket + 1] : 0.0f;

        if (MODE == MODE_GRAD || MODE == MODE_FUSED || MODE == MODE_FUSED_CODES || MODE == MODE_ADAMW) {
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
                    const float h = (float)((j & 1u) ? (word >> 16) : (word & 0xFFFFu));
                    c = grad_code(val[i], grid, Lg, h);
                }
                if (MODE == MODE_GRAD) {
                    code[i] = (uint8_t)(uint32_t)c;
                } else {
                    const float ghat = fmaf(c, grid.scale, gbase);
                    float xold;
                    if (MODE == MODE_FUSED_CODES) {
                        const int bit = i * p.wbits;
                        uint64_t two = old_words[bit >> 5];
                        if ((bit >> 5) + 1 < wpb_in) two |= (uint64_t)old_words[(bit >> 5) + 1] << 32;
                        const uint32_t cw = (uint32_t)(two >> (bit & 31)) & ((1u << p.wbits) - 1u);
                        xold = fmaf((float)cw, old_scale, old_base);
                    } else {
                        xold = p.x[e0 + i];
                    }
                    float mom = 0.0f, var = 0.0f;
                    if (MODE == MODE_ADAMW) {
                        mom = p.mom[e0 + i];
                        var = p.var[e0 + i];
                    }
                    val[i] = step_value<MODE>(p, xold, ghat, mom, var);
                    if (MODE == MODE_ADAMW) {
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
                                const float prob = (z - q0) / (levels[lower + 1] - q0);
                                c = lower + (h < prob * 65536.0f ? 1 : 0);
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
// Decoding: elementwise. A lane decodes E consecutive elements per row (E = 4 for fp32, 8 for
// bf16 output: one 16-byte store), a wave row is 64*E consecutive elements (one contiguous KiB
// of output), a wave handles U rows. Buckets are padded to full size in the code stream, so
// the codes of element e start at bit e*BITS of the whole buffer.
// ---------------------------------------------------------------------------------------
struct DequantParams {
    const uint32_t* codes;
    const float* meta;
    const float* levels;  // learned-level table (2^bits floats) or nullptr
    void* out;
    uint64_t n;
    uint64_t nwords;  // 32-bit words in the code buffer
    uint64_t ntiles;  // wave tiles of U*64*E elements
    uint32_t bucket32;      // bucket / 32
    int bucket32_shift;     // log2(bucket / 32) if that is a power of two, else -1 (division)
    // Gathered buffers (dequant_kernel only, one blockIdx.y per peer slot): peer p's codes start
    // p * codes_stride_words after `codes`, its meta p * meta_stride_floats after `meta`, its
    // elements p * n after `out`; n / nwords / ntiles describe every slot but the last, the
    // *_last fields the last one (for a plain call: the only one).
    uint64_t codes_stride_words, meta_stride_floats;
    uint64_t n_last, nwords_last, ntiles_last;
};

#ifndef QSDP_DEQ_ROWS
#define QSDP_DEQ_ROWS 2
#endif
constexpr int kDequantRows = QSDP_DEQ_ROWS;

// The E*BITS bits (at most 64) that start at bit `bit` of the code buffer.
template <int NBITS>
__device__ __forceinline__ uint64_t load_bits(const uint32_t* codes, uint64_t bit, uint64_t last_word) {
    const uint64_t word = bit >> 5;
    const uint32_t sh = (uint32_t)bit & 31u;
    if (NBITS == 64) {  // 8-byte aligned
        const u2 w = __builtin_nontemporal_load(reinterpret_cast<const u2*>(codes + word));
        return (uint64_t)w[0] | ((uint64_t)w[1] << 32);
    } else if (NBITS == 32) {
        return __builtin_nontemporal_load(codes + word);
    } else if (32 % NBITS == 0) {  // 16, 8 or 4 bits inside one word
        return (uint64_t)(codes[word] >> sh);
    } else {  // straddles words; the start bit is a multiple of gcd(NBITS, 32)
        constexpr int kStep = (NBITS % 16 == 0) ? 16 : (NBITS % 8 == 0) ? 8 : 4;
        const uint64_t w1i = word + 1 <= last_word ? word + 1 : last_word;
        const uint64_t lo64 = (uint64_t)codes[word] | ((uint64_t)codes[w1i] << 32);
        uint64_t v = lo64 >> sh;
        if (32 - kStep + NBITS > 64) {  // a third word is needed (56 bits from bit 24)
            const uint64_t w2i = word + 2 <= last_word ? word + 2 : last_word;
            const uint64_t w2 = codes[w2i];
            if (sh != 0) v |= w2 << (64 - sh);
        }
        return v;
    }
}

// How a decoder lane finds the bucket of element e (32-bit arithmetic; the host checks
// n < 2^37): by division, by shift (bucket a power of two), or once per wave tile when the
// bucket size is a multiple of the tile (the index is then wave-uniform: one meta-data fetch per
// tile, every lane reading the same 8 bytes, issued together with the code loads).
enum BucketIndexing { BK_DIVIDE = 0, BK_SHIFT = 1, BK_TILE_UNIFORM = 2 };

template <int BK>
__device__ __forceinline__ uint64_t bucket_of(uint64_t e, const DequantParams& p) {
    const uint32_t e32 = (uint32_t)(e >> 5);
    if (BK == BK_SHIFT) return e32 >> p.bucket32_shift;
    if (BK == BK_TILE_UNIFORM) return __builtin_amdgcn_readfirstlane(e32 / p.bucket32);
    return e32 / p.bucket32;
}

// `lut` = the level table in LDS (learned levels: the code indexes it), or nullptr (uniform
// levels: the code is the level).
template <int BITS, bool BF16, bool LUT>
__device__ __forceinline__ void decode_store(const DequantParams& p, uint64_t e, uint64_t bits, float base,
                                             float scale, bool whole, const float* lut, uint64_t limit) {
    constexpr int E = BF16 ? 8 : 4;
    float o[E];
#pragma unroll
    for (int i = 0; i < E; ++i) {
        const uint32_t c = (uint32_t)(bits >> (i * BITS)) & ((1u << BITS) - 1u);
        o[i] = fmaf(LUT ? lut[c] : (float)c, scale, base);
    }
    if (whole) {
        if (BF16) {
            u4 w;
#pragma unroll
            for (int i = 0; i < 4; ++i) w[i] = bf16_bits(o[2 * i]) | (bf16_bits(o[2 * i + 1]) << 16);
            __builtin_nontemporal_store(w, reinterpret_cast<u4*>(static_cast<uint16_t*>(p.out) + e));
        } else {
            const f4 a = {o[0], o[1], o[2], o[3]};
            __builtin_nontemporal_store(a, reinterpret_cast<f4*>(static_cast<float*>(p.out) + e));
        }
    } else {
        for (int i = 0; i < E; ++i) {
            if (e + i < limit) {
                if (BF16) static_cast<uint16_t*>(p.out)[e + i] = (uint16_t)bf16_bits(o[i]);
                else static_cast<float*>(p.out)[e + i] = o[i];
            }
        }
    }
}

template <int BITS, bool BF16, int BK, bool LUT>
__global__ void __launch_bounds__(256) dequant_kernel(const DequantParams p) {
    constexpr int E = BF16 ? 8 : 4;
    constexpr int U = kDequantRows;
    constexpr uint64_t T = (uint64_t)U * 64 * E;
    __shared__ float lut[LUT ? (1 << BITS) : 1];
    if (LUT) {
        for (int k = threadIdx.x; k < (1 << BITS); k += blockDim.x) lut[k] = p.levels[k];
        __syncthreads();
    }
    const int lane = threadIdx.x & 63;
    const uint32_t wave_in_block = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint64_t waves_per_block = blockDim.x >> 6;
    const uint64_t nwaves = (uint64_t)gridDim.x * waves_per_block;
    // the slot this workgroup decodes (the whole buffer for a plain call)
    const uint64_t peer = blockIdx.y;
    const bool last_peer = peer + 1 == gridDim.y;
    const uint32_t* codes = p.codes + peer * p.codes_stride_words;
    const float* meta = p.meta + peer * p.meta_stride_floats;
    const uint64_t out0 = peer * p.n;
    const uint64_t n = last_peer ? p.n_last : p.n;
    const uint64_t ntiles = last_peer ? p.ntiles_last : p.ntiles;
    const uint64_t last_word = (last_peer ? p.nwords_last : p.nwords) - 1;
    for (uint64_t tile = (uint64_t)blockIdx.x * waves_per_block + wave_in_block; tile < ntiles; tile += nwaves) {
        const uint64_t e0 = tile * T + (uint64_t)(lane * E);
        if ((tile + 1) * T <= n) {
            // whole tile in range (wave-uniform): all loads first, no per-lane control flow
            uint64_t bits[U];
            float base[U], scale[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const uint64_t e = e0 + (uint64_t)(u * 64 * E);
                bits[u] = load_bits<E * BITS>(codes, e * BITS, last_word);
                if (BK == BK_TILE_UNIFORM && u > 0) {  // the whole tile lies in one bucket
                    base[u] = base[0];
                    scale[u] = scale[0];
                } else {
                    const uint64_t bucket = bucket_of<BK>(e, p);
                    base[u] = meta[2 * bucket];
                    scale[u] = meta[2 * bucket + 1];
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u)
                decode_store<BITS, BF16, LUT>(p, out0 + e0 + (uint64_t)(u * 64 * E), bits[u], base[u], scale[u], true,
                                              lut, out0 + n);
        } else {
            // last, partial tile
            for (int u = 0; u < U; ++u) {
                const uint64_t e = e0 + (uint64_t)(u * 64 * E);
                if (e < n) {
                    const uint64_t bits = load_bits<E * BITS>(codes, e * BITS, last_word);
                    const uint64_t bucket = bucket_of<BK>(e, p);
                    decode_store<BITS, BF16, LUT>(p, out0 + e, bits, meta[2 * bucket], meta[2 * bucket + 1],
                                                  e + E <= n, lut, out0 + n);
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------------------
// Decoder for a multi-tensor code buffer: slot s of the padded code stream (bucket s / B of the
// whole buffer) belongs to the tensor whose bucket range holds that bucket and lands at element
// seg.offset + (s - seg.first_bucket * B) of the flat output, if the tensor has that element.
// Same tiling as dequant_kernel over SLOTS (p.n = number of slots). The tensor of a tile's
// first slot is found by a wave-uniform search (scalar loads, see find_segment). A tile that
// lies inside that tensor's elements (the common case) is decoded without per-lane control
// flow; a tile that reaches a tensor's padding or the next tensor goes lane by lane, each lane
// walking on from the tile's tensor to its own. LUT: learned levels, one table of 2^BITS floats
// per tensor at d.levels (tensor t's at d.levels + t * 2^BITS); a wave keeps the table of its
// tile's tensor in an LDS slot of its own and reads the tables through global memory on the
// lane-by-lane path.
// ---------------------------------------------------------------------------------------
struct DequantSegParams {
    DequantParams d;  // d.n: slots (total buckets * bucket); d.out: the flat output
    const Segment* segs;
    uint32_t nseg;
};

template <int BITS, bool BF16, int BK, bool LUT>
__global__ void __launch_bounds__(256) dequant_seg_kernel(const DequantSegParams q,
                                                          const Segment* __restrict__ segs) {
    const DequantParams& p = q.d;
    constexpr int K = 1 << BITS;
    __shared__ float lut_all[LUT ? 4 * K : 1];
    uint32_t loaded_tensor = ~0u;  // wave-uniform: whose table the wave's slot holds
    constexpr int E = BF16 ? 8 : 4;
    constexpr int U = kDequantRows;
    constexpr uint64_t T = (uint64_t)U * 64 * E;
    const int lane = threadIdx.x & 63;
    const uint32_t wave_in_block = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint64_t waves_per_block = blockDim.x >> 6;
    const uint64_t nwaves = (uint64_t)gridDim.x * waves_per_block;
    const uint64_t last_word = p.nwords - 1;
    const uint64_t B = (uint64_t)p.bucket32 * 32u;
    for (uint64_t tile = (uint64_t)blockIdx.x * waves_per_block + wave_in_block; tile < p.ntiles;
         tile += nwaves) {
        const uint64_t s0 = tile * T;
        const uint64_t bucket0 = (uint32_t)(s0 >> 5) / p.bucket32;  // wave-uniform
        uint32_t tensor0;
        const Segment seg0 = find_segment(segs, q.nseg, bucket0, bucket0, &tensor0);
        const uint64_t e0 = seg0.offset + (s0 - seg0.first_bucket * B);  // element of slot s0
        const uint64_t end0 = seg0.offset + seg0.n;
        if (e0 + T <= end0) {
            float* lut = lut_all + (LUT ? wave_in_block * K : 0);
            if (LUT && tensor0 != loaded_tensor) {
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");  // earlier reads of the slot are done
                __builtin_amdgcn_wave_barrier();
                for (int k = lane; k < K; k += 64) lut[k] = p.levels[(uint64_t)tensor0 * K + k];
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                loaded_tensor = tensor0;
            }
            uint64_t bits[U];
            float base[U], scale[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const uint64_t s = s0 + (uint64_t)(u * 64 * E + lane * E);
                bits[u] = load_bits<E * BITS>(p.codes, s * BITS, last_word);
                const uint64_t bucket = BK == BK_TILE_UNIFORM ? bucket0 : bucket_of<BK>(s, p);
                base[u] = p.meta[2 * bucket];
                scale[u] = p.meta[2 * bucket + 1];
            }
#pragma unroll
            for (int u = 0; u < U; ++u)
                decode_store<BITS, BF16, LUT>(p, e0 + (uint64_t)(u * 64 * E + lane * E), bits[u], base[u], scale[u],
                                              true, lut, end0);
        } else {
            for (int u = 0; u < U; ++u) {
                const uint64_t s = s0 + (uint64_t)(u * 64 * E + lane * E);
                if (s < p.n) {
                    const uint64_t bucket = bucket_of<BK>(s, p);
                    uint32_t tensor;
                    const Segment seg = find_segment(segs, q.nseg, bucket0, bucket, &tensor);
                    const uint64_t e = seg.offset + (s - seg.first_bucket * B);
                    const uint64_t end = seg.offset + seg.n;
                    if (e < end) {
                        const uint64_t bits = load_bits<E * BITS>(p.codes, s * BITS, last_word);
                        decode_store<BITS, BF16, LUT>(p, e, bits, p.meta[2 * bucket], p.meta[2 * bucket + 1],
                                                      e + E <= end, LUT ? p.levels + (uint64_t)tensor * K : nullptr, end);
                    }
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------------------
// Decode-and-sum of P peers' slices: out = alpha * (((d_0 + d_1) + d_2) + ...), d_p the decoded
// slice of peer p. Same tiling as the decoder with fp32 output; peers are read in order.
// ---------------------------------------------------------------------------------------
struct DequantAddParams {
    DequantParams d;             // d.codes / d.meta: peer 0; d.out: float[n]
    uint64_t codes_stride_words;  // peer p's codes start p * stride words further
    uint64_t meta_stride_floats;
    int npeers;
    float alpha;
};

template <int BITS, int BK>
__global__ void __launch_bounds__(256) dequant_add_kernel(const DequantAddParams q) {
    constexpr int E = 4;
    constexpr int U = kDequantRows;
    constexpr uint64_t T = (uint64_t)U * 64 * E;
    const DequantParams& p = q.d;
    const int lane = threadIdx.x & 63;
    const uint32_t wave_in_block = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint64_t waves_per_block = blockDim.x >> 6;
    const uint64_t nwaves = (uint64_t)gridDim.x * waves_per_block;
    const uint64_t last_word = p.nwords - 1;
    float* out = static_cast<float*>(p.out);
    for (uint64_t tile = (uint64_t)blockIdx.x * waves_per_block + wave_in_block; tile < p.ntiles;
         tile += nwaves) {
        const uint64_t e0 = tile * T + (uint64_t)(lane * E);
        const bool whole_tile = (tile + 1) * T <= p.n;  // wave-uniform
        float sum[U][E];
        uint64_t bucket[U];
        bool in_range[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint64_t e = e0 + (uint64_t)(u * 64 * E);
            in_range[u] = whole_tile || e < p.n;
            // tile-uniform: the whole tile lies in the bucket of its first element (lane 0, row 0)
            bucket[u] = (BK == BK_TILE_UNIFORM && u > 0) ? bucket[0] : bucket_of<BK>(in_range[u] ? e : 0, p);
        }
        // peers in groups of kPeerGroup: all loads of a group are issued before the first add
        constexpr int kPeerGroup = 4;
        for (int peer0 = 0; peer0 < q.npeers; peer0 += kPeerGroup) {
            uint64_t bits[kPeerGroup][U];
            float base[kPeerGroup][U], scale[kPeerGroup][U];
#pragma unroll
            for (int k = 0; k < kPeerGroup; ++k) {
                // past the last peer: re-read the last one (in bounds), its values are not used
                const int peer = peer0 + k < q.npeers ? peer0 + k : q.npeers - 1;
                const uint32_t* codes = p.codes + (uint64_t)peer * q.codes_stride_words;
                const float* meta = p.meta + (uint64_t)peer * q.meta_stride_floats;
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const uint64_t e = in_range[u] ? e0 + (uint64_t)(u * 64 * E) : 0;
                    bits[k][u] = load_bits<E * BITS>(codes, e * BITS, last_word);
                    base[k][u] = meta[2 * bucket[u]];
                    scale[k][u] = meta[2 * bucket[u] + 1];
                }
            }
#pragma unroll
            for (int k = 0; k < kPeerGroup; ++k) {
                if (peer0 + k < q.npeers) {  // wave-uniform
#pragma unroll
                    for (int u = 0; u < U; ++u)
#pragma unroll
                        for (int i = 0; i < E; ++i) {
                            const uint32_t c = (uint32_t)(bits[k][u] >> (i * BITS)) & ((1u << BITS) - 1u);
                            const float d = fmaf((float)c, scale[k][u], base[k][u]);
                            sum[u][i] = (peer0 + k == 0) ? d : sum[u][i] + d;
                        }
                }
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint64_t e = e0 + (uint64_t)(u * 64 * E);
            if (whole_tile || e + E <= p.n) {
                const f4 a = {q.alpha * sum[u][0], q.alpha * sum[u][1], q.alpha * sum[u][2], q.alpha * sum[u][3]};
                __builtin_nontemporal_store(a, reinterpret_cast<f4*>(out + e));
            } else if (e < p.n) {
                for (int i = 0; i < E; ++i)
                    if (e + i < p.n) out[e + i] = q.alpha * sum[u][i];
            }
        }
    }
}

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
