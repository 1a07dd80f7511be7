// Wave kernels: a bucket is owned by an aligned group of G lanes of one wave (or by the W waves
// of a workgroup) and its values never leave registers. Layout and launch shape: see the
// overview in qsdp_kernels.hpp.
#pragma once

#include "qsdp_params.hpp"

// Workgroups (of 4 waves) per compute unit the compiler has to leave room for, i.e. waves per SIMD: caps the
// registers of a kernel. 1 = no constraint.
#ifndef QSDP_LEVELS_MIN_BLOCKS
#define QSDP_LEVELS_MIN_BLOCKS 4
#endif
#ifndef QSDP_ADAMW_MIN_BLOCKS
#define QSDP_ADAMW_MIN_BLOCKS 1
#endif
#ifndef QSDP_RECV_MIN_BLOCKS
#define QSDP_RECV_MIN_BLOCKS 5
#endif
#ifndef QSDP_FUSED_MIN_BLOCKS
#define QSDP_FUSED_MIN_BLOCKS 1
#endif

namespace qsdp {

// ---------------------------------------------------------------------------------------
// Wave kernels
// ---------------------------------------------------------------------------------------
// Lane l's rows of a tile of 4*G*R elements at `base`. `m` = how many of the tile's elements
// exist; `partial` (wave-uniform) selects the guarded element-wise path for a short bucket.
// Whether element i of row r of lane l, i.e. slot (r*G + l)*4 + i of the tile, lies below m. Written as a
// comparison of the lane's own offset with a per-slot bound so that the short-bucket paths need no
// per-slot index registers (those would be set up by every wave, short bucket or not).
template <int G>
__device__ __forceinline__ bool slot_exists(int l, int m, int r, int i) {
    int bound = m - (r * G * 4 + i);
    // keeps the compiler from folding this back into (r*G + l)*4 + i < m and hoisting the 4*R slot
    // indices out of the bucket loop into every wave's prologue
    asm volatile("" : "+v"(bound));
    return l * 4 < bound;
}

template <int G, int R>
__device__ __forceinline__ void load_rows(const float* base, int l, int m, bool partial, float (&v)[R][4]) {
    if (__builtin_expect(!partial, 1)) {
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
                v[r][i] = slot_exists<G>(l, m, r, i) ? base[idx] : 0.0f;
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
    if (__builtin_expect(!partial, 1)) {
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
                v[r][i] = slot_exists<G>(l, m, r, i) ? widen16<BF16>(base[idx]) : 0.0f;
            }
    }
}

template <int G, int R>
__device__ __forceinline__ void store_rows(float* base, int l, int m, bool partial, const float (&v)[R][4]) {
    if (__builtin_expect(!partial, 1)) {
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
                if (slot_exists<G>(l, m, r, i)) base[idx] = v[r][i];
            }
    }
}

// The tile rounded to a 2-byte format (bf16, or binary16 when f16), 8 bytes per lane and row.
template <int G, int R>
__device__ __forceinline__ void store_rows_half(uint16_t* base, int l, int m, bool partial, bool f16,
                                                const float (&v)[R][4]) {
    if (__builtin_expect(!partial, 1)) {
        u2* p = reinterpret_cast<u2*>(base) + l;
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const u2 a = {half_bits(v[r][0], f16) | (half_bits(v[r][1], f16) << 16),
                          half_bits(v[r][2], f16) | (half_bits(v[r][3], f16) << 16)};
            __builtin_nontemporal_store(a, p + r * G);
        }
    } else {
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int idx = (r * G + l) * 4 + i;
                if (slot_exists<G>(l, m, r, i)) base[idx] = (uint16_t)half_bits(v[r][i], f16);
            }
    }
}

// min and max over the bucket (the group's G lanes); slots at or past m do not take part
template <int G, int R>
__device__ __forceinline__ void rows_minmax(const float (&v)[R][4], int l, int m, bool partial, float& lo,
                                            float& hi) {
    if (__builtin_expect(!partial, 1)) {
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
                const bool valid = slot_exists<G>(l, m, r, i);
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
            if (!slot_exists<G>(l, m, r, i)) c[r][i] = CodeT(0);
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

// The learned-level encoders over a lane's rows: v -> codes (MODE_LEVELS: nearest level; MODE_LEVELS_COIN:
// coin flip between the enclosing levels). MASKED: only the lanes with `mine` keep their codes (a pass
// over the lanes of one tensor of a multi-tensor call).
template <int MODE, int G, int R, int BITS, bool MASKED, bool BY_CELL>
__device__ __forceinline__ void encode_levels_by(const float (&v)[R][4], uint32_t (&code)[R][4], bool mine, float lo,
                                                 float inv_cells, const float* lv, const LevelCell* cells,
                                                 const LevelNear* near, const LevelCoin* coin,
                                                 const LevelPivots& pivots, uint64_t block_e0, int l, PhiloxKey key) {
    constexpr bool by_cell = BY_CELL;
    if constexpr (MODE == MODE_LEVELS_COIN) {
#pragma unroll
        for (int cp = 0; cp < R / 2; ++cp) {
            uint32_t h[4];
            grad_uniforms_rows<G>(block_e0, cp, l, key.k0, key.k1, h);
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int r = 2 * cp + (i >> 2);
                const float z = (v[r][i & 3] - lo) * inv_cells;
                const uint32_t c = stochastic_level<BITS>(z, (float)uniform16(h, i), lv, cells, coin, pivots, by_cell);
                code[r][i & 3] = (!MASKED || mine) ? c : code[r][i & 3];
            }
        }
    } else {
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float z = (v[r][i] - lo) * inv_cells;
                const uint32_t c = nearest_level<BITS>(z, lv, cells, near, pivots, by_cell);
                code[r][i] = (!MASKED || mine) ? c : code[r][i];
            }
    }
}

// by_cell (wave-uniform) picks the counting method once for all of the lane's elements, so that each
// method is straight-line code over the rows and the LDS reads of different elements overlap.
template <int MODE, int G, int R, int BITS, bool MASKED>
__device__ __forceinline__ void encode_levels(const float (&v)[R][4], uint32_t (&code)[R][4], bool mine, float lo,
                                              float inv_cells, const float* lv, const LevelCell* cells,
                                              const LevelNear* near, const LevelCoin* coin, const LevelPivots& pivots,
                                              bool by_cell, uint64_t block_e0, int l, PhiloxKey key) {
    if (by_cell)
        encode_levels_by<MODE, G, R, BITS, MASKED, true>(v, code, mine, lo, inv_cells, lv, cells, near, coin, pivots,
                                                         block_e0, l, key);
    else
        encode_levels_by<MODE, G, R, BITS, MASKED, false>(v, code, mine, lo, inv_cells, lv, cells, near, coin, pivots,
                                                          block_e0, l, key);
}

// Every mode over the buckets first_bucket .. +num_buckets-1 (the last bucket of a tensor may
// be short). BITS is the width of the codes that are stored (0: a step without code output, or
// MODE_SUM). W = waves per bucket (W > 1: the workgroup has exactly W waves and owns one bucket
// per iteration). delta > 0 selects the explicit grid, p.flags the quantizer variants (both
// wave-uniform branches).
constexpr int mode_min_blocks(int mode) {
    return mode_is_levels(mode) ? QSDP_LEVELS_MIN_BLOCKS
           : mode == MODE_RECV_ADAMW ? QSDP_ADAMW_MIN_BLOCKS
           : mode == MODE_RECV ? QSDP_RECV_MIN_BLOCKS
           : mode == MODE_FUSED ? QSDP_FUSED_MIN_BLOCKS : 1;
}

template <int MODE, int G, int R, int BITS, int W>
__global__ void __launch_bounds__(256, mode_min_blocks(MODE)) wave_kernel(const Params p, const Segment* __restrict__ segs) {
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
    // Which units this wave (workgroup) works on: unit0, unit0 + stride, ... (the one-pass modes normally have
    // a wave per unit; the learned-level modes a resident grid, whose waves then sweep the buffer side by
    // side); a contiguous run of units where every tensor has its own level tables, which a wave should
    // have to set up as rarely as possible.
    uint64_t q_begin = unit0, q_end = nunits, q_step = unit_stride;
    if (mode_is_levels(MODE) && p.levels_per_tensor != 0 && segs != nullptr) {
        const uint64_t run = (nunits + unit_stride - 1) / unit_stride;
        q_begin = unit0 * run;
        q_end = q_begin + run < nunits ? q_begin + run : nunits;
        q_step = 1;
    }
    // The learned-level modes keep the values of the wave's next unit in flight while the current one is
    // encoded, and those of its first unit while the level tables are set up (the tables' own loads, the
    // barriers and the searches that fill them would otherwise all come before the first load of data).
    // unit_tile: where unit q's tile of the data lies.
    struct UnitTile {
        bool active;         // the lane's bucket exists
        uint64_t bucket;     // the lane's bucket (the unit's first one for a lane without a bucket)
        uint32_t tensor;     // the tensor the bucket belongs to (multi-tensor calls)
        uint32_t part0;      // first element of this wave's part of the bucket (W > 1)
        uint64_t e0;         // first element of the wave's tile
        int m;               // elements of the tile that exist
        bool partial;        // wave-uniform: some lane's tile is short
    };
    auto unit_tile = [&](uint64_t q) -> UnitTile {
        UnitTile t;
        const uint64_t rel = q * BPW + sub;  // bucket within this launch
        t.active = rel < p.num_buckets;
        const uint64_t bucket0 = p.first_bucket + q * BPW;  // wave-uniform
        t.bucket = t.active ? p.first_bucket + rel : bucket0;
        const BucketRef ref = locate_bucket(p, segs, bucket0, t.bucket, B);
        t.tensor = ref.tensor;
        // this wave's tile of the bucket: all of it, or the wave's 1/W
        t.part0 = W > 1 ? wave_in_block * (uint32_t)T : 0u;
        t.e0 = ref.e0 + t.part0;
        t.m = ref.m > t.part0 ? (int)(ref.m - t.part0 < (uint32_t)T ? ref.m - t.part0 : (uint32_t)T) : 0;
        t.partial = __builtin_amdgcn_ballot_w64(t.m < T) != 0;
        return t;
    };
    float next_w[mode_is_levels(MODE) ? R : 1][4];
    if constexpr (mode_is_levels(MODE)) {
        if (q_begin < q_end) {
            const UnitTile t = unit_tile(q_begin);
            load_rows<G, R>(p.xin + t.e0, l, t.m, t.partial, next_w);
        }
    }
    // Learned levels (see the section of that name in qsdp_device.hpp): the level table in LDS, scaled
    // to cell units, the cell table and the landing table of the mode's encoder, and the binary
    // search's first pivots in scalar registers. One table for the whole call is set up once per
    // workgroup; with one table per tensor every wave keeps the tables of the tensor it works on in
    // slots of its own and sets them up again when its buckets move on to another tensor.
    constexpr int kLevels = 1 << SB;
    constexpr int kCellSlot = kLevelCells + 1;
    __shared__ float level_tables[mode_is_levels(MODE) ? 4 * kLevels : 1];
    __shared__ LevelCell level_cells_all[mode_is_levels(MODE) ? 4 * kCellSlot : 1];
    __shared__ LevelNear level_nears[MODE == MODE_LEVELS ? 4 * kLevels : 1];
    __shared__ LevelCoin level_coins[MODE == MODE_LEVELS_COIN ? 4 * kLevels : 1];
    __shared__ int level_cells_crowded;
    const bool levels_per_tensor = mode_is_levels(MODE) && p.levels_per_tensor != 0 && segs != nullptr;
    const uint32_t level_slot = levels_per_tensor ? wave_in_block * (uint32_t)kLevels : 0u;
    float* level_table = level_tables + level_slot;
    LevelCell* level_cells = level_cells_all + (levels_per_tensor ? wave_in_block * (uint32_t)kCellSlot : 0u);
    LevelNear* level_near = level_nears + (MODE == MODE_LEVELS ? level_slot : 0u);
    LevelCoin* level_coin = level_coins + (MODE == MODE_LEVELS_COIN ? level_slot : 0u);
    LevelPivots pivots = {0.0f, 0.0f, 0.0f, 0.0f};
    bool count_by_cell = false;    // wave-uniform: no cell of the current table holds two levels
    uint32_t loaded_tensor = ~0u;  // wave-uniform: whose tables the wave's slots hold
    if constexpr (mode_is_levels(MODE)) {
        if (!levels_per_tensor) {
            if (threadIdx.x == 0) level_cells_crowded = 0;
            constexpr int kThreads = W == 1 ? 256 : 64 * W;  // the launch's workgroup size
            constexpr int kRounds = (kLevels + kThreads - 1) / kThreads;
            float lv_mine[kRounds];  // this thread's levels
#pragma unroll
            for (int i = 0; i < kRounds; ++i) {
                const int k = threadIdx.x + i * kThreads;
                lv_mine[i] = k < kLevels ? p.levels[k] : 0.0f;
            }
#pragma unroll
            for (int i = 0; i < kRounds; ++i) {
                const int k = threadIdx.x + i * kThreads;
                if (k < kLevels) level_tables[k] = lv_mine[i] * kLevelCellsF;
            }
            __syncthreads();
            bool crowded;
            if constexpr (MODE == MODE_LEVELS) {
                fill_level_near(level_tables, level_nears, kLevels, threadIdx.x, blockDim.x);
                crowded = fill_level_cells<false>(level_tables, level_cells_all, kLevels - 1, threadIdx.x, blockDim.x);
            } else {
                fill_level_coin(level_tables, level_coins, kLevels, threadIdx.x, blockDim.x);
                crowded = fill_level_cells<true>(level_tables, level_cells_all, kLevels, threadIdx.x, blockDim.x);
            }
            if (crowded) level_cells_crowded = 1;
            __syncthreads();
            count_by_cell = __builtin_amdgcn_readfirstlane(level_cells_crowded) == 0;
            pivots = load_level_pivots<SB>(level_tables);
        }
    }

    const float Lg = (float)((1 << p.gbits) - 1);
    const uint32_t top16_g = (uint32_t)((1 << p.gbits) - 1) << 16;  // L in units of 2^-16 of a cell
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

    for (uint64_t q = q_begin; q < q_end; q += q_step, parity ^= 1u) {
        const UnitTile tile = unit_tile(q);
        const bool active = tile.active;
        const uint64_t left = p.num_buckets - q * BPW;
        const int active_buckets = left < (uint64_t)BPW ? (int)left : BPW;
        const uint64_t bucket = tile.bucket;
        const uint32_t part0 = tile.part0;
        const uint64_t e0 = tile.e0;
        const int m = tile.m;
        const bool partial = tile.partial;
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
        uint32_t lcode[mode_is_levels(MODE) ? R : 1][4] = {};  // the learned-level modes' codes
        float base = 0.0f, scale = 0.0f;

        if (mode_local_gradient(MODE)) {
            float gv[R][4];
            uint32_t gcode[R][4];  // MODE_GRAD only
            float mom[R][4], var[R][4];  // AdamW modes only
            if (mode_mixed_precision(MODE) && p.g_half == 1)
                load_rows_half<G, R, true>(reinterpret_cast<const uint16_t*>(p.g) + e0, l, m, partial, gv);
            else if (mode_mixed_precision(MODE) && p.g_half == 2)
                load_rows_half<G, R, false>(reinterpret_cast<const uint16_t*>(p.g) + e0, l, m, partial, gv);
            else
                load_rows<G, R>(p.g + e0, l, m, partial, gv);
            if (MODE == MODE_FUSED || MODE == MODE_ADAMW) load_rows<G, R>(p.x + e0, l, m, partial, w);
            if constexpr (mode_local_adamw(MODE)) {
                load_rows<G, R>(p.mom + e0, l, m, partial, mom);
                load_rows<G, R>(p.var + e0, l, m, partial, var);
            }
            if constexpr (mode_codes_resident(MODE)) {
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
                    uint32_t h[4];
                    grad_uniforms_rows<G>(block_e0, cp, l, key.k0, key.k1, h);
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        const int r = 2 * cp + (i >> 2);
                        if constexpr (MODE == MODE_GRAD) {
                            gcode[r][i & 3] = grad_code_int(gv[r][i & 3], grid, top16_g, uniform16(h, i));
                        } else {
                            const float code = grad_code(gv[r][i & 3], grid, top16_g, uniform16(h, i));
                            const float ghat = fmaf(code, grid.scale, grid.lo);
                            w[r][i & 3] = step_value<MODE>(p, w[r][i & 3], ghat, mom[r][i & 3], var[r][i & 3]);
                        }
                    }
                }
            }
            if constexpr (mode_local_adamw(MODE)) {
                if (active) {
                    store_rows<G, R>(p.mom + e0, l, m, partial, mom);
                    store_rows<G, R>(p.var + e0, l, m, partial, var);
                }
            }
            if constexpr (MODE == MODE_GRAD) {
                if (__builtin_expect(partial, 0)) zero_slots_past_end<G, R>(gcode, l, m);
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
            if constexpr (mode_is_levels(MODE)) {
#pragma unroll
                for (int r = 0; r < R; ++r)
#pragma unroll
                    for (int i = 0; i < 4; ++i) w[r][i] = next_w[r][i];
                if (q + q_step < q_end) {
                    const UnitTile t = unit_tile(q + q_step);
                    load_rows<G, R>(p.xin + t.e0, l, t.m, t.partial, next_w);
                }
            } else {
                load_rows<G, R>(p.xin + e0, l, m, partial, w);
            }
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
            const float inv_cells = grid.inv * kLevelCellsF;  // normalised value in cell units: (v - lo) * inv_cells
            if (!levels_per_tensor) {
                encode_levels<MODE, G, R, SB, false>(w, lcode, true, grid.lo, inv_cells, level_table, level_cells, level_near,
                                                     level_coin, pivots, count_by_cell, block_e0, l, key);
            } else {
                // One pass per distinct tensor among the wave's buckets (one pass, unless the buckets
                // straddle tensors): every lane computes, the lanes of the pass's tensor keep the codes
                // (a lane belongs to exactly one pass). All lanes stay converged (the uniforms are
                // exchanged between lanes).
                uint64_t pending = ~0ull;
                do {
                    const uint32_t cur = (uint32_t)__builtin_amdgcn_readlane((int)tile.tensor, __builtin_ctzll(pending));
                    const bool mine = tile.tensor == cur;
                    if (cur != loaded_tensor) {
                        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");  // earlier reads of the slots are done
                        __builtin_amdgcn_wave_barrier();
                        for (int k = lane; k < kLevels; k += 64)
                            level_table[k] = p.levels[(uint64_t)cur * kLevels + k] * kLevelCellsF;
                        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                        __builtin_amdgcn_wave_barrier();
                        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                        bool crowded;
                        if constexpr (MODE == MODE_LEVELS) {
                            fill_level_near(level_table, level_near, kLevels, lane, 64);
                            crowded = fill_level_cells<false>(level_table, level_cells, kLevels - 1, lane, 64);
                        } else {
                            fill_level_coin(level_table, level_coin, kLevels, lane, 64);
                            crowded = fill_level_cells<true>(level_table, level_cells, kLevels, lane, 64);
                        }
                        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                        __builtin_amdgcn_wave_barrier();
                        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                        count_by_cell = __builtin_amdgcn_ballot_w64(crowded) == 0;
                        pivots = load_level_pivots<SB>(level_table);
                        loaded_tensor = cur;
                    }
                    encode_levels<MODE, G, R, SB, true>(w, lcode, mine, grid.lo, inv_cells, level_table, level_cells,
                                                        level_near, level_coin, pivots, count_by_cell, block_e0, l, key);
                    pending &= ~__builtin_amdgcn_ballot_w64(mine);
                } while (pending != 0);
            }
        } else if (lattice) {
            float lo, unused_hi;
            rows_minmax<G, R>(w, l, m, partial, lo, unused_hi);
            block_combine_minmax<W>(lo, unused_hi, red_w, wave_in_block);
            lo = lo + 0.0f;
            const float k0 = rintf(div_delta(lo, div) - xi);
            base = (k0 + xi) * p.delta;
            scale = p.delta;
            uint32_t sat_here = 0;
            if (__builtin_expect(!partial, 1)) {
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
                        const bool valid = slot_exists<G>(l, m, r, i);
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
            // Modes that only store 8-bit codes leave rounding and clamping to the packing instruction
            // (see pack4); the others need the code itself to decode the new weights.
            constexpr bool kPackRounds = BITS == 8 && (MODE == MODE_WEIGHT || mode_codes_resident(MODE));
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    w[r][i] = kPackRounds ? weight_position_minmax(w[r][i], grid, xi)
                                          : weight_code_minmax(w[r][i], grid, Lw, xi);
        }
        if constexpr (mode_is_levels(MODE)) {
            if (__builtin_expect(partial, 0)) zero_slots_past_end<G, R>(lcode, l, m);
            store_codes<G, R, SB>(stage, tile_out, lane, active_buckets, lcode);
        } else if (BITS != 0) {
            if (partial) zero_slots_past_end<G, R>(w, l, m);
            store_codes<G, R, SB>(stage, tile_out, lane, active_buckets, w);
        }
        if (BITS != 0) {
            if (writes_meta) {
                p.meta[2 * bucket] = base;
                p.meta[2 * bucket + 1] = scale;
            }
        }
        // the decoded new weights: into x (unless x keeps the unquantized value) and, on request, once
        // more in 16 bits (what a forward pass in reduced precision reads)
        const bool want16 = (MODE == MODE_FUSED || MODE == MODE_ADAMW) && p.x16 != nullptr;
        if (active && kWritesX && (!keep_master || want16)) {
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int i = 0; i < 4; ++i) w[r][i] = fmaf(w[r][i], scale, base);
            if (!keep_master) store_rows<G, R>(p.x + e0, l, m, partial, w);
            if (want16) store_rows_half<G, R>(static_cast<uint16_t*>(p.x16) + e0, l, m, partial, p.x16_f16 != 0, w);
        }
    }

    if (MODE != MODE_GRAD && p.n_saturated != nullptr) {
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) saturated += __shfl_down(saturated, off, 64);
        if (lane == 0 && saturated != 0) atomicAdd(p.n_saturated, (unsigned long long)saturated);
    }
}

}  // namespace qsdp
