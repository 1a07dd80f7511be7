// Decoders: packed codes + meta to fp32 / bf16 (single tensor, gathered peer slots, multi-tensor
// buffers) and the element-wise decode-and-sum of peer slices.
#pragma once

#include "qsdp_params.hpp"

namespace qsdp {

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
    uint32_t out_f16;  // 2-byte output: IEEE binary16 instead of bf16
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
// levels: the code is the level). BF16 selects the 2-byte output path (8 elements per 16-byte
// store): bf16, or binary16 when p.out_f16 is set (a wave-uniform choice of the conversion).
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
    const bool f16 = BF16 && p.out_f16 != 0;
    if (whole) {
        if (BF16) {
            u4 w;
#pragma unroll
            for (int i = 0; i < 4; ++i) w[i] = half_bits(o[2 * i], f16) | (half_bits(o[2 * i + 1], f16) << 16);
            __builtin_nontemporal_store(w, reinterpret_cast<u4*>(static_cast<uint16_t*>(p.out) + e));
        } else {
            const f4 a = {o[0], o[1], o[2], o[3]};
            __builtin_nontemporal_store(a, reinterpret_cast<f4*>(static_cast<float*>(p.out) + e));
        }
    } else {
        for (int i = 0; i < E; ++i) {
            if (e + i < limit) {
                if (BF16) static_cast<uint16_t*>(p.out)[e + i] = (uint16_t)half_bits(o[i], f16);
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

}  // namespace qsdp
