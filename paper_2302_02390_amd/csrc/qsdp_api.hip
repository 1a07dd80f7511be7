// C ABI of the QSDP codec library: argument validation, launch planning, and the kernels
// that are not specialised per bucket shape (block kernel, decoder).
#include "../../include/qsdp.h"

#include <cmath>
#include <cstdlib>
#include <cstring>

#include "qsdp_launch.hpp"

namespace qsdp {

hipError_t launch_block(int mode, const Params& p, unsigned grid, hipStream_t s) {
    switch (mode) {
        case MODE_GRAD: hipLaunchKernelGGL(block_kernel<MODE_GRAD>, dim3(grid), dim3(256), 0, s, p, p.segs); break;
        case MODE_WEIGHT: hipLaunchKernelGGL(block_kernel<MODE_WEIGHT>, dim3(grid), dim3(256), 0, s, p, p.segs); break;
        case MODE_FUSED: hipLaunchKernelGGL(block_kernel<MODE_FUSED>, dim3(grid), dim3(256), 0, s, p, p.segs); break;
        case MODE_FUSED_CODES: hipLaunchKernelGGL(block_kernel<MODE_FUSED_CODES>, dim3(grid), dim3(256), 0, s, p, p.segs); break;
        case MODE_LEVELS: hipLaunchKernelGGL(block_kernel<MODE_LEVELS>, dim3(grid), dim3(256), 0, s, p, p.segs); break;
        case MODE_ADAMW: hipLaunchKernelGGL(block_kernel<MODE_ADAMW>, dim3(grid), dim3(256), 0, s, p, p.segs); break;
        case MODE_ADAMW_CODES: hipLaunchKernelGGL(block_kernel<MODE_ADAMW_CODES>, dim3(grid), dim3(256), 0, s, p, p.segs); break;
        case MODE_RECV: hipLaunchKernelGGL(block_kernel<MODE_RECV>, dim3(grid), dim3(256), 0, s, p, p.segs); break;
        case MODE_RECV_ADAMW: hipLaunchKernelGGL(block_kernel<MODE_RECV_ADAMW>, dim3(grid), dim3(256), 0, s, p, p.segs); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

// Which bucket-index scheme the decoder kernels use for this call (tile = elements per wave).
static int bucket_indexing(const DequantParams& p, bool bf16) {
    const uint32_t tile32 = (uint32_t)kDequantRows * 64u * (bf16 ? 8u : 4u) / 32u;
    if (p.bucket32 % tile32 == 0) return BK_TILE_UNIFORM;
    return p.bucket32_shift >= 0 ? BK_SHIFT : BK_DIVIDE;
}

namespace {
template <int BITS, bool BF16, bool LUT>
void dequant_launch(int bk, const DequantParams& p, dim3 grid, hipStream_t s) {
    if (bk == BK_TILE_UNIFORM) hipLaunchKernelGGL((dequant_kernel<BITS, BF16, BK_TILE_UNIFORM, LUT>), grid, dim3(256), 0, s, p);
    else if (bk == BK_SHIFT) hipLaunchKernelGGL((dequant_kernel<BITS, BF16, BK_SHIFT, LUT>), grid, dim3(256), 0, s, p);
    else hipLaunchKernelGGL((dequant_kernel<BITS, BF16, BK_DIVIDE, LUT>), grid, dim3(256), 0, s, p);
}

template <int BITS>
hipError_t dequant_go(bool bf16, const DequantParams& p, dim3 grid, hipStream_t s) {
    const int bk = bucket_indexing(p, bf16);
    const bool lut = p.levels != nullptr;
    if (bf16 && lut) dequant_launch<BITS, true, true>(bk, p, grid, s);
    else if (bf16) dequant_launch<BITS, true, false>(bk, p, grid, s);
    else if (lut) dequant_launch<BITS, false, true>(bk, p, grid, s);
    else dequant_launch<BITS, false, false>(bk, p, grid, s);
    return hipGetLastError();
}
}  // namespace

namespace {
template <int BITS>
hipError_t dequant_add_go(const DequantAddParams& p, unsigned grid, hipStream_t s) {
    switch (bucket_indexing(p.d, false)) {
        case BK_TILE_UNIFORM: hipLaunchKernelGGL((dequant_add_kernel<BITS, BK_TILE_UNIFORM>), dim3(grid), dim3(256), 0, s, p); break;
        case BK_SHIFT: hipLaunchKernelGGL((dequant_add_kernel<BITS, BK_SHIFT>), dim3(grid), dim3(256), 0, s, p); break;
        default: hipLaunchKernelGGL((dequant_add_kernel<BITS, BK_DIVIDE>), dim3(grid), dim3(256), 0, s, p); break;
    }
    return hipGetLastError();
}
}  // namespace

hipError_t launch_dequant_add(int bits, const DequantAddParams& p, unsigned grid, hipStream_t s) {
    switch (bits) {
        case 1: return dequant_add_go<1>(p, grid, s);
        case 2: return dequant_add_go<2>(p, grid, s);
        case 3: return dequant_add_go<3>(p, grid, s);
        case 4: return dequant_add_go<4>(p, grid, s);
        case 5: return dequant_add_go<5>(p, grid, s);
        case 6: return dequant_add_go<6>(p, grid, s);
        case 7: return dequant_add_go<7>(p, grid, s);
        case 8: return dequant_add_go<8>(p, grid, s);
        default: return hipErrorInvalidValue;
    }
}

namespace {
template <int BITS, bool BF16, bool LUT>
void dequant_seg_launch(int bk, const DequantSegParams& q, unsigned grid, hipStream_t s) {
    if (bk == BK_TILE_UNIFORM) hipLaunchKernelGGL((dequant_seg_kernel<BITS, BF16, BK_TILE_UNIFORM, LUT>), dim3(grid), dim3(256), 0, s, q, q.segs);
    else if (bk == BK_SHIFT) hipLaunchKernelGGL((dequant_seg_kernel<BITS, BF16, BK_SHIFT, LUT>), dim3(grid), dim3(256), 0, s, q, q.segs);
    else hipLaunchKernelGGL((dequant_seg_kernel<BITS, BF16, BK_DIVIDE, LUT>), dim3(grid), dim3(256), 0, s, q, q.segs);
}

template <int BITS>
hipError_t dequant_seg_go(bool bf16, const DequantSegParams& q, unsigned grid, hipStream_t s) {
    const int bk = bucket_indexing(q.d, bf16);
    const bool lut = q.d.levels != nullptr;  // one table per tensor
    if (bf16 && lut) dequant_seg_launch<BITS, true, true>(bk, q, grid, s);
    else if (bf16) dequant_seg_launch<BITS, true, false>(bk, q, grid, s);
    else if (lut) dequant_seg_launch<BITS, false, true>(bk, q, grid, s);
    else dequant_seg_launch<BITS, false, false>(bk, q, grid, s);
    return hipGetLastError();
}
}  // namespace

hipError_t launch_dequant_seg(int bits, bool bf16, const DequantSegParams& q, unsigned grid, hipStream_t s) {
    switch (bits) {
        case 1: return dequant_seg_go<1>(bf16, q, grid, s);
        case 2: return dequant_seg_go<2>(bf16, q, grid, s);
        case 3: return dequant_seg_go<3>(bf16, q, grid, s);
        case 4: return dequant_seg_go<4>(bf16, q, grid, s);
        case 5: return dequant_seg_go<5>(bf16, q, grid, s);
        case 6: return dequant_seg_go<6>(bf16, q, grid, s);
        case 7: return dequant_seg_go<7>(bf16, q, grid, s);
        case 8: return dequant_seg_go<8>(bf16, q, grid, s);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_fit_levels(const FitParams& p, unsigned grid, hipStream_t s) {
    switch (p.bits) {
        case 1: hipLaunchKernelGGL(fit_levels_kernel<1>, dim3(grid), dim3(256), 0, s, p); break;
        case 2: hipLaunchKernelGGL(fit_levels_kernel<2>, dim3(grid), dim3(256), 0, s, p); break;
        case 3: hipLaunchKernelGGL(fit_levels_kernel<3>, dim3(grid), dim3(256), 0, s, p); break;
        case 4: hipLaunchKernelGGL(fit_levels_kernel<4>, dim3(grid), dim3(256), 0, s, p); break;
        case 5: hipLaunchKernelGGL(fit_levels_kernel<5>, dim3(grid), dim3(256), 0, s, p); break;
        case 6: hipLaunchKernelGGL(fit_levels_kernel<6>, dim3(grid), dim3(256), 0, s, p); break;
        case 7: hipLaunchKernelGGL(fit_levels_kernel<7>, dim3(grid), dim3(256), 0, s, p); break;
        case 8: hipLaunchKernelGGL(fit_levels_kernel<8>, dim3(grid), dim3(256), 0, s, p); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_dequant(int bits, bool bf16, const DequantParams& p, dim3 grid, hipStream_t s) {
    switch (bits) {
        case 1: return dequant_go<1>(bf16, p, grid, s);
        case 2: return dequant_go<2>(bf16, p, grid, s);
        case 3: return dequant_go<3>(bf16, p, grid, s);
        case 4: return dequant_go<4>(bf16, p, grid, s);
        case 5: return dequant_go<5>(bf16, p, grid, s);
        case 6: return dequant_go<6>(bf16, p, grid, s);
        case 7: return dequant_go<7>(bf16, p, grid, s);
        case 8: return dequant_go<8>(bf16, p, grid, s);
        default: return hipErrorInvalidValue;
    }
}

namespace {

constexpr unsigned kMaxGrid = 1u << 20;
constexpr unsigned kLevelsGrid = 1u << 15;

// Workgroups to launch for `blocks` units of work: all of them up to kMaxGrid, the kernels stride
// beyond that. QSDP_DEBUG_MAXGRID (the library's one debug switch) lowers the cap so that the
// striding paths can be exercised on small inputs.
unsigned capped_grid(uint64_t blocks, unsigned cap = kMaxGrid) {
    if (const char* e = std::getenv("QSDP_DEBUG_MAXGRID")) {
        const long v = std::atol(e);
        if (v >= 1 && v < (long)cap) cap = (unsigned)v;
    }
    return (unsigned)(blocks < cap ? blocks : cap);
}

bool shape_ok(uint64_t n, int bits, int bucket) {
    return n >= 1 && bits >= 1 && bits <= 8 && bucket >= 32 && bucket <= kMaxBucket && bucket % 32 == 0;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

uint64_t ceil_div(uint64_t a, uint64_t b) { return (a + b - 1) / b; }

// 1/delta is exact iff delta is a normal power of two whose reciprocal is normal too.
bool reciprocal_exact(float delta) {
    uint32_t b;
    std::memcpy(&b, &delta, sizeof b);
    const uint32_t expo = (b >> 23) & 0xFFu;
    return (b & 0x7FFFFFu) == 0 && expo >= 2 && expo <= 252;
}

typedef hipError_t (*WaveLauncher)(int, int, const Params&, unsigned, hipStream_t);

WaveLauncher wave_launcher(int bucket, int* buckets_per_wave) {
    switch (bucket) {
        case 128: *buckets_per_wave = 8; return launch_wave_128;
        case 256: *buckets_per_wave = 4; return launch_wave_256;
        case 512: *buckets_per_wave = 2; return launch_wave_512;
        case 1024: *buckets_per_wave = 1; return launch_wave_1024;
        case 2048: *buckets_per_wave = 0; return launch_wave_2048;  // 0: a workgroup per bucket
        case 4096: *buckets_per_wave = 0; return launch_wave_4096;
        default: return nullptr;
    }
}

// Buckets go to the wave kernel of the bucket's shape when there is one for (bucket, stored
// code width; for MODE_RECV also the width of the peers' codes), else to the block kernel.
// p.num_buckets must be set.
int run(int mode, Params p, int stored_bits, hipStream_t s) {
    const uint64_t nb = p.num_buckets;
    p.first_bucket = 0;
    int bpw = 1;
    WaveLauncher wl = wave_launcher(p.bucket, &bpw);
    if (mode == MODE_WEIGHT && p.bucket == 1024 && p.segs == nullptr) {
        // memory-bound and light on arithmetic: two waves per bucket (half the tile per wave) stream
        // 4 % faster here; every mode with more arithmetic, and the multi-tensor form (one table search
        // per wave), is faster with one wave per bucket
        wl = launch_wave_1024w2;
        bpw = 0;
    }
    const bool peer_bits_ok = !mode_reads_peers(mode) || (p.gbits != 0 && wave_bits_supported(p.gbits));
    if (wl != nullptr && wave_bits_supported(stored_bits) && peer_bits_ok) {
        // 4 waves per workgroup, each on bpw buckets; or one workgroup per bucket
        const uint64_t blocks = bpw > 0 ? ceil_div(ceil_div(nb, (uint64_t)bpw), 4) : nb;
        // The learned-level encoders set up lookup tables per workgroup: their workgroups stay resident
        // and stride over the buckets (measured best around 128 workgroups per compute unit).
        const unsigned cap = mode_is_levels(mode) ? kLevelsGrid : kMaxGrid;
        if (wl(mode, stored_bits, p, capped_grid(blocks, cap), s) != hipSuccess) return QSDP_ELAUNCH;
    } else {
        if (launch_block(mode == MODE_LEVELS_COIN ? MODE_LEVELS : mode, p, capped_grid(nb), s) != hipSuccess)
            return QSDP_ELAUNCH;
    }
    return QSDP_OK;
}

void set_common(Params& p, uint64_t n, int bucket, uint64_t seed, uint64_t index_offset, float delta) {
    p.n = n;
    p.num_buckets = ceil_div(n, (uint64_t)bucket);
    p.bucket = bucket;
    p.block0 = index_offset >> 3;
    p.key0 = (uint32_t)seed;
    p.key1 = (uint32_t)(seed >> 32);
    p.delta = delta;
    p.delta_pow2 = (delta > 0.0f && reciprocal_exact(delta)) ? 1 : 0;
    p.inv_delta = p.delta_pow2 ? 1.0f / delta : 0.0f;
}

}  // namespace
}  // namespace qsdp

using namespace qsdp;

// A multi-tensor call's segment table (device pointer) as the segmented entry points receive it.
struct SegmentTable {
    const qsdp_segment* table;
    uint32_t nseg;
    uint64_t total_buckets;
};

// The AdamW moments and scalars of the AdamW-flavoured steps.
struct AdamScalars {
    float *m, *v;
    float beta1, beta2, eps, weight_decay, bias1, bias2;
};

static bool adam_ok(const AdamScalars& a) {
    return a.m && a.v && a.beta1 >= 0.0f && a.beta1 < 1.0f && a.beta2 >= 0.0f && a.beta2 < 1.0f && a.eps > 0.0f &&
           a.bias1 > 0.0f && a.bias2 > 0.0f && std::isfinite(a.weight_decay);
}

static void set_adam(Params& p, const AdamScalars& a) {
    p.mom = a.m;
    p.var = a.v;
    p.beta1 = a.beta1;
    p.beta2 = a.beta2;
    p.omb1 = 1.0f - a.beta1;
    p.omb2 = 1.0f - a.beta2;
    p.eps = a.eps;
    p.weight_decay = a.weight_decay;
    p.bias1 = a.bias1;
    p.bias2 = a.bias2;
}

// Validates a segment table argument; on success *n is replaced by the number of code slots.
static int segments_ok(const SegmentTable& segs, int bucket, uint64_t* n) {
    if (!segs.table || segs.nseg == 0 || segs.total_buckets < segs.nseg || bucket <= 0) return QSDP_EINVAL;
    if (reinterpret_cast<uintptr_t>(segs.table) & 7u) return QSDP_EALIGN;
    *n = segs.total_buckets * (uint64_t)bucket;
    return QSDP_OK;
}

static void set_segments(Params& p, const SegmentTable& segs) {
    p.segs = reinterpret_cast<const Segment*>(segs.table);
    p.nseg = segs.nseg;
    p.num_buckets = segs.total_buckets;
}

static_assert(sizeof(qsdp_segment) == sizeof(Segment), "segment layout");

extern "C" {

uint32_t qsdp_spec_version(void) { return 3u; }

size_t qsdp_codes_bytes(uint64_t n, int bits, int bucket) {
    if (!shape_ok(n, bits, bucket)) return 0;
    return (size_t)(ceil_div(n, (uint64_t)bucket) * (uint64_t)bucket * (uint64_t)bits / 8u);
}

size_t qsdp_meta_bytes(uint64_t n, int bucket) {
    if (!shape_ok(n, 8, bucket)) return 0;
    return (size_t)(ceil_div(n, (uint64_t)bucket) * 2u * sizeof(float));
}

const char* qsdp_status_string(int status) {
    switch (status) {
        case QSDP_OK: return "ok";
        case QSDP_EINVAL: return "invalid argument";
        case QSDP_EALIGN: return "pointer not 16-byte aligned";
        case QSDP_ELAUNCH: return "kernel launch failed";
        default: return "unknown status";
    }
}

int qsdp_quantize_grad(const float* g, uint64_t n, int bits, int bucket, uint64_t seed,
                       uint64_t index_offset, uint32_t* codes, float* meta, void* stream) {
    return qsdp_quantize_grad_ex(g, n, bits, bucket, seed, index_offset, 0u, codes, meta, stream);
}

static int quantize_grad_common(uint32_t g_half, const void* g, uint64_t n, int bits, int bucket, uint64_t seed,
                                uint64_t index_offset, uint32_t flags, uint32_t* codes, float* meta, void* stream) {
    if (!g || !codes || !meta || !shape_ok(n, bits, bucket) || (index_offset & 7u) || (flags & ~QSDP_FLAG_ALL))
        return QSDP_EINVAL;
    if (!aligned16(g) || !aligned16(codes) || !aligned16(meta)) return QSDP_EALIGN;
    Params p = {};
    set_common(p, n, bucket, seed, index_offset, 0.0f);
    p.flags = flags;
    p.g = static_cast<const float*>(g);
    p.g_half = g_half;
    p.codes = codes;
    p.meta = meta;
    p.gbits = bits;
    p.wbits = bits;
    return run(MODE_GRAD, p, bits, static_cast<hipStream_t>(stream));
}

int qsdp_quantize_grad_ex(const float* g, uint64_t n, int bits, int bucket, uint64_t seed,
                          uint64_t index_offset, uint32_t flags, uint32_t* codes, float* meta, void* stream) {
    return quantize_grad_common(0u, g, n, bits, bucket, seed, index_offset, flags, codes, meta, stream);
}

// 1 / 2 for a 2-byte gradient format of the C header, 0 for anything else
static uint32_t half_format(qsdp_dtype t) { return t == QSDP_BF16 ? 1u : t == QSDP_F16 ? 2u : 0u; }

int qsdp_quantize_grad_g16(const void* g, qsdp_dtype g_dtype, uint64_t n, int bits, int bucket, uint64_t seed,
                           uint64_t index_offset, uint32_t flags, uint32_t* codes, float* meta, void* stream) {
    if (half_format(g_dtype) == 0u) return QSDP_EINVAL;
    return quantize_grad_common(half_format(g_dtype), g, n, bits, bucket, seed, index_offset, flags, codes, meta,
                                stream);
}

int qsdp_quantize_weight(const float* x, uint64_t n, int bits, int bucket, float delta,
                         uint64_t seed, uint32_t* codes, float* meta, uint64_t* n_saturated,
                         void* stream) {
    return qsdp_quantize_weight_ex(x, n, bits, bucket, delta, seed, 0u, codes, meta, n_saturated, stream);
}

int qsdp_quantize_weight_ex(const float* x, uint64_t n, int bits, int bucket, float delta,
                            uint64_t seed, uint32_t flags, uint32_t* codes, float* meta,
                            uint64_t* n_saturated, void* stream) {
    if (!x || !codes || !meta || !shape_ok(n, bits, bucket) || (flags & ~QSDP_FLAG_ALL)) return QSDP_EINVAL;
    if (!(delta >= 0.0f) || !std::isfinite(delta)) return QSDP_EINVAL;
    if (!aligned16(x) || !aligned16(codes) || !aligned16(meta)) return QSDP_EALIGN;
    if (n_saturated && (reinterpret_cast<uintptr_t>(n_saturated) & 7u)) return QSDP_EALIGN;
    Params p = {};
    set_common(p, n, bucket, seed, 0, delta);
    p.flags = flags;
    p.xin = x;
    p.codes = codes;
    p.meta = meta;
    p.n_saturated = reinterpret_cast<unsigned long long*>(n_saturated);
    p.gbits = bits;
    p.wbits = bits;
    return run(MODE_WEIGHT, p, bits, static_cast<hipStream_t>(stream));
}

static DequantParams decoder_params(const uint32_t* codes, const float* meta, uint64_t n, int bits,
                                    int bucket, bool bf16, void* out, unsigned* grid) {
    DequantParams p = {};
    p.codes = codes;
    p.meta = meta;
    p.out = out;
    p.n = n;
    p.nwords = qsdp_codes_bytes(n, bits, bucket) / 4;
    const uint64_t tile = (uint64_t)kDequantRows * 64u * (bf16 ? 8u : 4u);
    p.ntiles = ceil_div(n, tile);
    p.bucket32 = (uint32_t)bucket / 32u;
    p.bucket32_shift = -1;
    for (int sh = 0; sh < 9; ++sh)
        if (p.bucket32 == (1u << sh)) p.bucket32_shift = sh;
    const uint64_t blocks = ceil_div(p.ntiles, 4);
    *grid = capped_grid(blocks);
    p.n_last = p.n;
    p.nwords_last = p.nwords;
    p.ntiles_last = p.ntiles;
    return p;
}

int qsdp_dequantize(const uint32_t* codes, const float* meta, uint64_t n, int bits, int bucket,
                    qsdp_dtype out_dtype, void* out, void* stream) {
    if (!codes || !meta || !out || !shape_ok(n, bits, bucket)) return QSDP_EINVAL;
    if (out_dtype != QSDP_F32 && out_dtype != QSDP_BF16 && out_dtype != QSDP_F16) return QSDP_EINVAL;
    if (n >= (1ull << 37)) return QSDP_EINVAL;  // the decoder indexes buckets with 32-bit arithmetic
    if (!aligned16(codes) || !aligned16(meta) || !aligned16(out)) return QSDP_EALIGN;
    unsigned grid = 0;
    DequantParams p = decoder_params(codes, meta, n, bits, bucket, out_dtype != QSDP_F32, out, &grid);
    p.out_f16 = out_dtype == QSDP_F16 ? 1u : 0u;
    if (launch_dequant(bits, out_dtype != QSDP_F32, p, grid, static_cast<hipStream_t>(stream)) != hipSuccess)
        return QSDP_ELAUNCH;
    return QSDP_OK;
}

int qsdp_levels_uniform(int bits, float* levels) {
    if (bits < 1 || bits > 8 || !levels) return QSDP_EINVAL;
    const int K = 1 << bits;
    for (int k = 0; k < K; ++k) levels[k] = (float)k / (float)(K - 1);
    return QSDP_OK;
}

int qsdp_quantize_levels(const float* v, uint64_t n, int bits, int bucket, const float* levels,
                         uint32_t* codes, float* meta, void* stream) {
    if (!v || !levels || !codes || !meta || !shape_ok(n, bits, bucket)) return QSDP_EINVAL;
    if (!aligned16(v) || !aligned16(codes) || !aligned16(meta) || (reinterpret_cast<uintptr_t>(levels) & 3u))
        return QSDP_EALIGN;
    Params p = {};
    set_common(p, n, bucket, 0, 0, 0.0f);
    p.xin = v;
    p.levels = levels;
    p.codes = codes;
    p.meta = meta;
    p.gbits = bits;
    p.wbits = bits;
    return run(MODE_LEVELS, p, bits, static_cast<hipStream_t>(stream));
}

int qsdp_quantize_levels_stochastic(const float* v, uint64_t n, int bits, int bucket, const float* levels,
                                    uint64_t seed, uint64_t index_offset, uint32_t* codes, float* meta,
                                    void* stream) {
    if (!v || !levels || !codes || !meta || !shape_ok(n, bits, bucket) || (index_offset & 7u)) return QSDP_EINVAL;
    if (!aligned16(v) || !aligned16(codes) || !aligned16(meta) || (reinterpret_cast<uintptr_t>(levels) & 3u))
        return QSDP_EALIGN;
    Params p = {};
    set_common(p, n, bucket, seed, index_offset, 0.0f);
    p.flags = FLAG_LEVELS_STOCHASTIC;
    p.xin = v;
    p.levels = levels;
    p.codes = codes;
    p.meta = meta;
    p.gbits = bits;
    p.wbits = bits;
    return run(MODE_LEVELS_COIN, p, bits, static_cast<hipStream_t>(stream));
}

int qsdp_dequantize_levels(const uint32_t* codes, const float* meta, uint64_t n, int bits, int bucket,
                           const float* levels, qsdp_dtype out_dtype, void* out, void* stream) {
    if (!codes || !meta || !levels || !out || !shape_ok(n, bits, bucket)) return QSDP_EINVAL;
    if (out_dtype != QSDP_F32 && out_dtype != QSDP_BF16 && out_dtype != QSDP_F16) return QSDP_EINVAL;
    if (n >= (1ull << 37)) return QSDP_EINVAL;
    if (!aligned16(codes) || !aligned16(meta) || !aligned16(out) || (reinterpret_cast<uintptr_t>(levels) & 3u))
        return QSDP_EALIGN;
    unsigned grid = 0;
    DequantParams p = decoder_params(codes, meta, n, bits, bucket, out_dtype != QSDP_F32, out, &grid);
    p.levels = levels;
    p.out_f16 = out_dtype == QSDP_F16 ? 1u : 0u;
    if (launch_dequant(bits, out_dtype != QSDP_F32, p, grid, static_cast<hipStream_t>(stream)) != hipSuccess)
        return QSDP_ELAUNCH;
    return QSDP_OK;
}

int qsdp_fit_levels(const float* v, uint64_t n, int bits, int bucket, float lr, uint64_t max_batches,
                    float* levels, void* stream) {
    if (!v || !levels || !shape_ok(n, bits, bucket) || !(lr > 0.0f && lr < 1.0f)) return QSDP_EINVAL;
    if (!aligned16(v) || (reinterpret_cast<uintptr_t>(levels) & 3u)) return QSDP_EALIGN;
    FitParams p = {};
    p.v = v;
    p.levels = levels;
    p.n = n;
    p.num_batches = ceil_div(n, (uint64_t)bucket);
    if (max_batches > 0 && max_batches < p.num_batches) p.num_batches = max_batches;
    p.bucket = bucket;
    p.bits = bits;
    p.lr = lr;
    if (launch_fit_levels(p, 1u, static_cast<hipStream_t>(stream)) != hipSuccess) return QSDP_ELAUNCH;
    return QSDP_OK;
}

int qsdp_fit_levels_segmented(const float* v, const qsdp_segment* table, uint32_t nseg, int bits, int bucket,
                              float lr, uint64_t max_batches, float* levels, void* stream) {
    if (!v || !table || nseg == 0 || !levels || !shape_ok(1, bits, bucket) || !(lr > 0.0f && lr < 1.0f))
        return QSDP_EINVAL;
    if (!aligned16(v) || (reinterpret_cast<uintptr_t>(levels) & 3u) || (reinterpret_cast<uintptr_t>(table) & 7u))
        return QSDP_EALIGN;
    FitParams p = {};
    p.v = v;
    p.levels = levels;
    p.num_batches = max_batches;
    p.segs = reinterpret_cast<const Segment*>(table);
    p.bucket = bucket;
    p.bits = bits;
    p.lr = lr;
    if (launch_fit_levels(p, nseg, static_cast<hipStream_t>(stream)) != hipSuccess) return QSDP_ELAUNCH;
    return QSDP_OK;
}

int qsdp_dequantize_add(const uint32_t* codes, uint64_t codes_stride_bytes, const float* meta,
                        uint64_t meta_stride_bytes, int npeers, uint64_t n, int bits, int bucket,
                        float alpha, float* out, void* stream) {
    if (!codes || !meta || !out || npeers < 1 || !shape_ok(n, bits, bucket) || !std::isfinite(alpha))
        return QSDP_EINVAL;
    if (n >= (1ull << 37)) return QSDP_EINVAL;
    if (npeers > 1 && (codes_stride_bytes < qsdp_codes_bytes(n, bits, bucket) ||
                       meta_stride_bytes < qsdp_meta_bytes(n, bucket)))
        return QSDP_EINVAL;
    if (!aligned16(codes) || !aligned16(meta) || !aligned16(out) || (codes_stride_bytes & 3u) ||
        (meta_stride_bytes & 3u))
        return QSDP_EALIGN;
    int unused_bpw = 0;
    if (wave_launcher(bucket, &unused_bpw) != nullptr && (codes_stride_bytes & 15u) == 0) {
        // a bucket size the wave kernels cover: 16-byte code fetches staged through LDS instead of
        // per-lane word loads
        Params p = {};
        set_common(p, n, bucket, 0, 0, 0.0f);
        p.x = out;
        p.peer_codes = codes;
        p.peer_meta = meta;
        p.peer_codes_stride_words = codes_stride_bytes / 4;
        p.peer_meta_stride_floats = meta_stride_bytes / 4;
        p.npeers = npeers;
        p.alpha = alpha;
        p.gbits = bits;
        p.wbits = bits;
        return run(MODE_SUM, p, 0, static_cast<hipStream_t>(stream));
    }
    DequantAddParams q = {};
    unsigned grid = 0;
    q.d = decoder_params(codes, meta, n, bits, bucket, false, out, &grid);
    q.codes_stride_words = codes_stride_bytes / 4;
    q.meta_stride_floats = meta_stride_bytes / 4;
    q.npeers = npeers;
    q.alpha = alpha;
    if (launch_dequant_add(bits, q, grid, static_cast<hipStream_t>(stream)) != hipSuccess) return QSDP_ELAUNCH;
    return QSDP_OK;
}

// Every form of the fused step (SGD or AdamW between the quantizers) from one options block.
static int step_from_options(bool adamw, float* x, const void* g, uint64_t n, float lr, int wbits, int gbits,
                             int bucket, float delta, uint64_t seed, uint64_t index_offset,
                             const qsdp_step_options* opt, void* stream) {
    qsdp_step_options o = {};
    if (opt != nullptr) {
        if (opt->size != sizeof(qsdp_step_options)) return QSDP_EINVAL;
        o = *opt;
    }
    const bool multi = o.segments != nullptr;
    const SegmentTable segs = {o.segments, o.nseg, o.total_buckets};
    if (multi) {
        const int rc = segments_ok(segs, bucket, &n);
        if (rc != QSDP_OK) return rc;
    }
    if (o.g_dtype != QSDP_F32 && half_format(o.g_dtype) == 0u) return QSDP_EINVAL;
    if (o.x16 != nullptr && half_format(o.x16_dtype) == 0u) return QSDP_EINVAL;
    const AdamScalars adam = {o.m, o.v, o.beta1, o.beta2, o.eps, o.weight_decay, o.bias1, o.bias2};
    if (!x || !g || !shape_ok(n, wbits, bucket) || !shape_ok(n, gbits, bucket) || (adamw && !adam_ok(adam)) ||
        (o.flags & ~(uint32_t)(QSDP_FLAG_ALL | QSDP_FLAG_KEEP_MASTER)))
        return QSDP_EINVAL;
    if (!(delta >= 0.0f) || !std::isfinite(delta) || !std::isfinite(lr)) return QSDP_EINVAL;
    if ((o.wcodes == nullptr) != (o.wmeta == nullptr) || (index_offset & 7u)) return QSDP_EINVAL;
    if (!aligned16(x) || !aligned16(g) || !aligned16(o.wcodes) || !aligned16(o.wmeta) || !aligned16(o.x16))
        return QSDP_EALIGN;
    if (adamw && (!aligned16(adam.m) || !aligned16(adam.v))) return QSDP_EALIGN;
    if (o.n_saturated && (reinterpret_cast<uintptr_t>(o.n_saturated) & 7u)) return QSDP_EALIGN;
    if (o.seed_increment && (reinterpret_cast<uintptr_t>(o.seed_increment) & 7u)) return QSDP_EALIGN;
    Params p = {};
    set_common(p, multi ? 0 : n, bucket, seed, index_offset, delta);
    if (multi) set_segments(p, segs);
    p.flags = o.flags;
    p.x = x;
    p.x16 = o.x16;
    p.x16_f16 = o.x16_dtype == QSDP_F16 ? 1u : 0u;
    p.g = static_cast<const float*>(g);
    p.g_half = half_format(o.g_dtype);
    p.codes = o.wcodes;
    p.meta = o.wmeta;
    p.n_saturated = reinterpret_cast<unsigned long long*>(o.n_saturated);
    p.gbits = gbits;
    p.wbits = wbits;
    p.lr = lr;
    p.seed_dev = reinterpret_cast<const unsigned long long*>(o.seed_increment);
    if (adamw) set_adam(p, adam);
    return run(adamw ? MODE_ADAMW : MODE_FUSED, p, o.wcodes ? wbits : 0, static_cast<hipStream_t>(stream));
}

int qsdp_fused_step_opts(float* x, const void* g, uint64_t n, float lr, int wbits, int gbits, int bucket,
                         float delta, uint64_t seed, uint64_t index_offset, const qsdp_step_options* opt,
                         void* stream) {
    return step_from_options(false, x, g, n, lr, wbits, gbits, bucket, delta, seed, index_offset, opt, stream);
}

int qsdp_fused_adamw_step_opts(float* x, const void* g, uint64_t n, float lr, int wbits, int gbits, int bucket,
                               float delta, uint64_t seed, uint64_t index_offset, const qsdp_step_options* opt,
                               void* stream) {
    return step_from_options(true, x, g, n, lr, wbits, gbits, bucket, delta, seed, index_offset, opt, stream);
}

// ---- thin forwards of the two calls above: each fills the options block from its argument list ----
static qsdp_step_options options_for(uint32_t flags, uint32_t* wcodes, float* wmeta, uint64_t* n_saturated) {
    qsdp_step_options o = {};
    o.size = sizeof o;
    o.flags = flags;
    o.wcodes = wcodes;
    o.wmeta = wmeta;
    o.n_saturated = n_saturated;
    return o;
}

static void set_adam_options(qsdp_step_options& o, float* m, float* v, float beta1, float beta2, float eps,
                             float weight_decay, float bias1, float bias2) {
    o.m = m; o.v = v; o.beta1 = beta1; o.beta2 = beta2; o.eps = eps; o.weight_decay = weight_decay;
    o.bias1 = bias1; o.bias2 = bias2;
}

static void set_segment_options(qsdp_step_options& o, const qsdp_segment* table, uint32_t nseg, uint64_t total_buckets) {
    o.segments = table; o.nseg = nseg; o.total_buckets = total_buckets;
}

int qsdp_fused_step(float* x, const float* g, uint64_t n, float lr, int wbits, int gbits, int bucket,
                    float delta, uint64_t seed, uint64_t index_offset, uint32_t* wcodes, float* wmeta,
                    uint64_t* n_saturated, void* stream) {
    const qsdp_step_options o = options_for(0u, wcodes, wmeta, n_saturated);
    return qsdp_fused_step_opts(x, g, n, lr, wbits, gbits, bucket, delta, seed, index_offset, &o, stream);
}

int qsdp_fused_step_ex(float* x, const float* g, uint64_t n, float lr, int wbits, int gbits, int bucket,
                       float delta, uint64_t seed, uint64_t index_offset, uint32_t flags, uint32_t* wcodes,
                       float* wmeta, uint64_t* n_saturated, void* stream) {
    const qsdp_step_options o = options_for(flags, wcodes, wmeta, n_saturated);
    return qsdp_fused_step_opts(x, g, n, lr, wbits, gbits, bucket, delta, seed, index_offset, &o, stream);
}

int qsdp_fused_step_dseed(float* x, const float* g, uint64_t n, float lr, int wbits, int gbits, int bucket,
                          float delta, uint64_t seed, const uint64_t* seed_dev, uint64_t index_offset,
                          uint32_t flags, uint32_t* wcodes, float* wmeta, uint64_t* n_saturated, void* stream) {
    if (!seed_dev) return QSDP_EINVAL;
    qsdp_step_options o = options_for(flags, wcodes, wmeta, n_saturated);
    o.seed_increment = seed_dev;
    return qsdp_fused_step_opts(x, g, n, lr, wbits, gbits, bucket, delta, seed, index_offset, &o, stream);
}

int qsdp_fused_step_g16(float* x, const void* g, qsdp_dtype g_dtype, uint64_t n, float lr, int wbits, int gbits,
                        int bucket, float delta, uint64_t seed, uint64_t index_offset, uint32_t flags,
                        uint32_t* wcodes, float* wmeta, uint64_t* n_saturated, void* stream) {
    if (half_format(g_dtype) == 0u) return QSDP_EINVAL;
    qsdp_step_options o = options_for(flags, wcodes, wmeta, n_saturated);
    o.g_dtype = g_dtype;
    return qsdp_fused_step_opts(x, g, n, lr, wbits, gbits, bucket, delta, seed, index_offset, &o, stream);
}

int qsdp_fused_step_mp(float* x, const void* g, qsdp_dtype g_dtype, uint64_t n, float lr, int wbits, int gbits,
                       int bucket, float delta, uint64_t seed, uint64_t index_offset, uint32_t flags, uint32_t* wcodes,
                       float* wmeta, void* x16, qsdp_dtype x16_dtype, uint64_t* n_saturated, void* stream) {
    qsdp_step_options o = options_for(flags, wcodes, wmeta, n_saturated);
    o.g_dtype = g_dtype;
    o.x16 = x16;
    o.x16_dtype = x16_dtype;
    return qsdp_fused_step_opts(x, g, n, lr, wbits, gbits, bucket, delta, seed, index_offset, &o, stream);
}

int qsdp_fused_step_segmented_mp(float* x, const void* g, qsdp_dtype g_dtype, const qsdp_segment* table,
                                 uint32_t nseg, uint64_t total_buckets, float lr, int wbits, int gbits,
                                 int bucket, float delta, uint64_t seed, uint64_t index_offset, uint32_t flags,
                                 uint32_t* wcodes, float* wmeta, void* x16, qsdp_dtype x16_dtype,
                                 uint64_t* n_saturated, void* stream) {
    if (!table) return QSDP_EINVAL;
    qsdp_step_options o = options_for(flags, wcodes, wmeta, n_saturated);
    o.g_dtype = g_dtype;
    o.x16 = x16;
    o.x16_dtype = x16_dtype;
    set_segment_options(o, table, nseg, total_buckets);
    return qsdp_fused_step_opts(x, g, 0, lr, wbits, gbits, bucket, delta, seed, index_offset, &o, stream);
}

int qsdp_fused_adamw_step(float* x, const float* g, float* m, float* v, uint64_t n, float lr, float beta1,
                          float beta2, float eps, float weight_decay, float bias1, float bias2, int wbits,
                          int gbits, int bucket, float delta, uint64_t seed, uint64_t index_offset,
                          uint32_t flags, uint32_t* wcodes, float* wmeta, uint64_t* n_saturated, void* stream) {
    qsdp_step_options o = options_for(flags, wcodes, wmeta, n_saturated);
    set_adam_options(o, m, v, beta1, beta2, eps, weight_decay, bias1, bias2);
    return qsdp_fused_adamw_step_opts(x, g, n, lr, wbits, gbits, bucket, delta, seed, index_offset, &o, stream);
}

int qsdp_fused_adamw_step_mp(float* x, const void* g, qsdp_dtype g_dtype, float* m, float* v, uint64_t n, float lr,
                             float beta1, float beta2, float eps, float weight_decay, float bias1, float bias2,
                             int wbits, int gbits, int bucket, float delta, uint64_t seed, uint64_t index_offset,
                             uint32_t flags, uint32_t* wcodes, float* wmeta, void* x16, qsdp_dtype x16_dtype,
                             uint64_t* n_saturated, void* stream) {
    qsdp_step_options o = options_for(flags, wcodes, wmeta, n_saturated);
    set_adam_options(o, m, v, beta1, beta2, eps, weight_decay, bias1, bias2);
    o.g_dtype = g_dtype;
    o.x16 = x16;
    o.x16_dtype = x16_dtype;
    return qsdp_fused_adamw_step_opts(x, g, n, lr, wbits, gbits, bucket, delta, seed, index_offset, &o, stream);
}

int qsdp_fused_adamw_step_segmented(float* x, const float* g, float* m, float* v, const qsdp_segment* table,
                                    uint32_t nseg, uint64_t total_buckets, float lr, float beta1, float beta2,
                                    float eps, float weight_decay, float bias1, float bias2, int wbits, int gbits,
                                    int bucket, float delta, uint64_t seed, uint64_t index_offset,
                                    uint32_t flags, uint32_t* wcodes, float* wmeta, uint64_t* n_saturated,
                                    void* stream) {
    if (!table) return QSDP_EINVAL;
    qsdp_step_options o = options_for(flags, wcodes, wmeta, n_saturated);
    set_adam_options(o, m, v, beta1, beta2, eps, weight_decay, bias1, bias2);
    set_segment_options(o, table, nseg, total_buckets);
    return qsdp_fused_adamw_step_opts(x, g, 0, lr, wbits, gbits, bucket, delta, seed, index_offset, &o, stream);
}

static int fused_step_codes_common(const AdamScalars* adam, const SegmentTable* segs, uint32_t* wcodes, float* wmeta, const float* g,
                                   uint64_t n, float lr, int wbits, int gbits, int bucket, float delta,
                                   uint64_t seed, uint64_t index_offset, uint32_t flags, uint64_t* n_saturated,
                                   void* stream) {
    if (segs) {
        const int rc = segments_ok(*segs, bucket, &n);
        if (rc != QSDP_OK) return rc;
    }
    if (!wcodes || !wmeta || !g || !shape_ok(n, wbits, bucket) || !shape_ok(n, gbits, bucket) ||
        (flags & ~QSDP_FLAG_ALL))
        return QSDP_EINVAL;
    if (!(delta >= 0.0f) || !std::isfinite(delta) || !std::isfinite(lr) || (index_offset & 7u)) return QSDP_EINVAL;
    if (adam && !adam_ok(*adam)) return QSDP_EINVAL;
    if (!aligned16(wcodes) || !aligned16(wmeta) || !aligned16(g)) return QSDP_EALIGN;
    if (adam && (!aligned16(adam->m) || !aligned16(adam->v))) return QSDP_EALIGN;
    if (n_saturated && (reinterpret_cast<uintptr_t>(n_saturated) & 7u)) return QSDP_EALIGN;
    Params p = {};
    set_common(p, segs ? 0 : n, bucket, seed, index_offset, delta);
    if (segs) set_segments(p, *segs);
    p.flags = flags;
    p.g = g;
    p.codes = wcodes;
    p.meta = wmeta;
    p.n_saturated = reinterpret_cast<unsigned long long*>(n_saturated);
    p.gbits = gbits;
    p.wbits = wbits;
    p.lr = lr;
    if (adam) set_adam(p, *adam);
    return run(adam ? MODE_ADAMW_CODES : MODE_FUSED_CODES, p, wbits, static_cast<hipStream_t>(stream));
}

int qsdp_fused_step_codes(uint32_t* wcodes, float* wmeta, const float* g, uint64_t n, float lr, int wbits,
                          int gbits, int bucket, float delta, uint64_t seed, uint64_t index_offset,
                          uint32_t flags, uint64_t* n_saturated, void* stream) {
    return fused_step_codes_common(nullptr, nullptr, wcodes, wmeta, g, n, lr, wbits, gbits, bucket, delta, seed, index_offset,
                                   flags, n_saturated, stream);
}

int qsdp_fused_step_codes_segmented(uint32_t* wcodes, float* wmeta, const float* g, const qsdp_segment* table,
                                    uint32_t nseg, uint64_t total_buckets, float lr, int wbits, int gbits,
                                    int bucket, float delta, uint64_t seed, uint64_t index_offset,
                                    uint32_t flags, uint64_t* n_saturated, void* stream) {
    const SegmentTable segs = {table, nseg, total_buckets};
    return fused_step_codes_common(nullptr, &segs, wcodes, wmeta, g, 0, lr, wbits, gbits, bucket, delta, seed, index_offset,
                                   flags, n_saturated, stream);
}

int qsdp_fused_adamw_step_codes(uint32_t* wcodes, float* wmeta, const float* g, float* m, float* v, uint64_t n,
                                float lr, float beta1, float beta2, float eps, float weight_decay, float bias1,
                                float bias2, int wbits, int gbits, int bucket, float delta, uint64_t seed,
                                uint64_t index_offset, uint32_t flags, uint64_t* n_saturated, void* stream) {
    const AdamScalars adam = {m, v, beta1, beta2, eps, weight_decay, bias1, bias2};
    return fused_step_codes_common(&adam, nullptr, wcodes, wmeta, g, n, lr, wbits, gbits, bucket, delta, seed,
                                   index_offset, flags, n_saturated, stream);
}

uint64_t qsdp_segments_build(const uint64_t* sizes, uint32_t nseg, int bucket, qsdp_segment* table) {
    if (!sizes || !table || nseg == 0 || !shape_ok(1, 8, bucket)) return 0;
    uint64_t offset = 0, buckets = 0;
    for (uint32_t t = 0; t < nseg; ++t) {
        if (sizes[t] == 0 || (t + 1 < nseg && (sizes[t] & 7u))) return 0;
        table[t].offset = offset;
        table[t].n = sizes[t];
        table[t].first_bucket = buckets;
        offset += sizes[t];
        buckets += ceil_div(sizes[t], (uint64_t)bucket);
    }
    return buckets;
}

int qsdp_quantize_grad_segmented(const float* g, const qsdp_segment* table, uint32_t nseg,
                                 uint64_t total_buckets, int bits, int bucket, uint64_t seed,
                                 uint64_t index_offset, uint32_t* codes, float* meta, void* stream) {
    if (!g || !table || nseg == 0 || total_buckets < nseg || !codes || !meta || !shape_ok(1, bits, bucket) ||
        (index_offset & 7u))
        return QSDP_EINVAL;
    if (!aligned16(g) || !aligned16(codes) || !aligned16(meta) || (reinterpret_cast<uintptr_t>(table) & 7u))
        return QSDP_EALIGN;
    Params p = {};
    set_common(p, 0, bucket, seed, index_offset, 0.0f);
    p.segs = reinterpret_cast<const Segment*>(table);
    p.nseg = nseg;
    p.num_buckets = total_buckets;
    p.g = g;
    p.codes = codes;
    p.meta = meta;
    p.gbits = bits;
    p.wbits = bits;
    return run(MODE_GRAD, p, bits, static_cast<hipStream_t>(stream));
}

int qsdp_quantize_weight_segmented(const float* x, const qsdp_segment* table, uint32_t nseg,
                                   uint64_t total_buckets, int bits, int bucket, float delta,
                                   uint64_t seed, uint32_t* codes, float* meta, uint64_t* n_saturated,
                                   void* stream) {
    if (!x || !table || nseg == 0 || total_buckets < nseg || !codes || !meta || !shape_ok(1, bits, bucket))
        return QSDP_EINVAL;
    if (!(delta >= 0.0f) || !std::isfinite(delta)) return QSDP_EINVAL;
    if (!aligned16(x) || !aligned16(codes) || !aligned16(meta) || (reinterpret_cast<uintptr_t>(table) & 7u))
        return QSDP_EALIGN;
    if (n_saturated && (reinterpret_cast<uintptr_t>(n_saturated) & 7u)) return QSDP_EALIGN;
    Params p = {};
    set_common(p, 0, bucket, seed, 0, delta);
    p.segs = reinterpret_cast<const Segment*>(table);
    p.nseg = nseg;
    p.num_buckets = total_buckets;
    p.xin = x;
    p.codes = codes;
    p.meta = meta;
    p.n_saturated = reinterpret_cast<unsigned long long*>(n_saturated);
    p.gbits = bits;
    p.wbits = bits;
    return run(MODE_WEIGHT, p, bits, static_cast<hipStream_t>(stream));
}

int qsdp_fused_step_segmented(float* x, const float* g, const qsdp_segment* table, uint32_t nseg,
                              uint64_t total_buckets, float lr, int wbits, int gbits, int bucket,
                              float delta, uint64_t seed, uint64_t index_offset, uint32_t* wcodes,
                              float* wmeta, uint64_t* n_saturated, void* stream) {
    if (!table) return QSDP_EINVAL;
    qsdp_step_options o = options_for(0u, wcodes, wmeta, n_saturated);
    set_segment_options(o, table, nseg, total_buckets);
    return qsdp_fused_step_opts(x, g, 0, lr, wbits, gbits, bucket, delta, seed, index_offset, &o, stream);
}

int qsdp_quantize_levels_segmented(const float* v, const qsdp_segment* table, uint32_t nseg,
                                   uint64_t total_buckets, int bits, int bucket, const float* levels,
                                   int stochastic, uint64_t seed, uint64_t index_offset, uint32_t* codes,
                                   float* meta, void* stream) {
    if (!v || !levels || !codes || !meta || !table || nseg == 0 || total_buckets < nseg || !shape_ok(1, bits, bucket))
        return QSDP_EINVAL;
    if ((stochastic != 0 && stochastic != 1) || (index_offset & 7u)) return QSDP_EINVAL;
    if (!aligned16(v) || !aligned16(codes) || !aligned16(meta) || (reinterpret_cast<uintptr_t>(table) & 7u) ||
        (reinterpret_cast<uintptr_t>(levels) & 3u))
        return QSDP_EALIGN;
    Params p = {};
    set_common(p, 0, bucket, seed, index_offset, 0.0f);
    p.segs = reinterpret_cast<const Segment*>(table);
    p.nseg = nseg;
    p.num_buckets = total_buckets;
    p.flags = stochastic ? FLAG_LEVELS_STOCHASTIC : 0u;
    p.xin = v;
    p.levels = levels;
    p.levels_per_tensor = 1u;
    p.codes = codes;
    p.meta = meta;
    p.gbits = bits;
    p.wbits = bits;
    return run(stochastic ? MODE_LEVELS_COIN : MODE_LEVELS, p, bits, static_cast<hipStream_t>(stream));
}

static int dequantize_segmented_common(const float* levels, const uint32_t* codes, const float* meta,
                                       const qsdp_segment* table, uint32_t nseg, uint64_t total_buckets, int bits,
                                       int bucket, qsdp_dtype out_dtype, void* out, void* stream) {
    if (!codes || !meta || !table || !out || nseg == 0 || total_buckets < nseg || !shape_ok(1, bits, bucket))
        return QSDP_EINVAL;
    if (out_dtype != QSDP_F32 && out_dtype != QSDP_BF16 && out_dtype != QSDP_F16) return QSDP_EINVAL;
    if (total_buckets >= (1ull << 37) / (uint64_t)bucket) return QSDP_EINVAL;  // 32-bit bucket indexing
    if (!aligned16(codes) || !aligned16(meta) || !aligned16(out) || (reinterpret_cast<uintptr_t>(table) & 7u))
        return QSDP_EALIGN;
    unsigned grid = 0;
    DequantSegParams q = {};
    q.d = decoder_params(codes, meta, total_buckets * (uint64_t)bucket, bits, bucket, out_dtype != QSDP_F32, out,
                         &grid);
    q.d.out_f16 = out_dtype == QSDP_F16 ? 1u : 0u;
    q.d.levels = levels;
    q.segs = reinterpret_cast<const Segment*>(table);
    q.nseg = nseg;
    if (launch_dequant_seg(bits, out_dtype != QSDP_F32, q, grid, static_cast<hipStream_t>(stream)) != hipSuccess)
        return QSDP_ELAUNCH;
    return QSDP_OK;
}

int qsdp_dequantize_segmented(const uint32_t* codes, const float* meta, const qsdp_segment* table,
                              uint32_t nseg, uint64_t total_buckets, int bits, int bucket,
                              qsdp_dtype out_dtype, void* out, void* stream) {
    return dequantize_segmented_common(nullptr, codes, meta, table, nseg, total_buckets, bits, bucket, out_dtype, out,
                                       stream);
}

int qsdp_dequantize_levels_segmented(const uint32_t* codes, const float* meta, const qsdp_segment* table,
                                     uint32_t nseg, uint64_t total_buckets, int bits, int bucket,
                                     const float* levels, qsdp_dtype out_dtype, void* out, void* stream) {
    if (!levels) return QSDP_EINVAL;
    if (reinterpret_cast<uintptr_t>(levels) & 3u) return QSDP_EALIGN;
    return dequantize_segmented_common(levels, codes, meta, table, nseg, total_buckets, bits, bucket, out_dtype, out,
                                       stream);
}

static int dequantize_gathered_common(const float* levels, const uint32_t* codes, uint64_t codes_stride_bytes,
                                      const float* meta, uint64_t meta_stride_bytes, int npeers, uint64_t n,
                                      uint64_t shard, int bits, int bucket, qsdp_dtype out_dtype, void* out,
                                      void* stream) {
    if (!codes || !meta || !out || !shape_ok(n, bits, bucket) || npeers < 1 || npeers > 65535) return QSDP_EINVAL;
    if (out_dtype != QSDP_F32 && out_dtype != QSDP_BF16 && out_dtype != QSDP_F16) return QSDP_EINVAL;
    if (shard == 0 || shard % (uint64_t)bucket != 0 || ceil_div(n, shard) != (uint64_t)npeers) return QSDP_EINVAL;
    if (shard >= (1ull << 37)) return QSDP_EINVAL;
    if ((codes_stride_bytes & 15u) || (meta_stride_bytes & 15u)) return QSDP_EALIGN;
    if (!aligned16(codes) || !aligned16(meta) || !aligned16(out)) return QSDP_EALIGN;
    const uint64_t first = npeers > 1 ? shard : n;  // elements of every slot but the last
    if (npeers > 1 && (codes_stride_bytes < qsdp_codes_bytes(shard, bits, bucket) ||
                       meta_stride_bytes < qsdp_meta_bytes(shard, bucket)))
        return QSDP_EINVAL;
    const bool bf16 = out_dtype != QSDP_F32;  // a 2-byte output format
    unsigned grid = 0, grid_last = 0;
    DequantParams p = decoder_params(codes, meta, first, bits, bucket, bf16, out, &grid);
    const DequantParams last = decoder_params(codes, meta, n - (uint64_t)(npeers - 1) * shard, bits, bucket, bf16, out,
                                              &grid_last);
    p.n_last = last.n;
    p.nwords_last = last.nwords;
    p.ntiles_last = last.ntiles;
    p.codes_stride_words = codes_stride_bytes / 4;
    p.meta_stride_floats = meta_stride_bytes / 4;
    p.levels = levels;
    p.out_f16 = out_dtype == QSDP_F16 ? 1u : 0u;
    if (launch_dequant(bits, bf16, p, dim3(grid, (unsigned)npeers), static_cast<hipStream_t>(stream)) != hipSuccess)
        return QSDP_ELAUNCH;
    return QSDP_OK;
}

int qsdp_dequantize_gathered(const uint32_t* codes, uint64_t codes_stride_bytes, const float* meta,
                             uint64_t meta_stride_bytes, int npeers, uint64_t n, uint64_t shard, int bits,
                             int bucket, qsdp_dtype out_dtype, void* out, void* stream) {
    return dequantize_gathered_common(nullptr, codes, codes_stride_bytes, meta, meta_stride_bytes, npeers, n, shard,
                                      bits, bucket, out_dtype, out, stream);
}

int qsdp_dequantize_levels_gathered(const uint32_t* codes, uint64_t codes_stride_bytes, const float* meta,
                                    uint64_t meta_stride_bytes, int npeers, uint64_t n, uint64_t shard, int bits,
                                    int bucket, const float* levels, qsdp_dtype out_dtype, void* out,
                                    void* stream) {
    if (!levels) return QSDP_EINVAL;
    if (reinterpret_cast<uintptr_t>(levels) & 3u) return QSDP_EALIGN;
    return dequantize_gathered_common(levels, codes, codes_stride_bytes, meta, meta_stride_bytes, npeers, n, shard,
                                      bits, bucket, out_dtype, out, stream);
}

static int recv_step_common(const AdamScalars* adam, const SegmentTable* segs, float* x, const uint32_t* gcodes,
                            uint64_t gcodes_stride_bytes,
                            const float* gmeta, uint64_t gmeta_stride_bytes, int npeers, uint64_t n, float alpha,
                            float lr, int wbits, int gbits, int bucket, float delta, uint64_t seed, uint32_t flags,
                            uint32_t* wcodes, float* wmeta, uint64_t* n_saturated, void* stream) {
    if (segs) {  // multi-tensor call: the slots of all buckets count as the "vector" for the size checks
        const int rc = segments_ok(*segs, bucket, &n);
        if (rc != QSDP_OK) return rc;
    }
    if (!x || !gcodes || !gmeta || npeers < 1 || !shape_ok(n, wbits, bucket) || !shape_ok(n, gbits, bucket) ||
        (flags & ~(uint32_t)(QSDP_FLAG_NO_SHIFT | QSDP_FLAG_SYMMETRIC | QSDP_FLAG_KEEP_MASTER)))
        return QSDP_EINVAL;
    if (!(delta >= 0.0f) || !std::isfinite(delta) || !std::isfinite(lr) || !std::isfinite(alpha)) return QSDP_EINVAL;
    if ((wcodes == nullptr) != (wmeta == nullptr)) return QSDP_EINVAL;
    if (npeers > 1 && (gcodes_stride_bytes < qsdp_codes_bytes(n, gbits, bucket) ||
                       gmeta_stride_bytes < qsdp_meta_bytes(n, bucket)))
        return QSDP_EINVAL;
    if (adam && !adam_ok(*adam)) return QSDP_EINVAL;
    if ((gcodes_stride_bytes & 15u) || (gmeta_stride_bytes & 3u)) return QSDP_EALIGN;
    if (!aligned16(x) || !aligned16(gcodes) || !aligned16(wcodes) || !aligned16(wmeta) ||
        (reinterpret_cast<uintptr_t>(gmeta) & 3u))
        return QSDP_EALIGN;
    if (adam && (!aligned16(adam->m) || !aligned16(adam->v))) return QSDP_EALIGN;
    if (n_saturated && (reinterpret_cast<uintptr_t>(n_saturated) & 7u)) return QSDP_EALIGN;
    Params p = {};
    set_common(p, segs ? 0 : n, bucket, seed, 0, delta);
    if (segs) set_segments(p, *segs);
    p.flags = flags;
    p.x = x;
    p.peer_codes = gcodes;
    p.peer_meta = gmeta;
    p.peer_codes_stride_words = gcodes_stride_bytes / 4;
    p.peer_meta_stride_floats = gmeta_stride_bytes / 4;
    p.npeers = npeers;
    p.alpha = alpha;
    p.codes = wcodes;
    p.meta = wmeta;
    p.n_saturated = reinterpret_cast<unsigned long long*>(n_saturated);
    p.gbits = gbits;
    p.wbits = wbits;
    p.lr = lr;
    if (adam) set_adam(p, *adam);
    return run(adam ? MODE_RECV_ADAMW : MODE_RECV, p, wcodes ? wbits : 0, static_cast<hipStream_t>(stream));
}

int qsdp_recv_step(float* x, const uint32_t* gcodes, uint64_t gcodes_stride_bytes, const float* gmeta,
                   uint64_t gmeta_stride_bytes, int npeers, uint64_t n, float alpha, float lr, int wbits,
                   int gbits, int bucket, float delta, uint64_t seed, uint32_t flags, uint32_t* wcodes,
                   float* wmeta, uint64_t* n_saturated, void* stream) {
    return recv_step_common(nullptr, nullptr, x, gcodes, gcodes_stride_bytes, gmeta, gmeta_stride_bytes, npeers, n, alpha,
                            lr,
                            wbits, gbits, bucket, delta, seed, flags, wcodes, wmeta, n_saturated, stream);
}

int qsdp_recv_adamw_step(float* x, float* m, float* v, const uint32_t* gcodes, uint64_t gcodes_stride_bytes,
                         const float* gmeta, uint64_t gmeta_stride_bytes, int npeers, uint64_t n, float alpha,
                         float lr, float beta1, float beta2, float eps, float weight_decay, float bias1,
                         float bias2, int wbits, int gbits, int bucket, float delta, uint64_t seed,
                         uint32_t flags, uint32_t* wcodes, float* wmeta, uint64_t* n_saturated, void* stream) {
    const AdamScalars adam = {m, v, beta1, beta2, eps, weight_decay, bias1, bias2};
    return recv_step_common(&adam, nullptr, x, gcodes, gcodes_stride_bytes, gmeta, gmeta_stride_bytes, npeers, n, alpha,
                            lr,
                            wbits, gbits, bucket, delta, seed, flags, wcodes, wmeta, n_saturated, stream);
}

int qsdp_recv_step_segmented(float* x, const qsdp_segment* table, uint32_t nseg, uint64_t total_buckets,
                             const uint32_t* gcodes, uint64_t gcodes_stride_bytes, const float* gmeta,
                             uint64_t gmeta_stride_bytes, int npeers, float alpha, float lr, int wbits, int gbits,
                             int bucket, float delta, uint64_t seed, uint32_t flags, uint32_t* wcodes,
                             float* wmeta, uint64_t* n_saturated, void* stream) {
    const SegmentTable segs = {table, nseg, total_buckets};
    return recv_step_common(nullptr, &segs, x, gcodes, gcodes_stride_bytes, gmeta, gmeta_stride_bytes, npeers, 0, alpha,
                            lr, wbits, gbits, bucket, delta, seed, flags, wcodes, wmeta, n_saturated, stream);
}

int qsdp_recv_adamw_step_segmented(float* x, float* m, float* v, const qsdp_segment* table, uint32_t nseg,
                                   uint64_t total_buckets, const uint32_t* gcodes, uint64_t gcodes_stride_bytes,
                                   const float* gmeta, uint64_t gmeta_stride_bytes, int npeers, float alpha,
                                   float lr, float beta1, float beta2, float eps, float weight_decay,
                                   float bias1, float bias2, int wbits, int gbits, int bucket, float delta,
                                   uint64_t seed, uint32_t flags, uint32_t* wcodes, float* wmeta,
                                   uint64_t* n_saturated, void* stream) {
    const AdamScalars adam = {m, v, beta1, beta2, eps, weight_decay, bias1, bias2};
    const SegmentTable segs = {table, nseg, total_buckets};
    return recv_step_common(&adam, &segs, x, gcodes, gcodes_stride_bytes, gmeta, gmeta_stride_bytes, npeers, 0, alpha,
                            lr, wbits, gbits, bucket, delta, seed, flags, wcodes, wmeta, n_saturated, stream);
}

}  // extern "C"
