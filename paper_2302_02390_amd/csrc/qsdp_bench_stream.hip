// Benchmark support, not part of the codec's ABI: plain streaming kernels with the fused step's
// access pattern (a wave owns a contiguous 4 KiB tile of each operand and moves it as four
// 16-byte non-temporal accesses per lane, one contiguous KiB per instruction) and next to no
// arithmetic. They measure what this memory system sustains for a given mix of reads and writes,
// the ceiling a codec kernel with the same traffic can be held against:
//   read         one operand read                      (4 B per element)
//   fill         one operand written                   (4 B per element)
//   copy         one read, one written                 (8 B per element)
//   axpy         x <- x - lr*g: two read, one written  (12 B per element, the fused step's mix)
//   moments      m <- b*m + g, v <- b*v + g*g, x <- x - lr*m: four read, three written (28 B per
//                element, the AdamW step's mix; three fused multiply-adds per element, no division)
//   encode       one read, `bits`/8 B written per element with the encoders' store shape (the lanes
//                that hold a 16-byte piece of the wave's code tile store it): the encoders' mix
// All take device pointers (16-byte aligned), n a multiple of 1024, a hipStream_t as void*;
// return 0, or -1 for a bad argument, -3 if the launch was refused. Built into libqsdp_bench.so.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef float f4 __attribute__((ext_vector_type(4)));
constexpr int kRows = 4;          // 16-byte rows per lane
constexpr int kTile = 64 * 4 * kRows;  // elements per wave

__device__ __forceinline__ uint64_t wave_tile() {
    return (uint64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
}

__global__ void __launch_bounds__(256) read_kernel(const float* __restrict__ a, uint64_t ntiles, float* sink) {
    const uint64_t t = wave_tile();
    if (t >= ntiles) return;
    const f4* p = reinterpret_cast<const f4*>(a + t * kTile) + (threadIdx.x & 63);
    f4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int r = 0; r < kRows; ++r) acc += __builtin_nontemporal_load(p + r * 64);
    // never true for finite data of the benchmark's scale; keeps the loads alive
    if (acc[0] + acc[1] + acc[2] + acc[3] == 0x1p120f) sink[0] = acc[0];
}

__global__ void __launch_bounds__(256) fill_kernel(float* a, uint64_t ntiles, float v) {
    const uint64_t t = wave_tile();
    if (t >= ntiles) return;
    f4* p = reinterpret_cast<f4*>(a + t * kTile) + (threadIdx.x & 63);
    const f4 w = {v, v, v, v};
#pragma unroll
    for (int r = 0; r < kRows; ++r) __builtin_nontemporal_store(w, p + r * 64);
}

__global__ void __launch_bounds__(256) copy_kernel(const float* __restrict__ a, float* __restrict__ b, uint64_t ntiles) {
    const uint64_t t = wave_tile();
    if (t >= ntiles) return;
    const f4* p = reinterpret_cast<const f4*>(a + t * kTile) + (threadIdx.x & 63);
    f4* q = reinterpret_cast<f4*>(b + t * kTile) + (threadIdx.x & 63);
    f4 v[kRows];
#pragma unroll
    for (int r = 0; r < kRows; ++r) v[r] = __builtin_nontemporal_load(p + r * 64);
#pragma unroll
    for (int r = 0; r < kRows; ++r) __builtin_nontemporal_store(v[r], q + r * 64);
}

__global__ void __launch_bounds__(256) axpy_kernel(float* x, const float* __restrict__ g, uint64_t ntiles, float lr) {
    const uint64_t t = wave_tile();
    if (t >= ntiles) return;
    f4* px = reinterpret_cast<f4*>(x + t * kTile) + (threadIdx.x & 63);
    const f4* pg = reinterpret_cast<const f4*>(g + t * kTile) + (threadIdx.x & 63);
    f4 gv[kRows], xv[kRows];
#pragma unroll
    for (int r = 0; r < kRows; ++r) gv[r] = __builtin_nontemporal_load(pg + r * 64);
#pragma unroll
    for (int r = 0; r < kRows; ++r) xv[r] = __builtin_nontemporal_load(px + r * 64);
#pragma unroll
    for (int r = 0; r < kRows; ++r) {
        f4 y;
#pragma unroll
        for (int i = 0; i < 4; ++i) y[i] = fmaf(-lr, gv[r][i], xv[r][i]);
        __builtin_nontemporal_store(y, px + r * 64);
    }
}

__global__ void __launch_bounds__(256) moments_kernel(float* x, const float* __restrict__ g, float* m, float* v,
                                                      uint64_t ntiles, float lr, float b) {
    const uint64_t t = wave_tile();
    if (t >= ntiles) return;
    const uint64_t at = t * kTile;
    const int lane = threadIdx.x & 63;
    f4* px = reinterpret_cast<f4*>(x + at) + lane;
    f4* pm = reinterpret_cast<f4*>(m + at) + lane;
    f4* pv = reinterpret_cast<f4*>(v + at) + lane;
    const f4* pg = reinterpret_cast<const f4*>(g + at) + lane;
    f4 gv[kRows], xv[kRows], mv[kRows], vv[kRows];
#pragma unroll
    for (int r = 0; r < kRows; ++r) gv[r] = __builtin_nontemporal_load(pg + r * 64);
#pragma unroll
    for (int r = 0; r < kRows; ++r) xv[r] = __builtin_nontemporal_load(px + r * 64);
#pragma unroll
    for (int r = 0; r < kRows; ++r) mv[r] = __builtin_nontemporal_load(pm + r * 64);
#pragma unroll
    for (int r = 0; r < kRows; ++r) vv[r] = __builtin_nontemporal_load(pv + r * 64);
#pragma unroll
    for (int r = 0; r < kRows; ++r) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            mv[r][i] = fmaf(b, mv[r][i], gv[r][i]);
            vv[r][i] = fmaf(b, vv[r][i], gv[r][i] * gv[r][i]);
            xv[r][i] = fmaf(-lr, mv[r][i], xv[r][i]);
        }
        __builtin_nontemporal_store(mv[r], pm + r * 64);
        __builtin_nontemporal_store(vv[r], pv + r * 64);
        __builtin_nontemporal_store(xv[r], px + r * 64);
    }
}

typedef uint32_t u4 __attribute__((ext_vector_type(4)));

// pieces = 16-byte pieces of output per wave tile (32 for 4-bit codes, 64 for 8-bit codes)
__global__ void __launch_bounds__(256) encode_kernel(const float* __restrict__ a, u4* out, uint64_t ntiles, int pieces) {
    const uint64_t t = wave_tile();
    if (t >= ntiles) return;
    const int lane = threadIdx.x & 63;
    const f4* p = reinterpret_cast<const f4*>(a + t * kTile) + lane;
    u4 w;
#pragma unroll
    for (int r = 0; r < kRows; ++r) {
        const f4 v = __builtin_nontemporal_load(p + r * 64);
        w[r] = __float_as_uint(v[0]) ^ __float_as_uint(v[1]) ^ __float_as_uint(v[2]) ^ __float_as_uint(v[3]);
    }
    // every lane's loads feed a stored piece: with fewer pieces than lanes the upper lanes' words are
    // folded into the lower lanes' (otherwise their loads would be dead code)
    if (pieces < 64) {
#pragma unroll
        for (int r = 0; r < kRows; ++r) w[r] ^= (uint32_t)__shfl_xor((int)w[r], 32, 64);
    }
    if (lane < pieces) __builtin_nontemporal_store(w, out + t * (uint64_t)pieces + lane);
}

bool ok(const void* p, uint64_t n) {
    return p != nullptr && (reinterpret_cast<uintptr_t>(p) & 15u) == 0 && n >= (uint64_t)kTile && n % kTile == 0 &&
           n / kTile / 4 + 1 < (1ull << 31);
}

unsigned grid_for(uint64_t n) { return (unsigned)((n / kTile + 3) / 4); }

}  // namespace

extern "C" {

int qsdp_bench_read(const float* a, uint64_t n, float* sink, void* stream) {
    if (!ok(a, n) || sink == nullptr) return -1;
    hipLaunchKernelGGL(read_kernel, dim3(grid_for(n)), dim3(256), 0, static_cast<hipStream_t>(stream), a, n / kTile, sink);
    return hipGetLastError() == hipSuccess ? 0 : -3;
}

int qsdp_bench_fill(float* a, uint64_t n, float v, void* stream) {
    if (!ok(a, n)) return -1;
    hipLaunchKernelGGL(fill_kernel, dim3(grid_for(n)), dim3(256), 0, static_cast<hipStream_t>(stream), a, n / kTile, v);
    return hipGetLastError() == hipSuccess ? 0 : -3;
}

int qsdp_bench_copy(const float* a, float* b, uint64_t n, void* stream) {
    if (!ok(a, n) || !ok(b, n)) return -1;
    hipLaunchKernelGGL(copy_kernel, dim3(grid_for(n)), dim3(256), 0, static_cast<hipStream_t>(stream), a, b, n / kTile);
    return hipGetLastError() == hipSuccess ? 0 : -3;
}

// resident_cap_lds: bytes of dynamic LDS requested and never touched, which caps the workgroups resident per
// compute unit (the codec's step kernels are launched that way; 0 = no cap)
int qsdp_bench_axpy(float* x, const float* g, uint64_t n, float lr, unsigned resident_cap_lds, void* stream) {
    if (!ok(x, n) || !ok(g, n) || resident_cap_lds > 65536u) return -1;
    hipLaunchKernelGGL(axpy_kernel, dim3(grid_for(n)), dim3(256), resident_cap_lds, static_cast<hipStream_t>(stream), x, g,
                       n / kTile, lr);
    return hipGetLastError() == hipSuccess ? 0 : -3;
}

int qsdp_bench_moments(float* x, const float* g, float* m, float* v, uint64_t n, float lr, float b,
                       unsigned resident_cap_lds, void* stream) {
    if (!ok(x, n) || !ok(g, n) || !ok(m, n) || !ok(v, n) || resident_cap_lds > 65536u) return -1;
    hipLaunchKernelGGL(moments_kernel, dim3(grid_for(n)), dim3(256), resident_cap_lds, static_cast<hipStream_t>(stream),
                       x, g, m, v, n / kTile, lr, b);
    return hipGetLastError() == hipSuccess ? 0 : -3;
}

int qsdp_bench_encode(const float* a, uint64_t n, int bits, uint32_t* out, void* stream) {
    if (!ok(a, n) || out == nullptr || (reinterpret_cast<uintptr_t>(out) & 15u) != 0 || (bits != 4 && bits != 8)) return -1;
    hipLaunchKernelGGL(encode_kernel, dim3(grid_for(n)), dim3(256), 0, static_cast<hipStream_t>(stream), a,
                       reinterpret_cast<u4*>(out), n / kTile, bits * 8);
    return hipGetLastError() == hipSuccess ? 0 : -3;
}

}  // extern "C"
