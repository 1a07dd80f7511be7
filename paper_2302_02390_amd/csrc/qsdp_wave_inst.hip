// Instantiations of the wave kernels for one bucket shape; compiled with
// -DQSDP_G=<lanes per bucket> -DQSDP_R=<rows of 4*G elements per wave> -DQSDP_W=<waves per
// bucket> -DQSDP_B=<4*G*R*W>. With -DQSDP_WEIGHT_ONLY=<name suffix> only the weight quantizer is
// instantiated, as launch_wave_<suffix> (a second shape for a bucket size that has one already).
#include "qsdp_launch.hpp"

#if !defined(QSDP_G) || !defined(QSDP_R) || !defined(QSDP_W) || !defined(QSDP_B)
#error "define QSDP_G, QSDP_R, QSDP_W and QSDP_B"
#endif
static_assert(QSDP_B == 4 * QSDP_G * QSDP_R * QSDP_W, "bucket = 4 * G * R * W");

#define QSDP_CAT2(a, b) a##b
#define QSDP_CAT(a, b) QSDP_CAT2(a, b)

namespace qsdp {
namespace {

// Dynamic LDS that a launch asks for and never touches: it only caps how many workgroups are resident on
// a compute unit (160 KB of LDS each). The streaming step kernels run faster with fewer waves in flight
// than their registers would allow (1.3B vector, same box, medians of 30: fused step 2.605-2.610 ms with
// 7 workgroups per compute unit, 2.546-2.569 with 5, 2.527-2.543 with 3; with code output 5 is best; AdamW
// step 6.45 ms with 3, 6.22-6.34 with 2); the encoders and the code-resident step, whose arithmetic has to
// overlap the memory latency, want all the waves they can get. Only for the one-wave-per-bucket shapes.
constexpr unsigned resident_cap_lds(int mode, int bits) {
    if (QSDP_W != 1) return 0u;
    if (mode == MODE_FUSED) return bits == 0 ? 50000u : 27000u;
    if (mode == MODE_ADAMW) return 60000u;
    return 0u;
}

template <int MODE, int BITS>
hipError_t go(const Params& p, unsigned grid, hipStream_t s) {
    // W == 1: 4 waves per workgroup, each on its own buckets; W > 1: W waves share a bucket
    const unsigned block = QSDP_W == 1 ? 256u : 64u * QSDP_W;
    hipLaunchKernelGGL((wave_kernel<MODE, QSDP_G, QSDP_R, BITS, QSDP_W>), dim3(grid), dim3(block),
                       resident_cap_lds(MODE, BITS), s, p, p.segs);
    return hipGetLastError();
}

template <int MODE>
hipError_t by_bits(int bits, const Params& p, unsigned grid, hipStream_t s) {
    switch (bits) {
        case 1: return go<MODE, 1>(p, grid, s);
        case 2: return go<MODE, 2>(p, grid, s);
        case 3: return go<MODE, 3>(p, grid, s);
        case 4: return go<MODE, 4>(p, grid, s);
        case 5: return go<MODE, 5>(p, grid, s);
        case 6: return go<MODE, 6>(p, grid, s);
        case 7: return go<MODE, 7>(p, grid, s);
        case 8: return go<MODE, 8>(p, grid, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

#ifdef QSDP_WEIGHT_ONLY
hipError_t QSDP_CAT(launch_wave_, QSDP_WEIGHT_ONLY)(int mode, int bits, const Params& p, unsigned grid,
                                                    hipStream_t s) {
    return mode == MODE_WEIGHT ? by_bits<MODE_WEIGHT>(bits, p, grid, s) : hipErrorInvalidValue;
}
#else
hipError_t QSDP_CAT(launch_wave_, QSDP_B)(int mode, int bits, const Params& p, unsigned grid,
                                          hipStream_t s) {
    switch (mode) {
        case MODE_GRAD: return by_bits<MODE_GRAD>(bits, p, grid, s);
        case MODE_WEIGHT: return by_bits<MODE_WEIGHT>(bits, p, grid, s);
        case MODE_FUSED:
            if (bits == 0) return go<MODE_FUSED, 0>(p, grid, s);
            return by_bits<MODE_FUSED>(bits, p, grid, s);
        case MODE_FUSED_CODES: return by_bits<MODE_FUSED_CODES>(bits, p, grid, s);
        case MODE_LEVELS: return by_bits<MODE_LEVELS>(bits, p, grid, s);
        case MODE_LEVELS_COIN: return by_bits<MODE_LEVELS_COIN>(bits, p, grid, s);
        case MODE_ADAMW:
            if (bits == 0) return go<MODE_ADAMW, 0>(p, grid, s);
            return by_bits<MODE_ADAMW>(bits, p, grid, s);
        case MODE_ADAMW_CODES: return by_bits<MODE_ADAMW_CODES>(bits, p, grid, s);
        case MODE_RECV:  // the width of the peers' codes (p.gbits) is a run-time value in these two
            if (bits == 0) return go<MODE_RECV, 0>(p, grid, s);
            return by_bits<MODE_RECV>(bits, p, grid, s);
        case MODE_SUM: return go<MODE_SUM, 0>(p, grid, s);
        case MODE_RECV_ADAMW:
            if (bits == 0) return go<MODE_RECV_ADAMW, 0>(p, grid, s);
            return by_bits<MODE_RECV_ADAMW>(bits, p, grid, s);
        default: return hipErrorInvalidValue;
    }
}
#endif

}  // namespace qsdp
