// Host-side launch interface between the C ABI (qsdp_api.hip) and the kernel translation
// units. Wave kernels are instantiated per bucket shape in qsdp_wave_inst.hip, compiled
// once per (G, P) pair.
#pragma once

#include <hip/hip_runtime.h>

#include "qsdp_kernels.hpp"

namespace qsdp {

// Code widths the wave kernels are instantiated for (0 = a step without code output).
inline bool wave_bits_supported(int bits) { return bits >= 0 && bits <= 8; }

// One launcher per instantiated bucket size. `bits` is the width of the codes stored.
#define QSDP_DECLARE_WAVE(B) \
    hipError_t launch_wave_##B(int mode, int bits, const Params& p, unsigned grid, hipStream_t s);
QSDP_DECLARE_WAVE(128)
QSDP_DECLARE_WAVE(256)
QSDP_DECLARE_WAVE(512)
QSDP_DECLARE_WAVE(1024)
QSDP_DECLARE_WAVE(2048)
QSDP_DECLARE_WAVE(4096)
QSDP_DECLARE_WAVE(1024w2)  // weight quantizer only: two waves per 1024-bucket
#undef QSDP_DECLARE_WAVE

hipError_t launch_block(int mode, const Params& p, unsigned grid, hipStream_t s);
hipError_t launch_dequant(int bits, bool bf16, const DequantParams& p, dim3 grid, hipStream_t s);
hipError_t launch_fit_levels(const FitParams& p, unsigned grid, hipStream_t s);
hipError_t launch_dequant_add(int bits, const DequantAddParams& p, unsigned grid, hipStream_t s);

}  // namespace qsdp
