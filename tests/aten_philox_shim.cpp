// Test helper: exposes the Philox4x32-10 engine that ships in PyTorch's headers
// (an implementation independent of this repository) through a C symbol.
// key = (seed lo, seed hi); counter = (offset lo, offset hi, subsequence lo, subsequence hi).
#include <ATen/core/PhiloxRNGEngine.h>
#include <cstdint>

extern "C" void aten_philox_block(uint64_t seed, uint64_t subsequence, uint64_t offset,
                                  uint32_t* out) {
    at::Philox4_32 engine(seed, subsequence, offset);
    for (int i = 0; i < 4; ++i) out[i] = engine();
}
