// Test-only shim: exposes the Philox4x32 engine that ships in PyTorch's public
// headers (a third-party implementation of the published generator) through a
// C symbol, so the CPU oracle's Philox can be pinned against it.
#include <ATen/core/PhiloxRNGEngine.h>
#include <cstdint>

extern "C" void aten_philox_words(uint64_t seed, uint64_t subsequence, uint64_t offset,
                                  uint32_t n, uint32_t* out) {
    at::Philox4_32 eng(seed, subsequence, offset);
    for (uint32_t i = 0; i < n; ++i) out[i] = eng();
}
