// Test helper: exposes PyTorch's own host-callable Philox4x32-10 engine
// (ATen/core/PhiloxRNGEngine.h, a library routine independent of this
// repository) through a C function, so the oracle's generator can be pinned
// against it.  key = seed, counter = (offset lo, offset hi, subseq lo, subseq hi).
#include <ATen/core/PhiloxRNGEngine.h>
#include <cstdint>
extern "C" void aten_philox4x32_10(uint64_t seed, uint64_t subsequence, uint64_t offset, uint32_t out[4])
{
    at::philox_engine eng(seed, subsequence, offset);
    for (int i = 0; i < 4; ++i) out[i] = eng();
}
