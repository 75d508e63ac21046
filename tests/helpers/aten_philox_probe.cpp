// Test-only helper: exposes PyTorch's own host-side Philox4x32-10 engine (an implementation
// written by other people) so that the oracle's and the library's generators can be checked
// against it.  Never linked into the product or the oracle.
#include <ATen/core/PhiloxRNGEngine.h>
#include <cstdint>

extern "C" void aten_philox4x32_10(uint64_t seed, uint64_t subsequence, uint64_t offset,
                                   uint32_t out[4])
{
    // counter = (offset low, offset high, subsequence low, subsequence high), key = seed.
    at::Philox4_32 engine(seed, subsequence, offset);
    for (int i = 0; i < 4; ++i)
        out[i] = engine();
}
