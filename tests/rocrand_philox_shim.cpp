// Host-side shim around rocRAND's own Philox4x32-10 engine (a __host__ __device__ class in the library's
// public header): the reference the oracle's generator is pinned against.  Built with g++ by the test; no GPU
// call is made.  seed -> key, subsequence -> the two high counter words, offset / 4 -> the two low counter words.
#include <hip/hip_runtime.h>
#include <rocrand/rocrand_philox4x32_10.h>
#include <stdint.h>

extern "C" void shim_philox_next4(uint64_t seed, uint64_t subsequence, uint64_t offset, uint32_t out[4]) {
    rocrand_device::philox4x32_10_engine engine(seed, subsequence, offset);
    for (int i = 0; i < 4; ++i) out[i] = engine.next();
}
