// Stateless SplitMix64 pool fill on the GPU: word k of the buffer (counted from
// start_word) receives output k of the stream with initial state state0, i.e.
// mix64(state0 + (k+1)*GAMMA).  Mirrors workload/splitmix.py; input generation
// only, nothing of the migration itself.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

__device__ __forceinline__ uint64_t wl_mix64(uint64_t z)
{
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

__global__ __launch_bounds__(256) void wl_fill_kernel(uint64_t *dst, uint64_t start_word,
                                                      uint64_t n_words, uint64_t state0)
{
    const uint64_t stride = uint64_t(gridDim.x) * blockDim.x;
    for (uint64_t i = uint64_t(blockIdx.x) * blockDim.x + threadIdx.x; i < n_words; i += stride)
        dst[i] = wl_mix64(state0 + (start_word + i + 1) * 0x9E3779B97F4A7C15ull);
}

__global__ __launch_bounds__(256) void wl_mismatch_kernel(const uint64_t *buf, uint64_t start_word,
                                                          uint64_t n_words, uint64_t state0,
                                                          unsigned long long *count)
{
    const uint64_t stride = uint64_t(gridDim.x) * blockDim.x;
    unsigned long long bad = 0;
    for (uint64_t i = uint64_t(blockIdx.x) * blockDim.x + threadIdx.x; i < n_words; i += stride)
        bad += buf[i] != wl_mix64(state0 + (start_word + i + 1) * 0x9E3779B97F4A7C15ull);
    if (bad) atomicAdd(count, bad);
}

}  // namespace

extern "C" {

// dst: device, n_words * 8 bytes.  Returns a hipError_t as int.
int wl_fill_words(void *dst, uint64_t start_word, uint64_t n_words, uint64_t state0, void *stream)
{
    if (n_words == 0) return 0;
    uint64_t blocks = (n_words + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(wl_fill_kernel, dim3((unsigned)blocks), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<uint64_t *>(dst), start_word, n_words, state0);
    return int(hipGetLastError());
}

// Adds to *count_dev (device uint64, caller zeroes it) the number of words of
// buf that differ from the fill pattern.
int wl_count_mismatch(const void *buf, uint64_t start_word, uint64_t n_words, uint64_t state0,
                      void *count_dev, void *stream)
{
    if (n_words == 0) return 0;
    uint64_t blocks = (n_words + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(wl_mismatch_kernel, dim3((unsigned)blocks), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const uint64_t *>(buf), start_word, n_words, state0,
                       static_cast<unsigned long long *>(count_dev));
    return int(hipGetLastError());
}

}  // extern "C"
