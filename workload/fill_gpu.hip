// Device helpers of the workload package: the stateless pool fill, and two measurement probes
// (matrix cores alone; a read-only stream) whose results bench.py reports as measured ceilings.
// Nothing of the migration or of the linear layer itself lives here.
//
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

// ---- measurement probes (ceilings that bench.py reports beside the nominal peaks) ----

typedef __bf16 wl_bf16x8 __attribute__((ext_vector_type(8)));
typedef float wl_f32x16 __attribute__((ext_vector_type(16)));

// Matrix cores alone: every wavefront keeps a 128 x 128 accumulator tile (4 x 4 MFMA tiles of 32 x 32,
// the register shape of a 256 x 256 workgroup tile) and issues `iters` rounds of the 16
// v_mfma_f32_32x32x16_bf16 of one k step on operands that stay in registers: no LDS, no memory.
// Operands are pseudo-random bf16 values in (-2, 2): the clock the chip sustains depends on the data.
__global__ __launch_bounds__(256) void wl_mfma_probe_kernel(float *out, uint32_t iters, uint64_t state0)
{
    wl_bf16x8 a[4], b[4];
    const uint64_t lane_key = state0 + (uint64_t(blockIdx.x) * 256u + threadIdx.x) * 64u;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const uint64_t ra = wl_mix64(lane_key + uint64_t(i * 8 + e)), rb = wl_mix64(lane_key + 32u + uint64_t(i * 8 + e));
            // sign, exponent 126..127 (values in [0.5, 2)), 7 random mantissa bits
            const uint16_t ba = uint16_t(((ra & 1u) << 15) | ((126u + ((ra >> 1) & 1u)) << 7) | ((ra >> 2) & 0x7fu));
            const uint16_t bb = uint16_t(((rb & 1u) << 15) | ((126u + ((rb >> 1) & 1u)) << 7) | ((rb >> 2) & 0x7fu));
            a[i][e] = __builtin_bit_cast(__bf16, ba);
            b[i][e] = __builtin_bit_cast(__bf16, bb);
        }
    wl_f32x16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    for (uint32_t it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[j], a[i], acc[i][j], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) s += acc[i][j][v];
    out[uint64_t(blockIdx.x) * 256u + threadIdx.x] = s;
}

// Read-only stream: eight independent 16-byte non-temporal loads per lane (8 KiB per wavefront-sized
// workgroup; with a single load per lane the wavefront launch rate, not HBM, sets the pace); the
// xor keeps the loads alive, and practically nothing is written.
typedef uint32_t wl_u32x4 __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(64) void wl_read_probe_kernel(const wl_u32x4 *__restrict__ src, uint32_t n_vec,
                                                           uint32_t *__restrict__ sink)
{
    const uint32_t base = blockIdx.x * 512u + threadIdx.x;
    wl_u32x4 x[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        const uint32_t i = base + 64u * uint32_t(k);
        x[k] = i < n_vec ? __builtin_nontemporal_load(src + i) : wl_u32x4{0u, 0u, 0u, 0u};
    }
    uint32_t h = 0;
#pragma unroll
    for (int k = 0; k < 8; ++k) h ^= x[k][0] ^ x[k][1] ^ x[k][2] ^ x[k][3];
    if (h == 0x9E3779B9u) sink[blockIdx.x & 1023u] = h;        // practically never taken
}

}  // namespace

extern "C" {

// Runs the matrix-core probe: n_workgroups of 256 threads, `iters` k steps each; out: device,
// n_workgroups * 256 floats.  Flop count = n_workgroups * 4 wavefronts * iters * 16 * 32768.
int wl_mfma_probe(void *out, uint32_t n_workgroups, uint32_t iters, uint64_t state0, void *stream)
{
    if (n_workgroups == 0) return 0;
    hipLaunchKernelGGL(wl_mfma_probe_kernel, dim3(n_workgroups), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<float *>(out), iters, state0);
    return int(hipGetLastError());
}

// Reads n_bytes (a multiple of 16, below 2^35) from src once; sink: device, 1024 uint32.
int wl_read_probe(const void *src, uint64_t n_bytes, void *sink, void *stream)
{
    const uint64_t n_vec = n_bytes / 16;
    if (n_vec == 0 || n_vec >= (uint64_t(1) << 31)) return int(hipErrorInvalidValue);
    hipLaunchKernelGGL(wl_read_probe_kernel, dim3(unsigned((n_vec + 511) / 512)), dim3(64), 0,
                       static_cast<hipStream_t>(stream), static_cast<const wl_u32x4 *>(src), uint32_t(n_vec),
                       static_cast<uint32_t *>(sink));
    return int(hipGetLastError());
}

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
