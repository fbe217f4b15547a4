// TP-shard-selecting linear layer (paper Sec. 3.2.1: one full weight copy per
// GPU, the rank's 1/N shard picked at execution time).  The shard is never
// copied: a column-parallel shard is a row block of the [n_out][n_in] weight,
// a row-parallel shard a column block, so both are a base offset plus the full
// matrix's row stride, and every kernel here computes
//     Y[M][Nn] = X[M][K] . A[Nn][K]^T        (A = the shard, row stride lda)
// with 16-bit inputs (bfloat16 or float16), fp32 accumulation on the matrix cores and
// one rounding to the input format.
//
// Small batches (M <= 64, decode): the weight shard is read exactly once and
// the kernel is bound by HBM bandwidth.  A wavefront owns 16 weight rows and a
// K slice; weight rows are the A operand of v_mfma_f32_16x16x32_bf16 and go
// from global memory straight into registers (no LDS: no reuse), the batch is
// the B operand and sits in LDS.  Lane (i = lane%16, g = lane/16) of the MFMA
// holds 8 consecutive k of row i; which k they are is free as long as both
// operands agree, so inside a 64-wide k block lane group g takes k = 16g+8s+e
// for the block's two MFMAs s = 0,1: each lane then reads 32 contiguous bytes
// and the four lanes of a row cover one full 128-byte line.
#include <algorithm>

#include "nts_internal.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kSkinnyChunk = 256;          // k per LDS refill: four 64-wide blocks
constexpr int kLdsRow = kSkinnyChunk * 2 + 16;   // bytes per batch row in LDS (padded)

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return uint16_t((u >> 16) | 0x40u);   // NaN stays NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return uint16_t(u >> 16);
}

__device__ __forceinline__ uint16_t f32_to_f16_rne(float f)
{
    const _Float16 h = static_cast<_Float16>(f);      // v_cvt_f16_f32: round to nearest even
    return __builtin_bit_cast(uint16_t, h);
}

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// The two 16-bit element formats: matrix-core instructions and the final rounding.
struct Bf16 {
    typedef bf16x8 vec8;
    static __device__ __forceinline__ f32x4 mfma16(vec8 a, vec8 b, f32x4 c) { return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0); }
    static __device__ __forceinline__ f32x16 mfma32(vec8 a, vec8 b, f32x16 c) { return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0); }
    static __device__ __forceinline__ uint16_t round(float f) { return f32_to_bf16_rne(f); }
};
struct F16 {
    typedef f16x8 vec8;
    static __device__ __forceinline__ f32x4 mfma16(vec8 a, vec8 b, f32x4 c) { return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0); }
    static __device__ __forceinline__ f32x16 mfma32(vec8 a, vec8 b, f32x16 c) { return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0); }
    static __device__ __forceinline__ uint16_t round(float f) { return f32_to_f16_rne(f); }
};

// MT = number of 16-row batch tiles (M <= 16*MT); RT = 16-row weight tiles per wavefront.
// A larger RT reuses every staged X chunk and every X fragment for more weight rows, which
// is what matters once the batch is wide (MT 3..4); RT = 1 keeps more wavefronts in flight.
template <class E, int MT, int RT, int WAVES>
__global__ __launch_bounds__(WAVES * 64) void nts_linear_skinny_kernel(
    const uint16_t *__restrict__ X, int64_t ldx, const uint16_t *__restrict__ A, int64_t lda,
    uint16_t *__restrict__ Y, int64_t ldy, float *__restrict__ part, int M, int Nn, int K,
    int chunks_per_split)
{
    __shared__ __attribute__((aligned(16))) unsigned char xs[16 * MT * kLdsRow];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int i = lane & 15, g = lane >> 4;
    const int n0 = (blockIdx.x * WAVES + wv) * 16 * RT;     // first weight row of this wavefront
    const int split = blockIdx.y;
    const int n_chunks = (K + kSkinnyChunk - 1) / kSkinnyChunk;
    const int c_lo = split * chunks_per_split;
    const int c_hi = min(n_chunks, c_lo + chunks_per_split);
    const unsigned char *arow[RT];
#pragma unroll
    for (int r = 0; r < RT; ++r)                                    // clamp: rows past the end are computed, not stored
        arow[r] = reinterpret_cast<const unsigned char *>(A + int64_t(min(n0 + r * 16 + i, Nn - 1)) * lda);

    f32x4 acc[RT][MT];
#pragma unroll
    for (int r = 0; r < RT; ++r)
#pragma unroll
        for (int t = 0; t < MT; ++t) acc[r][t] = f32x4{0.f, 0.f, 0.f, 0.f};

    // weight loads run one chunk ahead of the MFMAs: 2 x 16 B per lane and 64-wide block
    u32x4 wreg[RT][8], wnext[RT][8];
#define NTS_LOAD_W(DST, chunk)                                                                        \
    {                                                                                                 \
        const int k0_ = (chunk) * kSkinnyChunk;                                                       \
        const int nblk_ = min(4, (K - k0_) / 64);                                                     \
        _Pragma("unroll") for (int r = 0; r < RT; ++r)                                                \
            _Pragma("unroll") for (int b = 0; b < 4; ++b) {                                           \
                if (b < nblk_) {                                                                      \
                    const unsigned char *p = arow[r] + (int64_t(k0_) + b * 64 + g * 16) * 2;          \
                    DST[r][2 * b] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));   \
                    DST[r][2 * b + 1] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p + 16)); \
                }                                                                                     \
            }                                                                                         \
    }
    constexpr bool kAhead = RT == 1;        // with two row tiles the second register set costs occupancy
    if (kAhead && c_lo < c_hi) NTS_LOAD_W(wnext, c_lo)
    for (int c = c_lo; c < c_hi; ++c) {
        const int k0 = c * kSkinnyChunk;
        const int nblk = min(4, (K - k0) / 64);                     // K is a multiple of 64
        if (kAhead) {
#pragma unroll
            for (int r = 0; r < RT; ++r)
#pragma unroll
                for (int q = 0; q < 8; ++q) wreg[r][q] = wnext[r][q];
            if (c + 1 < c_hi) NTS_LOAD_W(wnext, c + 1)
        } else {
            NTS_LOAD_W(wreg, c)
        }
        __syncthreads();                                            // previous chunk's LDS reads are done
        // stage X[0:16*MT][k0 : k0+256] (rows >= M and k >= K as zeros)
        for (int v = threadIdx.x; v < 16 * MT * (kSkinnyChunk / 8); v += WAVES * 64) {
            const int r = v / (kSkinnyChunk / 8), kv = v % (kSkinnyChunk / 8);
            u32x4 x = {0u, 0u, 0u, 0u};
            if (r < M && k0 + kv * 8 < K)
                x = *reinterpret_cast<const u32x4 *>(X + int64_t(r) * ldx + k0 + kv * 8);
            *reinterpret_cast<u32x4 *>(xs + r * kLdsRow + kv * 16) = x;
        }
        __syncthreads();
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            if (b < nblk) {
#pragma unroll
                for (int s = 0; s < 2; ++s) {
#pragma unroll
                    for (int t = 0; t < MT; ++t) {
                        typedef typename E::vec8 vec8;
                        const vec8 xb = __builtin_bit_cast(vec8, *reinterpret_cast<const u32x4 *>(
                            xs + (t * 16 + i) * kLdsRow + (b * 64 + g * 16 + s * 8) * 2));
#pragma unroll
                        for (int r = 0; r < RT; ++r)
                            acc[r][t] = E::mfma16(__builtin_bit_cast(vec8, wreg[r][2 * b + s]), xb, acc[r][t]);
                    }
                }
            }
        }
    }
    // D[row = g*4+v][col = i]: weight row n0 + r*16 + g*4 + v, batch row t*16 + i
#pragma unroll
    for (int r = 0; r < RT; ++r) {
        const int nb = n0 + r * 16 + g * 4;
#pragma unroll
        for (int t = 0; t < MT; ++t) {
            const int m = t * 16 + i;
            if (m < M) {
                if (part) {
                    float *dst = part + (int64_t(split) * M + m) * Nn + nb;
#pragma unroll
                    for (int v = 0; v < 4; ++v)
                        if (nb + v < Nn) dst[v] = acc[r][t][v];
                } else {
                    uint16_t *dst = Y + int64_t(m) * ldy + nb;
#pragma unroll
                    for (int v = 0; v < 4; ++v)
                        if (nb + v < Nn) dst[v] = E::round(acc[r][t][v]);
                }
            }
        }
    }
}

#undef NTS_LOAD_W

// Y[m][n] = sum over splits, in split order, rounded once
template <class E>
__global__ __launch_bounds__(256) void nts_linear_reduce_kernel(const float *__restrict__ part, int splits,
                                                                int M, int Nn, uint16_t *__restrict__ Y,
                                                                int64_t ldy)
{
    const int64_t idx = int64_t(blockIdx.x) * 256 + threadIdx.x;
    if (idx >= int64_t(M) * Nn) return;
    float s = 0.f;
    for (int k = 0; k < splits; ++k) s += part[int64_t(k) * M * Nn + idx];
    Y[(idx / Nn) * ldy + idx % Nn] = E::round(s);
}


// ---------------------------------------------------------------------------
// Large batches (M > 64, prefill): bound by the matrix cores.  A 256-thread
// workgroup computes a 256 x 256 tile of Y; each of its four wavefronts owns a
// 128 x 128 quadrant as 4 x 4 tiles of v_mfma_f32_32x32x16_bf16 (256 fp32
// accumulators per lane, one wavefront per SIMD).  X and weight rows are both
// contiguous along k, so both operands are staged the same way: 64-wide k
// slabs go global -> registers -> LDS (row pitch 144 B, which spreads the 32
// rows a ds_read_b128 touches over all banks).  LDS holds two slabs: while the
// MFMAs of slab s read one buffer, slab s+1 is written into the other and the
// global loads of slab s+2 are in flight; one barrier per slab.
constexpr int kTileM = 256, kTileN = 256, kTileK = 64;
constexpr int kSupM = 4, kSupN = 8;                     // tiles per XCD-resident block
constexpr int kPitch = kTileK * 2 + 16;                 // bytes per LDS row
constexpr int kTileLds = (kTileM + kTileN) * kPitch;    // 73728 B per buffer, two buffers of dynamic LDS

template <class E>
__global__ __launch_bounds__(256) void nts_linear_tiled_kernel(
    const uint16_t *__restrict__ X, int64_t ldx, const uint16_t *__restrict__ A, int64_t lda,
    uint16_t *__restrict__ Y, int64_t ldy, int M, int Nn, int K)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int wm = wv >> 1, wn = wv & 1;                // quadrant of this wavefront
    // Workgroup -> tile.  Consecutive workgroup ids go to the 8 XCDs in turn and each XCD has
    // its own L2, so the 32 workgroups that run together on one XCD are given a 4 x 8 block of
    // tiles: every X slab is then fetched into that L2 once for 8 tiles and every weight slab
    // once for 4, instead of each workgroup streaming a weight tile of its own.
    const int tiles_m = (M + kTileM - 1) / kTileM, tiles_n = (Nn + kTileN - 1) / kTileN;
    const int sup_n = (tiles_n + kSupN - 1) / kSupN;
    const int xcd = blockIdx.x & 7, seq = blockIdx.x >> 3;
    const int sup = (seq / (kSupM * kSupN)) * 8 + xcd, in_sup = seq % (kSupM * kSupN);
    const int tm = (sup / sup_n) * kSupM + in_sup / kSupN, tn = (sup % sup_n) * kSupN + in_sup % kSupN;
    if (tm >= tiles_m || tn >= tiles_n) return;         // whole workgroup leaves before any barrier
    const int m0 = tm * kTileM, n0 = tn * kTileN;

    // staging map: 256 rows x 8 vectors of 16 B per operand and slab; thread t takes
    // vector (t & 7) of rows (t >> 3) + 32 * q, q = 0..7: eight lanes read one 128 B line.
    // Row offsets are kept as 32-bit counts of 16-byte units from the operand's base.
    const int sv = tid & 7, sr = tid >> 3;
    uint32_t xo[8], ao[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) {
        const int r = sr + 32 * q;
        xo[q] = uint32_t((int64_t(min(m0 + r, M - 1)) * ldx) >> 3) + sv;
        ao[q] = uint32_t((int64_t(min(n0 + r, Nn - 1)) * lda) >> 3) + sv;
    }
    const u32x4 *xb = reinterpret_cast<const u32x4 *>(X), *ab = reinterpret_cast<const u32x4 *>(A);

    f32x16 acc[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

    const int fr = lane & 31, fg = lane >> 5;           // fragment row and k group of this lane
    const int n_slabs = K / kTileK;
    const int st_off = sr * kPitch + sv * 16;           // where this thread's staged vectors go

    // prologue: slab 0 into LDS buffer 0, slab 1 into registers
    u32x4 xr[8], ar[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) {
        xr[q] = xb[xo[q]];
        ar[q] = ab[ao[q]];
    }
#pragma unroll
    for (int q = 0; q < 8; ++q) {
        *reinterpret_cast<u32x4 *>(lds + st_off + 32 * q * kPitch) = xr[q];
        *reinterpret_cast<u32x4 *>(lds + kTileM * kPitch + st_off + 32 * q * kPitch) = ar[q];
    }
    if (n_slabs > 1) {
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            xr[q] = xb[xo[q] + kTileK * 2 / 16];
            ar[q] = ab[ao[q] + kTileK * 2 / 16];
        }
    }
    __syncthreads();

    // fragments of k step kk+1 are read from LDS while the MFMAs of step kk run
#define NTS_LOAD_FRAGS(kk, XF, AF)                                                                     \
    {                                                                                                  \
        _Pragma("unroll") for (int a = 0; a < 4; ++a)                                                  \
            XF[a] = __builtin_bit_cast(vec8, *reinterpret_cast<const u32x4 *>(                       \
                xs + (wm * 128 + a * 32 + fr) * kPitch + ((kk) * 16 + fg * 8) * 2));                   \
        _Pragma("unroll") for (int b = 0; b < 4; ++b)                                                  \
            AF[b] = __builtin_bit_cast(vec8, *reinterpret_cast<const u32x4 *>(                       \
                as + (wn * 128 + b * 32 + fr) * kPitch + ((kk) * 16 + fg * 8) * 2));                   \
    }
#define NTS_MFMAS(XF, AF)                                                                              \
    {                                                                                                  \
        _Pragma("unroll") for (int a = 0; a < 4; ++a)                                                  \
            _Pragma("unroll") for (int b = 0; b < 4; ++b)                                              \
                acc[a][b] = E::mfma32(XF[a], AF[b], acc[a][b]);                                       \
    }

    for (int s = 0; s < n_slabs; ++s) {
        const unsigned char *xs = lds + (s & 1) * kTileLds, *as = xs + kTileM * kPitch;
        unsigned char *nx = lds + ((s + 1) & 1) * kTileLds;
        typedef typename E::vec8 vec8;
        vec8 xf0[4], af0[4], xf1[4], af1[4];
        NTS_LOAD_FRAGS(0, xf0, af0)
        NTS_LOAD_FRAGS(1, xf1, af1)
        NTS_MFMAS(xf0, af0)
        // slab s+1 (in registers) goes to the other LDS buffer and the loads of slab s+2 start
        // while the matrix cores work on the first k step
        if (s + 1 < n_slabs) {
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                *reinterpret_cast<u32x4 *>(nx + st_off + 32 * q * kPitch) = xr[q];
                *reinterpret_cast<u32x4 *>(nx + kTileM * kPitch + st_off + 32 * q * kPitch) = ar[q];
            }
            if (s + 2 < n_slabs) {
                const uint32_t off = uint32_t(s + 2) * (kTileK * 2 / 16);
#pragma unroll
                for (int q = 0; q < 8; ++q) {
                    xr[q] = xb[xo[q] + off];
                    ar[q] = ab[ao[q] + off];
                }
            }
        }
        NTS_LOAD_FRAGS(2, xf0, af0)
        NTS_MFMAS(xf1, af1)
        NTS_LOAD_FRAGS(3, xf1, af1)
        NTS_MFMAS(xf0, af0)
        NTS_MFMAS(xf1, af1)
        __syncthreads();                                // buffer s&1 is free, buffer (s+1)&1 is complete
    }
#undef NTS_LOAD_FRAGS
#undef NTS_MFMAS
    // D[i = (v/4)*8 + (lane/32)*4 + v%4][j = lane%32]: batch row i, weight row j
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int n = n0 + wn * 128 + b * 32 + fr;
            if (n < Nn) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int m = m0 + wm * 128 + a * 32 + (v / 4) * 8 + fg * 4 + (v % 4);
                    if (m < M) Y[int64_t(m) * ldy + n] = E::round(acc[a][b][v]);
                }
            }
        }
}

}  // namespace

static int skinny_row_tiles(int M) { return M > 32 ? 2 : 1; }
static int skinny_waves(int) { return 4; }   // 8 wavefronts per workgroup measured slower for wide batches

int nts_linear_skinny_splits(int M, int Nn, int K)
{
    const int waves = (Nn + 16 * skinny_row_tiles(M) - 1) / (16 * skinny_row_tiles(M));
    const int n_chunks = (K + kSkinnyChunk - 1) / kSkinnyChunk;
    int splits = (2048 + waves - 1) / waves;          // aim at >= 8 wavefronts per compute unit (swept: 512..8192)
    // the fp32 partial sums are written and read back by the reduction: keep that traffic
    // (splits * M * Nn * 8 bytes) under a fifth of the weight bytes, or 16 MiB if that is more
    const int64_t budget = std::max<int64_t>(int64_t(Nn) * K * 2 / 5, int64_t(16) << 20);
    const int64_t cap = budget / (int64_t(M) * Nn * 8);
    if (splits > cap) splits = int(cap);
    if (splits > n_chunks) splits = n_chunks;
    if (splits < 1) splits = 1;
    const int cps = (n_chunks + splits - 1) / splits;
    return (n_chunks + cps - 1) / cps;                // no empty split
}

hipError_t nts_launch_linear_skinny(const uint16_t *X, int64_t ldx, const uint16_t *A, int64_t lda,
                                    uint16_t *Y, int64_t ldy, float *part, int splits, int M, int Nn,
                                    int K, bool f16, hipStream_t st)
{
    const int n_chunks = (K + kSkinnyChunk - 1) / kSkinnyChunk;
    const int cps = (n_chunks + splits - 1) / splits;
    const int rows_per_wg = 16 * skinny_row_tiles(M) * skinny_waves(M);
    const dim3 grid((Nn + rows_per_wg - 1) / rows_per_wg, splits), block(skinny_waves(M) * 64);
    float *p = splits > 1 ? part : nullptr;
    const int mt = (M + 15) / 16;
#define NTS_SK(MT, RT, WV)                                                                                            \
    {                                                                                                               \
        if (f16) hipLaunchKernelGGL((nts_linear_skinny_kernel<F16, MT, RT, WV>), grid, block, 0, st, X, ldx, A, lda, Y, ldy, p, M, Nn, K, cps); \
        else hipLaunchKernelGGL((nts_linear_skinny_kernel<Bf16, MT, RT, WV>), grid, block, 0, st, X, ldx, A, lda, Y, ldy, p, M, Nn, K, cps);    \
    }
    if (mt == 1) NTS_SK(1, 1, 4)
    else if (mt == 2) NTS_SK(2, 1, 4)
    else if (mt == 3) NTS_SK(3, 2, 4)
    else NTS_SK(4, 2, 4)
#undef NTS_SK
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || splits <= 1) return e;
    const int64_t n = int64_t(M) * Nn;
    if (f16) hipLaunchKernelGGL(nts_linear_reduce_kernel<F16>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, part, splits, M, Nn, Y, ldy);
    else hipLaunchKernelGGL(nts_linear_reduce_kernel<Bf16>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, part, splits, M, Nn, Y, ldy);
    return hipGetLastError();
}

hipError_t nts_launch_linear_tiled(const uint16_t *X, int64_t ldx, const uint16_t *A, int64_t lda,
                                   uint16_t *Y, int64_t ldy, int M, int Nn, int K, bool f16, hipStream_t st)
{
    static bool configured = false;
    if (!configured) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(nts_linear_tiled_kernel<Bf16>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 2 * kTileLds);
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(nts_linear_tiled_kernel<F16>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, 2 * kTileLds);
        if (e != hipSuccess) return e;
        configured = true;
    }
    const int tiles_m = (M + kTileM - 1) / kTileM, tiles_n = (Nn + kTileN - 1) / kTileN;
    const int sups = ((tiles_m + kSupM - 1) / kSupM) * ((tiles_n + kSupN - 1) / kSupN);
    const dim3 grid(unsigned((sups + 7) / 8) * 8u * kSupM * kSupN), block(256);
    if (f16) hipLaunchKernelGGL(nts_linear_tiled_kernel<F16>, grid, block, 2 * kTileLds, st, X, ldx, A, lda, Y, ldy, M, Nn, K);
    else hipLaunchKernelGGL(nts_linear_tiled_kernel<Bf16>, grid, block, 2 * kTileLds, st, X, ldx, A, lda, Y, ldy, M, Nn, K);
    return hipGetLastError();
}
