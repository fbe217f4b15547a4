// TP-shard-selecting linear layer (paper Sec. 3.2.1: one full weight copy per
// GPU, the rank's 1/N shard picked at execution time).  The shard is never
// copied: a column-parallel shard is a row block of the [n_out][n_in] weight,
// a row-parallel shard a column block, so both are a base offset plus the full
// matrix's row stride, and every kernel here computes
//     Y[M][Nn] = X[M][K] . A[Nn][K]^T        (A = the shard, row stride lda)
// with 16-bit inputs (bfloat16 or float16), fp32 accumulation on the matrix cores and
// one rounding to the input format.
//
// Three kernels: a decode kernel for batches of at most 16 rows on mid-size shards (16-row
// blocks, a workgroup's wavefronts share the K range), a weight-streaming kernel for batches
// up to a few hundred rows (decode and short prefill chunks; both bound by reading the shard
// once from HBM) and a 256 x 256 tiled kernel for long prefill batches (bound by the matrix
// cores).  Each is described where it is defined.
#include <algorithm>

#include "nts_internal.h"

#include <atomic>

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

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
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// The two 16-bit element formats: matrix-core instructions and the final rounding.
struct Bf16 {
    typedef bf16x8 vec8;
    static __device__ __forceinline__ f32x4 mfma16(vec8 a, vec8 b, f32x4 c) { return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0); }
    static __device__ __forceinline__ f32x16 mfma32(vec8 a, vec8 b, f32x16 c) { return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0); }
    static __device__ __forceinline__ uint16_t round(float f) { return f32_to_bf16_rne(f); }
    // two values at once (lo in bits 0..15): one v_cvt_pk_bf16_f32, round to nearest even
    static __device__ __forceinline__ uint32_t round2(float lo, float hi)
    {
        const f32x2 v = {lo, hi};
        return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
    }
};
struct F16 {
    typedef f16x8 vec8;
    static __device__ __forceinline__ f32x4 mfma16(vec8 a, vec8 b, f32x4 c) { return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0); }
    static __device__ __forceinline__ f32x16 mfma32(vec8 a, vec8 b, f32x16 c) { return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0); }
    static __device__ __forceinline__ uint16_t round(float f) { return f32_to_f16_rne(f); }
    static __device__ __forceinline__ uint32_t round2(float lo, float hi)
    {
        const f32x2 v = {lo, hi};
        return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2));
    }
};

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
// Weight-streaming kernel (decode batches and short prefill chunks): bound by the
// weight bytes, read exactly once; for wider batches there is also enough
// matrix-core and LDS work that neither may be wasted.  A workgroup takes 32*MT
// batch rows and 32*RT*CW weight rows.  CW "consumer" wavefronts each own 32*RT
// weight rows for all of the batch rows, as MT x RT tiles of
// v_mfma_f32_32x32x16 (RT = 1 in every configuration in use: two tiles per
// consumer halve the LDS reads per MFMA but measured slower).  A weight row is
// used by one wavefront only, so weights go from global memory straight into
// registers: lane (row = lane%32, g = lane/32) holds, for a 64-wide slab, the
// four 16-byte pieces k = 16s + 8g .. +7 (s = 0..3) of its row, one per MFMA
// step; the batch fragments are read from LDS with the same k.  The loads are
// plain, not non-temporal: the two lanes and two instructions that share a
// 64-byte half line then meet in the L1 instead of each going to the L2, which
// alone was worth 88 -> 54 us on a 224 MiB shard.  The batch slab (32*MT rows x
// 64 k) is shared by the consumers and is brought into LDS by one more,
// "producer" wavefront.  Splitting the roles matters because a wavefront's
// loads return in order: a consumer that also fetched batch rows would, each
// time it waits for them, wait for every weight load issued before them.
// Consumers keep NSETS-1 slabs of weights in flight (NSETS register sets used in
// rotation; the slab loop is unrolled by NSETS so the sets are fixed registers).
// K can be split over blockIdx.y (fp32 partial sums, reduced in split order by
// nts_linear_reduce_kernel).  Workgroup order: the batch tiles of one weight
// block run back to back on one XCD, so that block is fetched from HBM once and
// then served by that XCD's L2.

// Workgroup barrier that orders LDS accesses only.  __syncthreads() also waits for every
// outstanding global load (its fences cover global memory), which would drain the weight
// prefetch at every slab.
__device__ __forceinline__ void nts_lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

constexpr int kStrK = 64;
constexpr int kStrPitch = kStrK * 2 + 16;          // bytes per batch row in LDS

template <class E, int MT, int CW, int NSETS, int RT>
__global__ __launch_bounds__(64 * (CW + 1)) void nts_linear_stream_kernel(
    const uint16_t *__restrict__ X, int64_t ldx, const uint16_t *__restrict__ A, int64_t lda,
    uint16_t *__restrict__ Y, int64_t ldy, float *__restrict__ part, int M, int Nn, int K,
    int slabs_per_split, int tiles_m, int blocks_n)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    typedef typename E::vec8 vec8;
    constexpr int kBuf = 32 * MT * kStrPitch;           // one of three batch-slab buffers
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int xcd = blockIdx.x & 7, seq = blockIdx.x >> 3;
    const int by = seq % tiles_m, bx = (seq / tiles_m) * 8 + xcd;
    if (bx >= blocks_n) return;                         // whole workgroup leaves before any barrier
    const int m0 = by * 32 * MT;
    const int split = blockIdx.y;
    const int n_slabs = K / kStrK;
    const int s_lo = split * slabs_per_split, s_hi = min(n_slabs, s_lo + slabs_per_split);
    // Workgroups walk their k range from different starting slabs (and wrap around): rows are
    // a power-of-two number of bytes apart, so workgroups that all read the same k at the same
    // time would keep hitting the same few memory channels (measured: 10 % on a 224 MiB shard at
    // 64 batch rows).  Tall batch tiles do the opposite: their workgroups should read the same
    // batch slab at the same time so that it is fetched into the L2 once, and the weight bytes
    // per workgroup are too few to camp (2 to 5 % the other way at 256 rows).
    const int s_cnt = s_hi - s_lo, s_rot = MT >= 6 ? 0 : (bx * 5 + by) % s_cnt;
#define NTS_STR_PHYS(ss) (s_lo + ((min((ss), s_hi - 1) - s_lo + s_rot) % s_cnt))

    // Slab s lives in LDS buffer s % 3.  During slab period s the producer writes slab s+1
    // and the consumers read slab s; the one barrier per period (in its middle for the
    // consumers) publishes slab s+1 and retires slab s-1, so the consumers can read the first
    // fragments of slab s+1 during the last MFMA step of slab s.
    if (wv == CW) {
        // producer: lane moves 16-byte vector (lane & 7) of rows (lane >> 3) + 8 q
        const int sv = lane & 7, sr = lane >> 3;
        const u32x4 *xrow[4 * MT];
#pragma unroll
        for (int q = 0; q < 4 * MT; ++q)
            xrow[q] = reinterpret_cast<const u32x4 *>(X + int64_t(min(m0 + sr + 8 * q, M - 1)) * ldx + sv * 8);
        const int st_off = sr * kStrPitch + sv * 16;
        // XD register sets: the rows of slab s+1+XD are requested while slab s+1 is written,
        // so XD round trips overlap (one per slab would cap the slab rate at the loaded L2 latency)
        constexpr int XD = MT <= 2 ? 4 : (MT <= 4 ? 2 : 1);   // bounded by registers
        u32x4 xr[XD][4 * MT];
#define NTS_STR_LOAD_X(SET, slab)                                                              \
    _Pragma("unroll") for (int q = 0; q < 4 * MT; ++q)                                         \
        xr[SET][q] = xrow[q][NTS_STR_PHYS(slab) * (kStrK * 2 / 16)];
#define NTS_STR_STORE_X(SET, buf)                                                              \
    _Pragma("unroll") for (int q = 0; q < 4 * MT; ++q)                                         \
        *reinterpret_cast<u32x4 *>((buf) + st_off + 8 * q * kStrPitch) = xr[SET][q];
        NTS_STR_LOAD_X(0, s_lo)
        NTS_STR_STORE_X(0, lds)
#pragma unroll
        for (int d = 0; d < XD; ++d) NTS_STR_LOAD_X(d, s_lo + 1 + d)
        nts_lds_barrier();
        int nb = 1;                                     // buffer of slab s+1
#define NTS_STR_PERIOD(U, ss)                                                                  \
    {                                                                                          \
        NTS_STR_STORE_X(U, lds + nb * kBuf)  /* past the end: a copy of the last slab, never read */ \
        NTS_STR_LOAD_X(U, (ss) + 1 + XD)                                                       \
        nts_lds_barrier();                                                                     \
        nb = nb == 2 ? 0 : nb + 1;                                                             \
    }
        int s = s_lo;
        for (; s + XD <= s_hi; s += XD) {
#pragma unroll
            for (int u = 0; u < XD; ++u) NTS_STR_PERIOD(u, s + u)
        }
#pragma unroll
        for (int u = 0; u < XD - 1; ++u)
            if (s + u < s_hi) NTS_STR_PERIOD(u, s + u)
#undef NTS_STR_PERIOD
#undef NTS_STR_LOAD_X
#undef NTS_STR_STORE_X
        return;
    }

    const int fr = lane & 31, fg = lane >> 5;
    const int n0 = (bx * CW + wv) * 32 * RT;
    // weight rows of this lane (rows past the end are computed from the last row, not stored)
    const u32x4 *arow[RT];
#pragma unroll
    for (int r = 0; r < RT; ++r)
        arow[r] = reinterpret_cast<const u32x4 *>(A + int64_t(min(n0 + r * 32 + fr, Nn - 1)) * lda + fg * 8);

    f32x16 acc[MT][RT];
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
        for (int r = 0; r < RT; ++r)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[t][r][v] = 0.f;

    u32x4 w[NSETS][RT][4];
#define NTS_STR_WLOAD(p) (*(p))
#define NTS_STR_LOAD_W(DST, slab)                                                              \
    _Pragma("unroll") for (int r = 0; r < RT; ++r)                                             \
        _Pragma("unroll") for (int q = 0; q < 4; ++q)                                          \
            DST[r][q] = NTS_STR_WLOAD(arow[r] + NTS_STR_PHYS(slab) * (kStrK * 2 / 16) + 2 * q);
    // One MFMA step = one batch tile t at one k step k4 (step i = k4*MT + t).  Its batch
    // fragment is read from LDS three steps ahead into a window of four registers; the last
    // three reads of a slab already fetch the first fragments of the next slab.
#define NTS_STR_FRAG(DST, buf, i)                                                              \
    DST = __builtin_bit_cast(vec8, *reinterpret_cast<const u32x4 *>(                           \
        (buf) + (((i) % MT) * 32 + fr) * kStrPitch + (((i) / MT) * 16 + fg * 8) * 2));
    // Nothing in a slab is conditional (the compiler's wait-count bookkeeping would otherwise
    // assume the shortest path and wait for the newest loads): past the end of this split's
    // k range the weight loads repeat its last slab, which is in cache.
#define NTS_STR_SLAB(U, ss)                                                                    \
    {                                                                                          \
        const unsigned char *xs = lds + cur * kBuf;                                            \
        cur = cur == 2 ? 0 : cur + 1;                                                          \
        const unsigned char *nx = lds + cur * kBuf;                                            \
        NTS_STR_LOAD_W(w[((U) + NSETS - 1) % NSETS], (ss) + NSETS - 1)                         \
        __builtin_amdgcn_sched_barrier(0);                                                     \
        _Pragma("unroll") for (int i = 0; i < kSteps; ++i) {                                   \
            if (i == kBarrierStep) nts_lds_barrier();                                          \
            if (i + 3 < kSteps) { NTS_STR_FRAG(xf[(i + 3) % 4], xs, i + 3) }                   \
            else { NTS_STR_FRAG(xf[(i + 3) % 4], nx, i + 3 - kSteps) }                         \
            _Pragma("unroll") for (int r = 0; r < RT; ++r)                                     \
                acc[i % MT][r] = E::mfma32(__builtin_bit_cast(vec8, w[(U) % NSETS][r][i / MT]), xf[i % 4], \
                                           acc[i % MT][r]);                                    \
            __builtin_amdgcn_sched_barrier(0);                                                 \
        }                                                                                      \
    }

    constexpr int kSteps = 4 * MT;
    // the barrier of a slab comes before the first read from the next slab's buffer
    constexpr int kBarrierStep = 2 * MT < kSteps - 3 ? 2 * MT : kSteps - 3;
#pragma unroll
    for (int d = 0; d < NSETS - 1; ++d) NTS_STR_LOAD_W(w[d], s_lo + d)
    nts_lds_barrier();
    vec8 xf[4];
    NTS_STR_FRAG(xf[0], lds, 0)
    NTS_STR_FRAG(xf[1], lds, 1)
    NTS_STR_FRAG(xf[2], lds, 2)
    int cur = 0;                                        // LDS buffer of the current slab
    int s = s_lo;
    for (; s + NSETS <= s_hi; s += NSETS) {
#pragma unroll
        for (int u = 0; u < NSETS; ++u) NTS_STR_SLAB(u, s + u)
    }
#pragma unroll
    for (int u = 0; u < NSETS - 1; ++u)
        if (s + u < s_hi) NTS_STR_SLAB(u, s + u)
#undef NTS_STR_SLAB
#undef NTS_STR_PHYS
#undef NTS_STR_LOAD_W
#undef NTS_STR_FRAG
    // The weight rows are the first MFMA operand, so D[i][j] has i = weight row, j = batch row:
    // lane (fr, fg) holds, of batch row fr of tile t, the output columns (v/4)*8 + fg*4 + v%4 of
    // tile r, four neighbours per group of v: one 8-byte store of four rounded values (two per
    // conversion instruction), or one 16-byte store of partial sums.
    const bool vec_ok = (Nn & 3) == 0;
#pragma unroll
    for (int t = 0; t < MT; ++t) {
        const int m = m0 + t * 32 + fr;
        if (m >= M) continue;
#pragma unroll
        for (int r = 0; r < RT; ++r)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int n = n0 + r * 32 + g * 8 + fg * 4;
                if (n >= Nn) continue;
                const float v0 = acc[t][r][4 * g], v1 = acc[t][r][4 * g + 1], v2 = acc[t][r][4 * g + 2],
                            v3 = acc[t][r][4 * g + 3];
                if (part) {
                    float *dst = part + (int64_t(split) * M + m) * Nn + n;
                    if (vec_ok) {                       // then n + 4 <= Nn and the address is 16-byte aligned
                        const f32x4 q = {v0, v1, v2, v3};
                        *reinterpret_cast<f32x4 *>(dst) = q;
                    } else {
                        dst[0] = v0;
                        if (n + 1 < Nn) dst[1] = v1;
                        if (n + 2 < Nn) dst[2] = v2;
                        if (n + 3 < Nn) dst[3] = v3;
                    }
                } else {
                    uint16_t *dst = Y + int64_t(m) * ldy + n;
                    const u32x2 pk = {E::round2(v0, v1), E::round2(v2, v3)};
                    if (n + 4 <= Nn) {
                        *reinterpret_cast<u32x2 *>(dst) = pk;
                    } else {
                        dst[0] = uint16_t(pk[0]);
                        if (n + 1 < Nn) dst[1] = uint16_t(pk[0] >> 16);
                        if (n + 2 < Nn) dst[2] = uint16_t(pk[1]);
                    }
                }
            }
    }
}

// ---------------------------------------------------------------------------
// Decode kernel (batches of at most 16 rows on shards too small to fill the chip with 32-row
// blocks): what a compute unit can stream depends on how many wavefronts ask, about 13 GB/s
// for one and HBM speed for four, so a mid-size shard needs a thousand wavefronts with their
// own weights.  A workgroup takes 16 weight rows (v_mfma_f32_16x16x32: weight rows first, so
// a lane ends with four neighbouring output columns of one batch row) and its KS wavefronts
// split the K range among themselves; a wavefront streams its weights and the matching
// batch elements (a few KiB, always in the L2) straight into NSETS register sets, with no
// LDS, no barrier and no producer in the loop, so the wavefronts' trip counts may differ.  At
// the end the partial tiles meet in LDS and wavefront 0 adds them in wavefront order: one
// launch, reproducible.  blockIdx.y can split K further (partial planes + reduce kernel, as
// in the streaming kernel).
template <class E, int KS, int RB, int NSETS>
__global__ __launch_bounds__(64 * KS) void nts_linear_decode_kernel(
    const uint16_t *__restrict__ X, int64_t ldx, const uint16_t *__restrict__ A, int64_t lda,
    uint16_t *__restrict__ Y, int64_t ldy, float *__restrict__ part, int M, int Nn, int K, int slabs_per_split)
{
    typedef typename E::vec8 vec8;
    __shared__ f32x4 red[KS > 1 ? KS - 1 : 1][RB][64];
    const int lane = threadIdx.x & 63, g = threadIdx.x >> 6;
    const int n0 = blockIdx.x * 16 * RB, split = blockIdx.y;
    const int n_slabs = K / kStrK;
    const int wg_lo = split * slabs_per_split, wg_hi = min(n_slabs, wg_lo + slabs_per_split);
    // this wavefront's share of the workgroup's slabs: contiguous, sizes differ by at most one
    const int cnt = wg_hi - wg_lo, per = cnt / KS, rem = cnt % KS;
    const int lo = wg_lo + g * per + min(g, rem), hi = lo + per + (g < rem ? 1 : 0);
    const int last = max(min(hi, n_slabs) - 1, 0);      // requests past the end repeat a slab inside the matrix
    const int fr = lane & 15, kg = lane >> 4;           // row and k group of this lane in both operands
    const u32x4 *wrow[RB];
#pragma unroll
    for (int r = 0; r < RB; ++r)
        wrow[r] = reinterpret_cast<const u32x4 *>(A + int64_t(min(n0 + r * 16 + fr, Nn - 1)) * lda + kg * 8);
    const u32x4 *xrow = reinterpret_cast<const u32x4 *>(X + int64_t(min(fr, M - 1)) * ldx + kg * 8);

    f32x4 acc[RB];
#pragma unroll
    for (int r = 0; r < RB; ++r) acc[r] = f32x4{0.f, 0.f, 0.f, 0.f};
    u32x4 w[NSETS][RB][2], x[NSETS][2];
#define NTS_DEC_LOAD(SET, slab)                                                                \
    {                                                                                          \
        const int off_ = min((slab), last) * (kStrK * 2 / 16);                                 \
        _Pragma("unroll") for (int r = 0; r < RB; ++r) {                                       \
            w[SET][r][0] = wrow[r][off_];                                                      \
            w[SET][r][1] = wrow[r][off_ + 4];                                                  \
        }                                                                                      \
        x[SET][0] = xrow[off_];                                                                \
        x[SET][1] = xrow[off_ + 4];                                                            \
    }
#define NTS_DEC_SLAB(U, ss)                                                                    \
    {                                                                                          \
        NTS_DEC_LOAD(((U) + NSETS - 1) % NSETS, (ss) + NSETS - 1)                              \
        _Pragma("unroll") for (int q = 0; q < 2; ++q)                                          \
            _Pragma("unroll") for (int r = 0; r < RB; ++r)                                     \
                acc[r] = E::mfma16(__builtin_bit_cast(vec8, w[(U) % NSETS][r][q]),             \
                                   __builtin_bit_cast(vec8, x[(U) % NSETS][q]), acc[r]);       \
    }
#pragma unroll
    for (int d = 0; d < NSETS - 1; ++d) NTS_DEC_LOAD(d, lo + d)
    int s = lo;
    for (; s + NSETS <= hi; s += NSETS) {
#pragma unroll
        for (int u = 0; u < NSETS; ++u) NTS_DEC_SLAB(u, s + u)
    }
#pragma unroll
    for (int u = 0; u < NSETS - 1; ++u)
        if (s + u < hi) NTS_DEC_SLAB(u, s + u)
#undef NTS_DEC_SLAB
#undef NTS_DEC_LOAD
    if (KS > 1) {
        if (g > 0) {
#pragma unroll
            for (int r = 0; r < RB; ++r) red[g - 1][r][lane] = acc[r];
        }
        __syncthreads();
        if (g > 0) return;
#pragma unroll
        for (int k = 1; k < KS; ++k)
#pragma unroll
            for (int r = 0; r < RB; ++r) acc[r] += red[k - 1][r][lane];
    }
    // D[i][j]: i = weight row = (lane / 16) * 4 + v, j = batch row = lane % 16
    const int m = fr;
    if (m >= M) return;
#pragma unroll
    for (int r = 0; r < RB; ++r) {
        const int n = n0 + r * 16 + kg * 4;
        if (n >= Nn) continue;
        if (part) {
            float *dst = part + (int64_t(split) * M + m) * Nn + n;
            if ((Nn & 3) == 0) {
                *reinterpret_cast<f32x4 *>(dst) = acc[r];
            } else {
                dst[0] = acc[r][0];
                if (n + 1 < Nn) dst[1] = acc[r][1];
                if (n + 2 < Nn) dst[2] = acc[r][2];
                if (n + 3 < Nn) dst[3] = acc[r][3];
            }
        } else {
            uint16_t *dst = Y + int64_t(m) * ldy + n;
            const u32x2 pk = {E::round2(acc[r][0], acc[r][1]), E::round2(acc[r][2], acc[r][3])};
            if (n + 4 <= Nn) {
                *reinterpret_cast<u32x2 *>(dst) = pk;
            } else {
                dst[0] = uint16_t(pk[0]);
                if (n + 1 < Nn) dst[1] = uint16_t(pk[0] >> 16);
                if (n + 2 < Nn) dst[2] = uint16_t(pk[1]);
            }
        }
    }
}

// ---------------------------------------------------------------------------
// Large batches (prefill): bound by the matrix cores.  A 256-thread workgroup computes a
// 64*MA x 64*NB tile of Y (MA = NB = 4: 256 x 256; MA = 4, NB = 2: 256 x 128; MA = NB = 2:
// 128 x 128; NB = 3: 256 x 192 and 128 x 192); each of its four wavefronts owns a 32*MA x 32*NB part as MA x NB tiles of
// v_mfma_f32_32x32x16 (16*MA*NB fp32 accumulators per lane, one wavefront per SIMD).  X and
// weight rows are both contiguous along k, so both operands are staged the same way: 64-wide k
// slabs go global -> registers -> LDS (row pitch 144 B, which spreads the 32 rows a
// ds_read_b128 touches over all banks).  LDS holds two slabs: while the MFMAs of slab s read
// one buffer, slab s+1 is written into the other and the global loads of slab s+2 are in
// flight; one barrier per slab.  The smaller tiles read more LDS bytes per MFMA (x1.5, x2) and
// reach 0.87 and about 0.75 of the 256 x 256 tile's rate per compute unit; they are for outputs
// whose 256 x 256 tiling leaves the last round of workgroups half empty or fills too few
// compute units (measured: 6144 outputs at M = 4096, 384 tiles of 256 x 256 in 1.5 rounds,
// 210 us; 768 of 256 x 128 in 3 rounds, 178 us; 4096 outputs at M = 1024, 64 tiles of
// 256 x 256, streaming kernel 56 us; 256 tiles of 128 x 128, 45 us).  The 192-wide tiles are
// for outputs they divide into a whole number of rounds where the others do not (6144 outputs:
// M = 2048, 192 tiles of 256 x 256, 106 us; 256 of 256 x 192, 87.5 us; M = 1024, 192 tiles of
// 256 x 128, 61.7 us; 256 of 128 x 192, 57 us); per compute unit they run at the wide tile's rate.
constexpr int kTileK = 64;                              // slab depth; a tile is 64 * MA rows by 64 * NB columns
constexpr int kSupM = 4, kSupN = 8;                     // tiles per XCD-resident block
constexpr int kPitch = kTileK * 2 + 16;                 // bytes per LDS row

template <class E, int NB, int MA>
__global__ __launch_bounds__(256) void nts_linear_tiled_kernel(
    const uint16_t *__restrict__ X, int64_t ldx, const uint16_t *__restrict__ A, int64_t lda,
    uint16_t *__restrict__ Y, int64_t ldy, int M, int Nn, int K)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    constexpr int kTN = 64 * NB;                        // tile width: two wavefronts of NB 32-wide tiles
    constexpr int kTM = 64 * MA;                        // tile height: two wavefronts of MA 32-row tiles
    constexpr int kLdsN = (kTM + kTN) * kPitch;         // bytes per LDS buffer
    constexpr int NX = 2 * MA;                          // 32-row passes of the batch operand
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int wm = wv >> 1, wn = wv & 1;                // quadrant of this wavefront
    // Workgroup -> tile.  Consecutive workgroup ids go to the 8 XCDs in turn and each XCD has
    // its own L2, so the 32 workgroups that run together on one XCD are given a 4 x 8 block of
    // tiles: every X slab is then fetched into that L2 once for 8 tiles and every weight slab
    // once for 4, instead of each workgroup streaming a weight tile of its own.
    const int tiles_m = (M + kTM - 1) / kTM, tiles_n = (Nn + kTN - 1) / kTN;
    const int sup_n = (tiles_n + kSupN - 1) / kSupN;
    const int xcd = blockIdx.x & 7, seq = blockIdx.x >> 3;
    const int sup = (seq / (kSupM * kSupN)) * 8 + xcd, in_sup = seq % (kSupM * kSupN);
    const int tm = (sup / sup_n) * kSupM + in_sup / kSupN, tn = (sup % sup_n) * kSupN + in_sup % kSupN;
    if (tm >= tiles_m || tn >= tiles_n) return;         // whole workgroup leaves before any barrier
    const int m0 = tm * kTM, n0 = tn * kTN;

    // staging map: rows x 8 vectors of 16 B per operand and slab; thread t takes vector
    // (t & 7) of rows (t >> 3) + 32 * q, q = 0 .. rows / 32 - 1: eight lanes read one 128 B line.
    // A load's address is a uniform 64-bit base (the tile's first row plus the slab) plus a
    // 32-bit byte offset per lane that never changes (row inside the tile times the row
    // stride), so the slab loop spends no vector instructions on addresses.
    const int sv = tid & 7, sr = tid >> 3;
    constexpr int NA = 2 * NB;                          // 32-row passes of the weight operand
    uint32_t xo[NX], ao[NA];
#pragma unroll
    for (int q = 0; q < NX; ++q) {
        const int r = sr + 32 * q;
        xo[q] = uint32_t(min(m0 + r, M - 1) - m0) * uint32_t(ldx * 2) + uint32_t(sv * 16);
    }
#pragma unroll
    for (int q = 0; q < NA; ++q) {
        const int r = sr + 32 * q;
        ao[q] = uint32_t(min(n0 + r, Nn - 1) - n0) * uint32_t(lda * 2) + uint32_t(sv * 16);
    }
    const char *xt = reinterpret_cast<const char *>(X) + int64_t(m0) * ldx * 2;
    const char *at = reinterpret_cast<const char *>(A) + int64_t(n0) * lda * 2;
#define NTS_GLOAD(base, o) (*reinterpret_cast<const u32x4 *>((base) + (o)))

    f32x16 acc[MA][NB];
#pragma unroll
    for (int a = 0; a < MA; ++a)
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

    const int fr = lane & 31, fg = lane >> 5;           // fragment row and k group of this lane
    const int n_slabs = K / kTileK;
    const int st_off = sr * kPitch + sv * 16;           // where this thread's staged vectors go

    // prologue: slab 0 into LDS buffer 0, slab 1 into registers; both slabs' loads are issued
    // before the first wait, so the tile starts after one memory latency, not two
    u32x4 xr[NX], ar[NA];
    {
        u32x4 x0[NX], a0[NA];
#pragma unroll
        for (int q = 0; q < NX; ++q) x0[q] = NTS_GLOAD(xt, xo[q]);
#pragma unroll
        for (int q = 0; q < NA; ++q) a0[q] = NTS_GLOAD(at, ao[q]);
        const int64_t off = int64_t(min(1, n_slabs - 1)) * (kTileK * 2);
        const char *xg = xt + off, *ag = at + off;
#pragma unroll
        for (int q = 0; q < NX; ++q) xr[q] = NTS_GLOAD(xg, xo[q]);
#pragma unroll
        for (int q = 0; q < NA; ++q) ar[q] = NTS_GLOAD(ag, ao[q]);
#pragma unroll
        for (int q = 0; q < NX; ++q) *reinterpret_cast<u32x4 *>(lds + st_off + 32 * q * kPitch) = x0[q];
#pragma unroll
        for (int q = 0; q < NA; ++q) *reinterpret_cast<u32x4 *>(lds + kTM * kPitch + st_off + 32 * q * kPitch) = a0[q];
    }
    nts_lds_barrier();

    // Two fragment sets: while the MA*NB MFMAs of k step kk run on one set, the MA+NB fragments
    // of step kk+1 are read from LDS into the other, one read every STRIDE MFMAs and in the order
    // the next step consumes them (X0, the weight fragments, X1 ...).  A wavefront issues in
    // order and can have only 15 LDS operations outstanding (4-bit counter), so everything that
    // goes through LDS is spread between the MFMAs instead of issued in bursts: the stores of
    // slab s+1 (in registers since the previous slab) and, right behind each store, the global
    // load of slab s+2 into the same register, one pair per PAIR MFMAs over the first three k
    // steps.  sched_barrier pins this order; left alone the compiler serialises read - wait -
    // MFMA.  With MA = NB = 4 the LDS is about three quarters busy over a slab, evenly.
    // One barrier per slab, before the last k step: by then every wavefront has read all of
    // slab s (so slab s+2 may overwrite its buffer from the next iteration on) and has written
    // its part of slab s+1 (so the first fragments of slab s+1 can be read during the last k
    // step).  The reads of the last k step are issued back to back in the step before it, so
    // the barrier's wait for LDS is short.  Nothing in the loop is conditional: past the end
    // the loads repeat the last slab and the spare buffer takes the copy.  Two slabs per trip,
    // so each slab's LDS buffer is a constant and fragment reads and stores carry their whole
    // address in the instruction's offset field from a few per-lane bases.
    constexpr int NF = MA + NB;                         // fragments per k step
    constexpr int NM = MA * NB;                         // MFMAs per k step
    constexpr int NS = NX + NA;                         // staged vectors per thread and slab
    constexpr int PAIR = (3 * NM) / NS;                 // MFMA slots per store/load pair (first three k steps)
    constexpr int LSLOT = PAIR > 1 ? 1 : 0;             // the load follows its store, in the same slot if pairs come every MFMA
#define NTS_READ_FRAG(base, kk, r, XF, AF)                                                             \
    {                                                                                                  \
        if ((r) == 0 || (r) > NB) {                                                                    \
            const int a_ = (r) == 0 ? 0 : (r) - NB;                                                    \
            XF[a_] = __builtin_bit_cast(vec8, *reinterpret_cast<const u32x4 *>(                      \
                (base) + (wm * 32 * MA + a_ * 32 + fr) * kPitch + ((kk) * 16 + fg * 8) * 2));              \
        } else {                                                                                       \
            const int b_ = (r) - 1;                                                                    \
            AF[b_] = __builtin_bit_cast(vec8, *reinterpret_cast<const u32x4 *>(                      \
                (base) + (kTM + wn * 32 * NB + b_ * 32 + fr) * kPitch + ((kk) * 16 + fg * 8) * 2)); \
        }                                                                                              \
    }
    // staged vector i of a slab: X and weight vectors alternate while there are weight vectors left
#define NTS_STORE_ONE(i)                                                                               \
    {                                                                                                  \
        constexpr int NI_ = 2 * (NA < NX ? NA : NX);     /* interleaved part */                        \
        if ((i) < NI_ ? ((i) & 1) : (NA > NX)) { const int q_ = (i) < NI_ ? (i) >> 1 : (i) - NX;       \
               *reinterpret_cast<u32x4 *>(nx + kTM * kPitch + st_off + 32 * q_ * kPitch) = ar[q_]; }   \
        else { const int q_ = (i) < NI_ ? (i) >> 1 : (i) - NA;                                         \
               *reinterpret_cast<u32x4 *>(nx + st_off + 32 * q_ * kPitch) = xr[q_]; }                  \
    }
#define NTS_LOAD_ONE(i)                                                                                \
    {                                                                                                  \
        constexpr int NI_ = 2 * (NA < NX ? NA : NX);                                                   \
        if ((i) < NI_ ? ((i) & 1) : (NA > NX)) { const int q_ = (i) < NI_ ? (i) >> 1 : (i) - NX; ar[q_] = NTS_GLOAD(ag, ao[q_]); } \
        else { const int q_ = (i) < NI_ ? (i) >> 1 : (i) - NA; xr[q_] = NTS_GLOAD(xg, xo[q_]); }       \
    }
#define NTS_KSTEP(XF, AF, G0, NBASE, NKK, NXF, NAF, STRIDE)                                            \
    {                                                                                                  \
        _Pragma("unroll") for (int a = 0; a < MA; ++a)                                                 \
            _Pragma("unroll") for (int b = 0; b < NB; ++b) {                                           \
                const int i = a * NB + b, g = (G0) + i;      /* constants after unrolling */           \
                acc[a][b] = E::mfma32(AF[b], XF[a], acc[a][b]);                                       \
                if (i % (STRIDE) == 0 && i / (STRIDE) < NF) NTS_READ_FRAG(NBASE, NKK, i / (STRIDE), NXF, NAF) \
                if (g % PAIR == 0 && g / PAIR < NS) NTS_STORE_ONE(g / PAIR)                            \
                if (g % PAIR == LSLOT && g / PAIR < NS) NTS_LOAD_ONE(g / PAIR)                             \
                __builtin_amdgcn_sched_barrier(0);                                                     \
            }                                                                                          \
    }
    typedef typename E::vec8 vec8;
    vec8 xf0[MA], af0[NB], xf1[MA], af1[NB];
#pragma unroll
    for (int r = 0; r < NF; ++r) NTS_READ_FRAG(lds, 0, r, xf0, af0)
    constexpr int S2 = NM / NF >= 2 ? 2 : 1;            // fragment reads every other MFMA where there is room
#define NTS_SLAB(XS, NX, S)                                                                            \
    {                                                                                                  \
        const unsigned char *xs = (XS);                                                                \
        unsigned char *nx = (NX);                                                                      \
        const int64_t off = int64_t(min((S) + 2, n_slabs - 1)) * (kTileK * 2);                         \
        const char *xg = xt + off, *ag = at + off;                                                     \
        NTS_KSTEP(xf0, af0, 0, xs, 1, xf1, af1, S2)                                                    \
        NTS_KSTEP(xf1, af1, NM, xs, 2, xf0, af0, S2)                                                   \
        NTS_KSTEP(xf0, af0, 2 * NM, xs, 3, xf1, af1, 1)                                                \
        nts_lds_barrier();                                                                             \
        NTS_KSTEP(xf1, af1, 3 * NM, nx, 0, xf0, af0, S2)                                               \
    }
    int s = 0;
    for (; s + 2 <= n_slabs; s += 2) {
        NTS_SLAB(lds, lds + kLdsN, s)
        NTS_SLAB(lds + kLdsN, lds, s + 1)
    }
    if (s < n_slabs) NTS_SLAB(lds, lds + kLdsN, s)
#undef NTS_SLAB
#undef NTS_GLOAD
#undef NTS_READ_FRAG
#undef NTS_STORE_ONE
#undef NTS_LOAD_ONE
#undef NTS_KSTEP
    // Epilogue.  The weight fragment is the first MFMA operand, so D[i][j] has i = weight row,
    // j = batch row: lane (fr, fg) holds, of batch row fr of tile a, the output columns
    // (v/4)*8 + fg*4 + v%4 of tile b, four neighbours per group of v.  Stored from there a row
    // would get 16 bytes per instruction; instead each wavefront rounds a 32 x 32*NB strip to 16
    // bits two values per instruction, puts it into its own piece of LDS 8 bytes per lane (row
    // pitch 64*NB + 8 bytes: the 32 rows of a store fall into different banks) and writes whole
    // row segments, 16 bytes per lane.
    nts_lds_barrier();                                  // every wavefront is done with the tile buffers
    {
        constexpr int kOutPitch = 64 * NB + 8;          // bytes per strip row in LDS
        constexpr int kLanesRow = 4 * NB, kRowsIns = 64 / kLanesRow;   // NB = 3: five rows a pass, four lanes idle
        constexpr int kPasses = (32 + kRowsIns - 1) / kRowsIns;
        constexpr bool kRagged = 64 % kLanesRow != 0 || 32 % kRowsIns != 0;
        unsigned char *strip = lds + wv * 32 * kOutPitch;
        const int orow = lane / kLanesRow, ocol = (lane % kLanesRow) * 8;
#pragma unroll
        for (int a = 0; a < MA; ++a) {
#pragma unroll
            for (int b = 0; b < NB; ++b)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const u32x2 pk = {E::round2(acc[a][b][4 * g], acc[a][b][4 * g + 1]),
                                      E::round2(acc[a][b][4 * g + 2], acc[a][b][4 * g + 3])};
                    *reinterpret_cast<u32x2 *>(strip + fr * kOutPitch + (b * 32 + g * 8 + fg * 4) * 2) = pk;
                }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");      // the strip is complete (LDS works in order)
#pragma unroll
            for (int j = 0; j < kPasses; ++j) {
                const int r = j * kRowsIns + orow;
                if (kRagged && (orow >= kRowsIns || r >= 32)) continue;
                const u32x2 lo = *reinterpret_cast<const u32x2 *>(strip + r * kOutPitch + ocol * 2);
                const u32x2 hi = *reinterpret_cast<const u32x2 *>(strip + r * kOutPitch + ocol * 2 + 8);
                const u32x4 val = {lo[0], lo[1], hi[0], hi[1]};
                const int m = m0 + wm * 32 * MA + a * 32 + r, n = n0 + wn * 32 * NB + ocol;
                if (m < M) {
                    uint16_t *dst = Y + int64_t(m) * ldy + n;
                    if (n + 8 <= Nn) {
                        *reinterpret_cast<u32x4 *>(dst) = val;
                    } else {
#pragma unroll
                        for (int e = 0; e < 8; ++e)
                            if (n + e < Nn) dst[e] = uint16_t(val[e >> 1] >> ((e & 1) * 16));
                    }
                }
            }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        }
    }
}

}  // namespace

// A kernel that wants more dynamic LDS than the default limit has to be told so once per
// device.  The devices done are kept as a bit set per kernel; two first calls at the same time
// only repeat the (idempotent) attribute call.
static hipError_t allow_dynamic_lds(std::atomic<uint64_t> &done, const void *kernel, int bytes)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const uint64_t bit = 1ull << (unsigned(dev) & 63u);
    if (done.load(std::memory_order_acquire) & bit) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess) done.fetch_or(bit, std::memory_order_release);
    return e;
}

template <class E, int MT, int CW, int NSETS, int RT>
static hipError_t launch_stream_one(const uint16_t *X, int64_t ldx, const uint16_t *A, int64_t lda, uint16_t *Y,
                                 int64_t ldy, float *part, int splits, int M, int Nn, int K, hipStream_t st)
{
    const int lds_bytes = 3 * 32 * MT * kStrPitch;
    static std::atomic<uint64_t> configured{0};
    const hipError_t ea = allow_dynamic_lds(
        configured, reinterpret_cast<const void *>(nts_linear_stream_kernel<E, MT, CW, NSETS, RT>), lds_bytes);
    if (ea != hipSuccess) return ea;
    const int tiles_m = (M + 32 * MT - 1) / (32 * MT), blocks_n = (Nn + 32 * CW * RT - 1) / (32 * CW * RT);
    const int n_slabs = K / kStrK;
    const int sps = (n_slabs + splits - 1) / splits;
    const dim3 grid(unsigned((blocks_n + 7) / 8) * 8u * unsigned(tiles_m), unsigned((n_slabs + sps - 1) / sps));
    hipLaunchKernelGGL((nts_linear_stream_kernel<E, MT, CW, NSETS, RT>), grid, dim3(64 * (CW + 1)), lds_bytes, st, X, ldx, A,
                       lda, Y, ldy, splits > 1 ? part : nullptr, M, Nn, K, sps, tiles_m, blocks_n);
    return hipGetLastError();
}

// Configuration of the streaming kernel for a problem: batch-tile height (any instantiated
// one up to the smallest that holds the batch, at most 256 rows; a batch longer than the tile
// takes several, whose workgroups share the weight block through one XCD's L2), workgroup
// width (4, 2 or 1 consumers) and K split with the smallest estimated time.  The estimate is
// in microseconds, from measurements on MI355X of every instantiation at one workgroup per
// compute unit:
//   * per 64-wide slab a workgroup needs its variant's slab_us, set by what its compute unit
//     can take in and feed to the matrix cores; workgroups that share a compute unit share
//     that rate (two take twice as long), so the slabs cost rounds * slabs * slab_us with
//     rounds = workgroups / 256 rounded up;
//   * all of them together cannot read the shard faster than about 6.1 TB/s;
//   * every round pays the variant's round_us for filling and draining its pipelines and for
//     the output (rounds that fit a compute unit together pay it once, plus 0.7 for each
//     further one), every launch 2.5;
//   * a split adds the second launch plus writing and reading splits * M * Nn fp32 partial
//     sums at about 4 TB/s; it keeps at least four slabs and the workspace under 512 MiB.
// Square-ish tiles take in the fewest bytes per product, small ones fill the chip when the
// output is small: the estimate weighs the two.  Candidates are tried from the plain
// configuration (tallest tile, four consumers, no split) outwards, and each must beat the
// best so far by 5 %.  The entries of the two tallest tiles are 8 % below what was measured for
// them alone: over the candidates timed on every prefill shape of two models their estimates had
// come out 10-13 % above the measured times while the other variants' were within 3 %.
struct StreamVariant {
    int mt, cw;
    double slab_us, round_us;
};
static const StreamVariant kStreamVariants[] = {
    {8, 4, 1.138, 6.6}, {6, 4, 0.963, 5.7}, {4, 4, 0.822, 4.9}, {4, 2, 0.529, 2.9},
    {4, 1, 0.402, 2.45}, {3, 4, 0.662, 4.2}, {2, 4, 0.556, 3.7}, {2, 2, 0.343, 2.0}, {2, 1, 0.243, 1.3},
    {1, 4, 0.490, 3.0}, {1, 1, 0.178, 1.25},
};

NtsStreamCfg nts_linear_stream_config(int M, int Nn, int K)
{
    NtsStreamCfg c;
    const int rows = M < 256 ? M : 256;
    const int mt_min = rows <= 32 ? 1 : rows <= 64 ? 2 : rows <= 96 ? 3 : rows <= 128 ? 4 : rows <= 192 ? 6 : 8;
    const int n_slabs = K / kStrK;
    const double out_elems = double(M) * Nn;
    const double hbm_us = double(Nn) * K * 2. / 6.1e6;
    double best_t = 0.;
    c.mt = mt_min;
    c.cw = 4;
    c.splits = 1;
    for (const StreamVariant &v : kStreamVariants) {
        if (v.mt > mt_min || (v.mt == 1 && mt_min > 1)) continue;
        const int tiles_m = (M + 32 * v.mt - 1) / (32 * v.mt);
        const int lds_fit = (160 * 1024) / (3 * 32 * v.mt * kStrPitch);
        const int per_cu = 4 / v.cw < lds_fit ? 4 / v.cw : lds_fit;     // workgroups a compute unit holds at a time
        const int64_t wgs = int64_t(tiles_m) * ((Nn + 32 * v.cw - 1) / (32 * v.cw));
        double best_here = 0.;
        int best_splits = 0;
        for (int splits = 1; splits <= 32 && splits <= (n_slabs >= 4 ? n_slabs / 4 : 1); ++splits) {
            const int sps = (n_slabs + splits - 1) / splits;
            if ((n_slabs + sps - 1) / sps != splits) continue;              // would leave an empty split
            if (splits > 1 && out_elems * splits * 4 > double(int64_t(512) << 20)) break;
            const int64_t total = wgs * splits;
            const int64_t rounds = (total + 255) / 256, seq_rounds = (total + 256 * per_cu - 1) / (256 * per_cu);
            const double cu_us = double(rounds) * sps * v.slab_us;
            double t = 2.5 + (cu_us > hbm_us ? cu_us : hbm_us) + v.round_us * double(seq_rounds) +
                       0.7 * double(rounds - seq_rounds);
            if (splits > 1) t += 2.5 + out_elems * splits * 8. / 4.0e6;
            if (best_splits == 0 || t < 0.95 * best_here) {
                best_splits = splits;
                best_here = t;
            }
        }
        if (best_t == 0. || best_here < 0.95 * best_t) {
            c.mt = v.mt;
            c.cw = v.cw;
            c.splits = best_splits;
            best_t = best_here;
        }
    }
    c.nsets = c.mt <= 4 ? 4 : 3;
    if (c.cw == 1 && c.mt == 1) c.nsets = 8;            // a lone consumer needs more weight bytes in flight
    if (M > 16) return c;

    // The decode kernel against the best of the above.  Its estimate: a wavefront alone streams
    // about 10 GB/s of weights, a compute unit at most 26, less 0.4 per batch row (every
    // wavefront fetches the batch rows of its own K range); the chip at most 6.1 TB/s; a launch 2.5, every round of workgroups 1, short
    // K ranges pay for their pipeline fill, and wide batches 0.05 per row.
    const double bytes = double(Nn) * K * 2.;
    double best_dec = 0.;
    int dec_ks = 0, dec_rb = 0, dec_splits = 0;
    for (int rb = 1; rb <= 2; ++rb)
        for (int ks = 2 * rb; ks <= 4; ks *= 2)     // eight wavefronts, or two with two blocks, never came out ahead
            for (int splits = 1; splits <= 4; splits *= 2) {
                const int sps = (n_slabs + splits - 1) / splits;
                if ((n_slabs + sps - 1) / sps != splits) continue;
                const int spw = sps / ks;                                   // slabs per wavefront
                if (spw < 4) continue;
                if (splits > 1 && out_elems * splits * 4 > double(int64_t(512) << 20)) continue;
                const int64_t wgs = int64_t((Nn + 16 * rb - 1) / (16 * rb)) * splits;
                if (wgs > 4096) continue;
                const int per_cu = 12 / ks;                                 // workgroups a compute unit holds
                const int64_t rounds = (wgs + 256 * per_cu - 1) / (256 * per_cu);
                const int64_t wg_cu = (wgs + 255) / 256;                    // workgroups of the busiest compute unit
                double rate = 10. * double(ks * (wg_cu < per_cu ? wg_cu : per_cu));
                const double cap = 26. - 0.4 * M;           // the batch rows every wavefront fetches take their share
                if (rate > cap) rate = cap;
                if (wg_cu > 1 && rate > 22.) rate = 22.;    // measured: two small workgroups stream less than one of twice the rows
                double stream_us = bytes / double(wgs) * double(wg_cu) / (rate * 1e3);
                if (stream_us < hbm_us) stream_us = hbm_us;
                double t = 2.5 + 1.0 * double(rounds) + stream_us + 0.05 * M + (spw < 16 ? 0.08 * (16 - spw) : 0.);
                if (splits > 1) t += 2.5 + out_elems * splits * 8. / 4.0e6;
                if (dec_ks == 0 || t < best_dec) {
                    best_dec = t;
                    dec_ks = ks;
                    dec_rb = rb;
                    dec_splits = splits;
                }
            }
    // the lone-consumer variant's table entry was measured with weight blocks shared through the L2
    // by four batch tiles; with the single tile of a decode batch it runs about 12 % slower
    const double stream_t = c.mt == 1 && c.cw == 1 ? 1.12 * best_t : best_t;
    if (dec_ks > 0 && best_dec < stream_t) {           // no margin: measured, the decode kernel wins more ties than it loses
        c.ks = dec_ks;
        c.rt = dec_rb;                                  // row blocks of 16 per wavefront
        c.splits = dec_splits;
        c.nsets = dec_rb == 1 ? 8 : 6;
    }
    return c;
}

template <class E, int KS, int RB>
static hipError_t launch_decode_one(const uint16_t *X, int64_t ldx, const uint16_t *A, int64_t lda, uint16_t *Y,
                                    int64_t ldy, float *part, int splits, int M, int Nn, int K, hipStream_t st)
{
    const int n_slabs = K / kStrK, sps = (n_slabs + splits - 1) / splits;
    const dim3 grid(unsigned((Nn + 16 * RB - 1) / (16 * RB)), unsigned((n_slabs + sps - 1) / sps));
    hipLaunchKernelGGL((nts_linear_decode_kernel<E, KS, RB, (RB == 1 ? 8 : 6)>), grid, dim3(64 * KS), 0, st, X, ldx, A,
                       lda, Y, ldy, splits > 1 ? part : nullptr, M, Nn, K, sps);
    return hipGetLastError();
}

hipError_t nts_launch_linear_stream(const uint16_t *X, int64_t ldx, const uint16_t *A, int64_t lda, uint16_t *Y,
                                    int64_t ldy, float *part, const NtsStreamCfg &c, int M, int Nn, int K,
                                    bool f16, hipStream_t st)
{
    hipError_t e = hipErrorInvalidValue;
    if (c.ks > 0) {
        if (M > 16) return hipErrorInvalidValue;
#define NTS_DEC(KS, RB)                                                                                        \
    if (c.ks == KS && c.rt == RB)                                                                              \
        e = f16 ? launch_decode_one<F16, KS, RB>(X, ldx, A, lda, Y, ldy, part, c.splits, M, Nn, K, st)         \
                : launch_decode_one<Bf16, KS, RB>(X, ldx, A, lda, Y, ldy, part, c.splits, M, Nn, K, st);
        NTS_DEC(2, 1) NTS_DEC(4, 1) NTS_DEC(4, 2)
#undef NTS_DEC
    } else {
#define NTS_STR(MT, CW, NS, RT)                                                                                \
    if (c.mt == MT && c.cw == CW && c.nsets == NS && c.rt == RT)                                               \
        e = f16 ? launch_stream_one<F16, MT, CW, NS, RT>(X, ldx, A, lda, Y, ldy, part, c.splits, M, Nn, K, st) \
                : launch_stream_one<Bf16, MT, CW, NS, RT>(X, ldx, A, lda, Y, ldy, part, c.splits, M, Nn, K, st);
    NTS_STR(1, 4, 4, 1) NTS_STR(2, 4, 4, 1) NTS_STR(3, 4, 4, 1) NTS_STR(4, 4, 4, 1) NTS_STR(6, 4, 3, 1) NTS_STR(8, 4, 3, 1)
    NTS_STR(1, 1, 8, 1) NTS_STR(2, 1, 4, 1) NTS_STR(4, 1, 4, 1)
    NTS_STR(2, 2, 4, 1) NTS_STR(4, 2, 4, 1)
#undef NTS_STR
    }
    if (e != hipSuccess || c.splits <= 1) return e;
    const int64_t n = int64_t(M) * Nn;
    if (f16) hipLaunchKernelGGL(nts_linear_reduce_kernel<F16>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, part, c.splits, M, Nn, Y, ldy);
    else hipLaunchKernelGGL(nts_linear_reduce_kernel<Bf16>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, part, c.splits, M, Nn, Y, ldy);
    return hipGetLastError();
}

// Estimated time of the tiled kernel with tiles of rows x cols: rounds of 256 workgroups, each
// round a fixed cost plus its slabs (measured per slab: 1.57 us for 256 x 256, 1.19 us for
// 256 x 192 (fitted over K = 256 ... 4096), 0.91 us for 256 x 128, 0.76 us for 128 x 192, 0.6 us for 128 x 128).
static double tiled_estimate_us(int M, int Nn, int K, int rows, int cols)
{
    const int64_t tiles = int64_t((M + rows - 1) / rows) * ((Nn + cols - 1) / cols);
    const int S = K / kTileK;
    const double per_round = cols == 256   ? 11. + 1.57 * S
                             : cols == 192 ? (rows == 256 ? 7.8 + 1.19 * S : 3.6 + 0.76 * S)
                             : rows == 256 ? 8. + 0.91 * S
                                           : 4. + 0.6 * S;
    return 2.5 + double((tiles + 255) / 256) * per_round;
}

// Tile of the tiled kernel for a problem (*rows x returned columns), 0 for the streaming kernel.
// The tiled kernel pays off once its tiles occupy most of the chip (measured break-even near
// 150 tiles of 256 x 256, 160 of the smaller ones); below that the streaming kernel (several
// batch tiles per weight block, K splits) is faster.  Between 256 x 256 and 256 x 128 the
// round estimate decides: the narrow tile does 13 % less per compute unit but wastes less of a
// ragged last round.  128 x 128 is for outputs too small for either (measured on every such
// prefill shape of the 8B model: level with or up to 30 % ahead of the streaming kernel, and
// behind the larger tiles wherever those qualify).
// The two 192-wide tiles replace that choice where their estimate is 5 % or more below its
// estimate (outputs they cut into a whole number of rounds: measured 5-17 % faster on the six such
// prefill shapes of the 8B model, never chosen on the other 43).
static int tiled_base_choice(int M, int Nn, int K, int *rows)
{
    *rows = 256;
    if (M < 256) return 0;
    const int64_t tm = (M + 255) / 256;
    const int64_t t256 = tm * ((Nn + 255) / 256), t128c = tm * ((Nn + 127) / 128);
    const int64_t t128s = int64_t((M + 127) / 128) * ((Nn + 127) / 128);
    const bool ok256 = M > 256 && t256 >= 160, ok128c = M >= 256 && t128c >= 160;
    if (ok256 && ok128c)
        return tiled_estimate_us(M, Nn, K, 256, 128) < 0.97 * tiled_estimate_us(M, Nn, K, 256, 256) ? 128 : 256;
    if (ok256) return 256;
    if (ok128c) return 128;
    // with fewer than four row tiles the streaming kernel stays ahead, and so it does with 160 to 191
    // tiles on long reductions, which it splits over the idle compute units (160 tiles of 5120 columns
    // at M = 512: tiled 11-17 % ahead for K = 640 ... 3456, 4 % behind at K = 5120, 26 % at K = 13824)
    if (M >= 512 && (t128s >= 192 || (t128s >= 160 && K <= 4096))) {
        *rows = 128;
        return 128;
    }
    return 0;
}

int nts_linear_use_tiled(int M, int Nn, int K, int *rows)
{
    const int base = tiled_base_choice(M, Nn, K, rows);
    if (!base) return 0;
    double best = 0.95 * tiled_estimate_us(M, Nn, K, *rows, base);
    int cols = base;
    const int64_t tn = (Nn + 191) / 192;
    for (int r = 256; r >= 128; r -= 128) {
        if (r == 256 ? M <= 256 : M < 512) continue;     // the same batch sizes as the other tiles of that height
        if (int64_t((M + r - 1) / r) * tn < 160) continue;
        const double t = tiled_estimate_us(M, Nn, K, r, 192);
        if (t < best) {
            best = t;
            cols = 192;
            *rows = r;
        }
    }
    return cols;
}

// Every configuration that may be fastest for a problem, for nts_shard_linear_tune to time: the
// streaming kernel's variants with each K split that is valid for them, the decode kernel's
// (row blocks, wavefronts per K range, K split) combinations for M <= 16, and the tiled kernel
// in its five tile shapes for M >= 128.  Each gets the same estimate nts_linear_stream_config uses
// (the tiled kernel: tiled_estimate_us); the list is cut to those within `slack` of
// the smallest estimate, sorted by estimate, at most `max_out`.  The configuration
// nts_shard_linear uses by default is always first.
int nts_linear_candidates(int M, int Nn, int K, double slack, NtsLinearCand *out, int max_out)
{
    std::vector<NtsLinearCand> all;
    const int rows = M < 256 ? M : 256;
    const int mt_min = rows <= 32 ? 1 : rows <= 64 ? 2 : rows <= 96 ? 3 : rows <= 128 ? 4 : rows <= 192 ? 6 : 8;
    const int n_slabs = K / kStrK;
    const double out_elems = double(M) * Nn;
    const double hbm_us = double(Nn) * K * 2. / 6.1e6;
    NtsLinearCand def;
    def.tiled = nts_linear_use_tiled(M, Nn, K, &def.tiled_rows);
    def.cfg = nts_linear_stream_config(M, Nn, K);
    if (def.tiled) def.cfg.splits = 1;
    def.est_us = 0.;
    for (const StreamVariant &v : kStreamVariants) {
        if (v.mt > mt_min || (v.mt == 1 && mt_min > 1)) continue;
        const int tiles_m = (M + 32 * v.mt - 1) / (32 * v.mt);
        const int lds_fit = (160 * 1024) / (3 * 32 * v.mt * kStrPitch);
        const int per_cu = 4 / v.cw < lds_fit ? 4 / v.cw : lds_fit;
        const int64_t wgs = int64_t(tiles_m) * ((Nn + 32 * v.cw - 1) / (32 * v.cw));
        for (int splits = 1; splits <= 32 && splits <= (n_slabs >= 4 ? n_slabs / 4 : 1); ++splits) {
            const int sps = (n_slabs + splits - 1) / splits;
            if ((n_slabs + sps - 1) / sps != splits) continue;
            if (splits > 1 && out_elems * splits * 4 > double(int64_t(512) << 20)) break;
            const int64_t total = wgs * splits;
            const int64_t rounds = (total + 255) / 256, seq_rounds = (total + 256 * per_cu - 1) / (256 * per_cu);
            const double cu_us = double(rounds) * sps * v.slab_us;
            double t = 2.5 + (cu_us > hbm_us ? cu_us : hbm_us) + v.round_us * double(seq_rounds) +
                       0.7 * double(rounds - seq_rounds);
            if (splits > 1) t += 2.5 + out_elems * splits * 8. / 4.0e6;
            NtsLinearCand c;
            c.tiled = 0;
            c.cfg.mt = v.mt;
            c.cfg.cw = v.cw;
            c.cfg.rt = 1;
            c.cfg.splits = splits;
            c.cfg.ks = 0;
            c.cfg.nsets = v.mt <= 4 ? 4 : 3;
            if (v.cw == 1 && v.mt == 1) c.cfg.nsets = 8;
            c.est_us = t;
            all.push_back(c);
        }
    }
    if (M <= 16) {
        const double bytes = double(Nn) * K * 2.;
        for (int rb = 1; rb <= 2; ++rb)
            for (int ks = 2 * rb; ks <= 4; ks *= 2)
                for (int splits = 1; splits <= 4; splits *= 2) {
                    const int sps = (n_slabs + splits - 1) / splits;
                    if ((n_slabs + sps - 1) / sps != splits) continue;
                    const int spw = sps / ks;
                    if (spw < 4) continue;
                    if (splits > 1 && out_elems * splits * 4 > double(int64_t(512) << 20)) continue;
                    const int64_t wgs = int64_t((Nn + 16 * rb - 1) / (16 * rb)) * splits;
                    const int per_cu = 12 / ks;
                    const int64_t rounds = (wgs + 256 * per_cu - 1) / (256 * per_cu);
                    const int64_t wg_cu = (wgs + 255) / 256;
                    double rate = 10. * double(ks * (wg_cu < per_cu ? wg_cu : per_cu));
                    const double cap = 26. - 0.4 * M;
                    if (rate > cap) rate = cap;
                    if (wg_cu > 1 && rate > 22.) rate = 22.;
                    double stream_us = bytes / double(wgs) * double(wg_cu) / (rate * 1e3);
                    if (stream_us < hbm_us) stream_us = hbm_us;
                    double t = 2.5 + 1.0 * double(rounds) + stream_us + 0.05 * M + (spw < 16 ? 0.08 * (16 - spw) : 0.);
                    if (splits > 1) t += 2.5 + out_elems * splits * 8. / 4.0e6;
                    NtsLinearCand c;
                    c.tiled = 0;
                    c.cfg.mt = 1;
                    c.cfg.cw = 4;
                    c.cfg.ks = ks;
                    c.cfg.rt = rb;
                    c.cfg.splits = splits;
                    c.cfg.nsets = rb == 1 ? 8 : 6;
                    c.est_us = t;
                    all.push_back(c);
                }
    }
    static const int kTiles[5][2] = {{256, 256}, {256, 192}, {256, 128}, {128, 192}, {128, 128}};
    for (const auto &t : kTiles) {
        if (M < t[0]) continue;
        NtsLinearCand c;
        c.tiled = t[1];
        c.tiled_rows = t[0];
        c.cfg = def.cfg;
        c.cfg.splits = 1;
        c.est_us = tiled_estimate_us(M, Nn, K, t[0], t[1]);
        all.push_back(c);
    }
    auto same = [](const NtsLinearCand &a, const NtsLinearCand &b) {
        if (a.tiled != b.tiled || (a.tiled && a.tiled_rows != b.tiled_rows)) return false;
        if (a.tiled) return true;
        if (a.cfg.ks != b.cfg.ks || a.cfg.rt != b.cfg.rt || a.cfg.splits != b.cfg.splits || a.cfg.nsets != b.cfg.nsets)
            return false;
        return a.cfg.ks > 0 || (a.cfg.mt == b.cfg.mt && a.cfg.cw == b.cfg.cw);   // the decode kernel has no tile fields
    };
    double best = 0.;
    for (const NtsLinearCand &c : all) {
        if (same(c, def)) def.est_us = c.est_us;
        if (best == 0. || c.est_us < best) best = c.est_us;
    }
    std::sort(all.begin(), all.end(), [](const NtsLinearCand &a, const NtsLinearCand &b) { return a.est_us < b.est_us; });
    int n = 0;
    if (max_out > 0) out[n++] = def;
    for (const NtsLinearCand &c : all) {
        if (n >= max_out) break;
        if (same(c, def) || c.est_us > slack * best) continue;
        out[n++] = c;
    }
    return n;
}

template <class E, int NB, int MA>
static hipError_t launch_tiled_one(const uint16_t *X, int64_t ldx, const uint16_t *A, int64_t lda, uint16_t *Y,
                                   int64_t ldy, int M, int Nn, int K, hipStream_t st)
{
    constexpr int rows = 64 * MA, cols = 64 * NB, lds_bytes = 2 * (rows + cols) * kPitch;
    static std::atomic<uint64_t> configured{0};
    const hipError_t ea = allow_dynamic_lds(configured, reinterpret_cast<const void *>(nts_linear_tiled_kernel<E, NB, MA>), lds_bytes);
    if (ea != hipSuccess) return ea;
    const int tiles_m = (M + rows - 1) / rows, tiles_n = (Nn + cols - 1) / cols;
    const int sups = ((tiles_m + kSupM - 1) / kSupM) * ((tiles_n + kSupN - 1) / kSupN);
    const dim3 grid(unsigned((sups + 7) / 8) * 8u * kSupM * kSupN), block(256);
    hipLaunchKernelGGL((nts_linear_tiled_kernel<E, NB, MA>), grid, block, lds_bytes, st, X, ldx, A, lda, Y, ldy, M, Nn, K);
    return hipGetLastError();
}

hipError_t nts_launch_linear_tiled(const uint16_t *X, int64_t ldx, const uint16_t *A, int64_t lda,
                                   uint16_t *Y, int64_t ldy, int M, int Nn, int K, int tile_rows, int tile_cols,
                                   bool f16, hipStream_t st)
{
#define NTS_TILED(NB, MA)                                                                              \
    return f16 ? launch_tiled_one<F16, NB, MA>(X, ldx, A, lda, Y, ldy, M, Nn, K, st)                   \
               : launch_tiled_one<Bf16, NB, MA>(X, ldx, A, lda, Y, ldy, M, Nn, K, st);
    if (tile_cols == 192) {
        if (tile_rows == 128) NTS_TILED(3, 2)
        NTS_TILED(3, 4)
    }
    if (tile_rows == 128) NTS_TILED(2, 2)
    if (tile_cols == 128) NTS_TILED(2, 4)
    NTS_TILED(4, 4)
#undef NTS_TILED
}
