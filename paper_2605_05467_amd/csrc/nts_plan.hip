// Planning step on the GPU: request list + page tables -> one slot per token.
//
// The metadata exchanged before a migration names requests, their context
// lengths and KV heads (paper Sec. 3.2.2); with paged KV each request also
// brings a page table.  Token t of request r lives in slot
// pages[r][t / p] * p + t % p.  Flattening and validation are data parallel
// over tokens (blockIdx.y picks the source or the destination table); the two
// prefix sums over requests (a few hundred entries) are done by the host in
// nts_plan_create.
#include "nts_internal.h"

namespace {

__global__ __launch_bounds__(256) void nts_flatten_kernel(
    const int32_t *__restrict__ tok_off, const int32_t *__restrict__ pg_off, int n_req, uint32_t T,
    int p, NtsFlattenSide src, NtsFlattenSide dst, int32_t *__restrict__ err)
{
    const uint32_t j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= T) return;
    const NtsFlattenSide &sd = blockIdx.y == 0 ? src : dst;
    // last request r with tok_off[r] <= j (requests of length zero are skipped)
    int lo = 0, hi = n_req;            // invariant: tok_off[lo] <= j < tok_off[hi]
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (uint32_t(tok_off[mid]) <= j) lo = mid; else hi = mid;
    }
    const uint32_t t = j - uint32_t(tok_off[lo]);
    const int32_t page = sd.pages[pg_off[lo] + int32_t(t / uint32_t(p))];
    if (page < 0 || int64_t(page) >= sd.n_pool_pages) {
        atomicOr(&err[0], 1);
        sd.slots[j] = 0;
        return;
    }
    const int64_t slot = int64_t(page) * p + int64_t(t % uint32_t(p));
    sd.slots[j] = int32_t(slot);
    if (sd.bitmap) {
        const uint32_t bit = 1u << (uint32_t(slot) & 31u);
        const uint32_t old = atomicOr(&sd.bitmap[slot >> 5], bit);
        if (old & bit) atomicOr(&err[1], 1);
    }
}

// Run detection (plan flag NTS_DETECT_RUNS): token j starts a run unless it sits in the slot
// after token j-1's on the source side and on the destination side.  With small pages a
// request's KV is scattered over many regions, with a contiguous per-request layout over few
// (paper Sec. 3.2.2); a run is one contiguous region per (layer, K|V) when a fragment is a
// whole token row.  Three launches, no atomics, so the list comes out in token order:
// heads per 256-token block, exclusive scan of the block counts by one workgroup, then every
// head writes its token index at (block offset + rank inside the block by ballot).
__device__ __forceinline__ bool nts_run_head(const int32_t *__restrict__ ss, const int32_t *__restrict__ ds,
                                             uint32_t j)
{
    return j == 0 || ss[j] != ss[j - 1] + 1 || ds[j] != ds[j - 1] + 1;
}

__global__ __launch_bounds__(256) void nts_run_count_kernel(const int32_t *__restrict__ ss,
                                                            const int32_t *__restrict__ ds, uint32_t T,
                                                            int32_t *__restrict__ block_count)
{
    const uint32_t j = blockIdx.x * 256u + threadIdx.x;
    const int n = __syncthreads_count(j < T && nts_run_head(ss, ds, j));
    if (threadIdx.x == 0) block_count[blockIdx.x] = n;
}

// One 256-thread workgroup: counts[0..n) -> exclusive prefix sums in place; returns the total
// (to every thread).  `part` and `carry` are the caller's shared memory.
__device__ __forceinline__ int32_t nts_scan_in_place(int32_t *__restrict__ counts, uint32_t n, int32_t *part,
                                                     int32_t *carry)
{
    if (threadIdx.x == 0) *carry = 0;
    __syncthreads();
    for (uint32_t base = 0; base < n; base += 256u) {
        const uint32_t i = base + threadIdx.x;
        const int32_t v = i < n ? counts[i] : 0;
        part[threadIdx.x] = v;
        __syncthreads();
        for (int d = 1; d < 256; d <<= 1) {                 // inclusive scan of the 256 entries
            const int32_t add = int(threadIdx.x) >= d ? part[threadIdx.x - d] : 0;
            __syncthreads();
            part[threadIdx.x] += add;
            __syncthreads();
        }
        const int32_t before = *carry;
        if (i < n) counts[i] = before + part[threadIdx.x] - v;
        __syncthreads();
        if (threadIdx.x == 255) *carry = before + part[255];
        __syncthreads();
    }
    return *carry;
}

// one workgroup: block_count[0..nb) -> exclusive offsets in place; the total goes to *n_runs and
// the closing entry run_start[total] = T is written here
__global__ __launch_bounds__(256) void nts_run_scan_kernel(int32_t *__restrict__ block_count, uint32_t nb,
                                                           uint32_t T, int32_t *__restrict__ run_start,
                                                           int32_t *__restrict__ n_runs)
{
    __shared__ int32_t part[256];
    __shared__ int32_t carry;
    const int32_t total = nts_scan_in_place(block_count, nb, part, &carry);
    if (threadIdx.x == 0) {
        run_start[total] = int32_t(T);
        *n_runs = total;
    }
}

__global__ __launch_bounds__(256) void nts_run_scatter_kernel(const int32_t *__restrict__ ss,
                                                              const int32_t *__restrict__ ds, uint32_t T,
                                                              const int32_t *__restrict__ block_off,
                                                              int32_t *__restrict__ run_start)
{
    __shared__ int32_t wave_heads[4];
    const uint32_t j = blockIdx.x * 256u + threadIdx.x;
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const bool head = j < T && nts_run_head(ss, ds, j);
    const unsigned long long m = __ballot(head);
    if (lane == 0) wave_heads[wv] = __popcll(m);
    __syncthreads();
    if (!head) return;
    int32_t at = block_off[blockIdx.x] + __popcll(m & ((1ull << lane) - 1ull));
    for (int w = 0; w < wv; ++w) at += wave_heads[w];
    run_start[at] = int32_t(j);
}

// Tokens ranked by destination slot (plan flag NTS_ORDER_BY_DST).  Destination slots are
// distinct and the uniqueness bitmap has exactly their bits set, so the rank of a token among
// the destination slots is the number of set bits below its own: popcounts per bitmap word,
// scanned within blocks of 256 words (this kernel), across blocks (one workgroup), and a
// scatter of both slot lists into rank order.  The pool-to-pool kernel walks the tokens in
// that order: its writes then sweep the destination pool upwards instead of landing at random.
__global__ __launch_bounds__(256) void nts_rank_count_kernel(const uint32_t *__restrict__ bitmap, uint32_t n_words,
                                                             int32_t *__restrict__ word_prefix,
                                                             int32_t *__restrict__ block_count)
{
    __shared__ int32_t part[256];
    const uint32_t w = blockIdx.x * 256u + threadIdx.x;
    const int32_t v = w < n_words ? __popc(bitmap[w]) : 0;
    part[threadIdx.x] = v;
    __syncthreads();
    for (int d = 1; d < 256; d <<= 1) {                     // inclusive scan of the 256 popcounts
        const int32_t add = int(threadIdx.x) >= d ? part[threadIdx.x - d] : 0;
        __syncthreads();
        part[threadIdx.x] += add;
        __syncthreads();
    }
    if (w < n_words) word_prefix[w] = part[threadIdx.x] - v;   // set bits before word w inside its block
    if (threadIdx.x == 255) block_count[blockIdx.x] = part[255];
}

// one workgroup: block_count[0..nb) -> exclusive offsets in place
__global__ __launch_bounds__(256) void nts_rank_scan_kernel(int32_t *__restrict__ block_count, uint32_t nb)
{
    __shared__ int32_t part[256];
    __shared__ int32_t carry;
    (void)nts_scan_in_place(block_count, nb, part, &carry);
}

__global__ __launch_bounds__(256) void nts_rank_scatter_kernel(const int32_t *__restrict__ ss,
                                                               const int32_t *__restrict__ ds, uint32_t T,
                                                               const uint32_t *__restrict__ bitmap,
                                                               const int32_t *__restrict__ word_prefix,
                                                               const int32_t *__restrict__ block_off,
                                                               int32_t *__restrict__ ss_sorted,
                                                               int32_t *__restrict__ ds_sorted)
{
    const uint32_t j = blockIdx.x * 256u + threadIdx.x;
    if (j >= T) return;
    const uint32_t d = uint32_t(ds[j]), w = d >> 5;
    const uint32_t rank = uint32_t(block_off[w >> 8]) + uint32_t(word_prefix[w]) +
                          uint32_t(__popc(bitmap[w] & ((1u << (d & 31u)) - 1u)));
    if (rank < T) {                                         // always, for distinct slots inside the pool
        ss_sorted[rank] = ss[j];
        ds_sorted[rank] = int32_t(d);
    }
}

}  // namespace

hipError_t nts_launch_rank_by_dst(const int32_t *d_sslot, const int32_t *d_dslot, uint32_t T,
                                  const uint32_t *d_bitmap, uint32_t n_words, int32_t *d_word_prefix,
                                  int32_t *d_block_count, int32_t *d_ss_sorted, int32_t *d_ds_sorted, hipStream_t st)
{
    if (T == 0 || n_words == 0) return hipSuccess;
    const uint32_t nb = (n_words + 255u) / 256u;
    hipLaunchKernelGGL(nts_rank_count_kernel, dim3(nb), dim3(256), 0, st, d_bitmap, n_words, d_word_prefix, d_block_count);
    hipLaunchKernelGGL(nts_rank_scan_kernel, dim3(1), dim3(256), 0, st, d_block_count, nb);
    hipLaunchKernelGGL(nts_rank_scatter_kernel, dim3((T + 255u) / 256u), dim3(256), 0, st, d_sslot, d_dslot, T, d_bitmap,
                       d_word_prefix, d_block_count, d_ss_sorted, d_ds_sorted);
    return hipGetLastError();
}

hipError_t nts_launch_detect_runs(const int32_t *d_sslot, const int32_t *d_dslot, uint32_t T,
                                  int32_t *d_block_count, int32_t *d_run_start, int32_t *d_n_runs,
                                  hipStream_t st)
{
    if (T == 0) return hipSuccess;
    const uint32_t nb = (T + 255u) / 256u;
    hipLaunchKernelGGL(nts_run_count_kernel, dim3(nb), dim3(256), 0, st, d_sslot, d_dslot, T, d_block_count);
    hipLaunchKernelGGL(nts_run_scan_kernel, dim3(1), dim3(256), 0, st, d_block_count, nb, T, d_run_start, d_n_runs);
    hipLaunchKernelGGL(nts_run_scatter_kernel, dim3(nb), dim3(256), 0, st, d_sslot, d_dslot, T, d_block_count,
                       d_run_start);
    return hipGetLastError();
}

hipError_t nts_launch_flatten(const int32_t *d_tok_off, const int32_t *d_pg_off, int n_req, uint32_t T,
                              int p, const NtsFlattenSide &src, const NtsFlattenSide &dst,
                              int32_t *d_err, hipStream_t st)
{
    if (T == 0) return hipSuccess;
    const dim3 block(256), grid((T + 255u) / 256u, 2);
    hipLaunchKernelGGL(nts_flatten_kernel, grid, block, 0, st, d_tok_off, d_pg_off, n_req, T, p, src, dst, d_err);
    return hipGetLastError();
}
