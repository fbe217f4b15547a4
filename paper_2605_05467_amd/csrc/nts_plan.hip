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

}  // namespace

hipError_t nts_launch_flatten(const int32_t *d_tok_off, const int32_t *d_pg_off, int n_req, uint32_t T,
                              int p, const NtsFlattenSide &src, const NtsFlattenSide &dst,
                              int32_t *d_err, hipStream_t st)
{
    if (T == 0) return hipSuccess;
    const dim3 block(256), grid((T + 255u) / 256u, 2);
    hipLaunchKernelGGL(nts_flatten_kernel, grid, block, 0, st, d_tok_off, d_pg_off, n_req, T, p, src, dst, d_err);
    return hipGetLastError();
}
