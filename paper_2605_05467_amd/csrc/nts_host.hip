// Host-side integer arithmetic of the library (see nts_host.h).  No GPU code and no
// GPU runtime calls in this file: it is also compiled as plain C++ for the sanitizer run.
#include "nts_host.h"

#include <algorithm>

namespace {
inline int64_t align_up(int64_t x, int64_t a) { return (x + a - 1) / a * a; }
}  // namespace

int nts_host_route(int H, int Ns, int rs, int Nd, int rd, int *src_head_off, int *dst_head_off, int *w)
{
    if (!src_head_off || !dst_head_off || !w) return NTS_EINVAL;
    if (H <= 0 || Ns <= 0 || Nd <= 0 || H % Ns || H % Nd) return NTS_EINVAL;
    if (rs < 0 || rs >= Ns || rd < 0 || rd >= Nd) return NTS_EINVAL;
    const int hs = H / Ns, hd = H / Nd;
    const int s_lo = rs * hs, s_hi = s_lo + hs;
    const int d_lo = rd * hd, d_hi = d_lo + hd;
    const int lo = s_lo > d_lo ? s_lo : d_lo;
    const int hi = s_hi < d_hi ? s_hi : d_hi;
    if (hi <= lo) {
        *src_head_off = *dst_head_off = *w = 0;
        return NTS_OK;
    }
    *src_head_off = lo - s_lo;
    *dst_head_off = lo - d_lo;
    *w = hi - lo;
    return NTS_OK;
}

int64_t nts_host_max_frags_per_launch(int64_t frag_bytes, int32_t vec)
{
    const int64_t V = frag_bytes / vec;
    const int64_t n = ((int64_t(1) << 31) - kNtsLanes) / V;
    return n < 1 ? 1 : n;
}

int nts_host_plan_geometry(const nts_desc *d, NtsGeometry *g, const char **why)
{
    const char *dummy;
    if (!why) why = &dummy;
#define NTS_BAD(msg) do { *why = (msg); return NTS_EINVAL; } while (0)
    if (!d || !g) NTS_BAD("null descriptor or output");
    if (d->L <= 0 || d->L > NTS_MAX_LAYERS) NTS_BAD("L outside 1..NTS_MAX_LAYERS");
    if (d->D <= 0 || d->page_size <= 0 || d->Hs <= 0 || d->Hd <= 0) NTS_BAD("D, page_size, Hs and Hd must be positive");
    if (d->D > (1 << 20) || d->Hs > (1 << 16) || d->Hd > (1 << 16)) NTS_BAD("D above 2^20 or more than 65536 heads");
    if (d->elem_bytes != 1 && d->elem_bytes != 2 && d->elem_bytes != 4) NTS_BAD("elem_bytes must be 1, 2 or 4");
    if (d->w <= 0) NTS_BAD("w must be positive");
    if (d->src_head_off < 0 || d->src_head_off > d->Hs - d->w) NTS_BAD("moved heads outside the source's heads");
    if (d->dst_head_off < 0 || d->dst_head_off > d->Hd - d->w) NTS_BAD("moved heads outside the destination's heads");
    if (d->n_req < 0 || (d->n_req > 0 && !d->ctx_len)) NTS_BAD("bad request list");
    if ((d->flags & NTS_ORDER_BY_DST) && !(d->flags & NTS_VALIDATE_UNIQUE_DST))
        NTS_BAD("NTS_ORDER_BY_DST needs NTS_VALIDATE_UNIQUE_DST (the ranking relies on distinct destination slots)");
    const int p = d->page_size;
    if (d->S_src <= 0 || d->S_dst <= 0 || d->S_src % p || d->S_dst % p)
        NTS_BAD("pool capacities must be positive multiples of the page size");
    if (d->S_src > INT32_MAX || d->S_dst > INT32_MAX) NTS_BAD("pool capacity above 2^31-1 slots");

    const int64_t head_bytes = int64_t(d->D) * d->elem_bytes;
    const int64_t frag = head_bytes * d->w;
    const int64_t src_row = head_bytes * d->Hs, dst_row = head_bytes * d->Hd;
    const int64_t src_stride = d->src_token_stride ? d->src_token_stride : src_row;
    const int64_t dst_stride = d->dst_token_stride ? d->dst_token_stride : dst_row;
    if (src_stride < src_row || dst_stride < dst_row) NTS_BAD("token stride smaller than a token row");
    // keeps slot * stride, the pool spans and the payload size inside 64 bits
    if (src_stride > (int64_t(1) << 30) || dst_stride > (int64_t(1) << 30)) NTS_BAD("token stride above 1 GiB");
    const int64_t so = head_bytes * d->src_head_off, dof = head_bytes * d->dst_head_off;
    int vec = 16;
    while (vec >= 4 && (frag % vec || src_stride % vec || dst_stride % vec || so % vec || dof % vec)) vec >>= 1;
    if (vec < 4) NTS_BAD("fragment size, head offsets and strides must be multiples of 4 bytes");

    // prefix sums over requests
    try {
        g->tok_off.assign(size_t(d->n_req) + 1, 0);
        g->pg_off.assign(size_t(d->n_req) + 1, 0);
    } catch (...) {
        *why = "host allocation failed";
        return NTS_ENOMEM;
    }
    int64_t T = 0, NP = 0;
    for (int r = 0; r < d->n_req; ++r) {
        const int32_t n = d->ctx_len[r];
        if (n < 0) NTS_BAD("negative context length");
        g->tok_off[size_t(r)] = int32_t(T);
        g->pg_off[size_t(r)] = int32_t(NP);
        T += n;
        NP += (int64_t(n) + p - 1) / p;
        if (T > INT32_MAX) NTS_BAD("more than 2^31-1 tokens");
    }
    g->tok_off[size_t(d->n_req)] = int32_t(T);
    g->pg_off[size_t(d->n_req)] = int32_t(NP);
    if (T > 0 && (!d->src_pages || !d->dst_pages)) NTS_BAD("null page table");

    g->src_stride = src_stride;
    g->dst_stride = dst_stride;
    g->frag_bytes = frag;
    g->vec = vec;
    g->T = T;
    g->NP = NP;
    g->F = T * 2 * d->L;
    if (g->F > INT64_MAX / frag) NTS_BAD("payload size does not fit 64 bits");
    g->X = g->F * frag;
    const int64_t B = d->staging_bytes > 0 ? d->staging_bytes : int64_t(NTS_DEFAULT_STAGING_BYTES);
    int64_t cf = B / frag;
    if (cf < 1) cf = 1;
    const int64_t cf_max = nts_host_max_frags_per_launch(frag, vec) / 2;   // a stage launch packs one chunk and unpacks another
    if (cf > cf_max) cf = cf_max > 1 ? cf_max : 1;
    g->chunk_frags = cf;
    g->chunk_bytes = cf * frag;
    g->n_chunks = (g->F + cf - 1) / cf;
    return NTS_OK;
#undef NTS_BAD
}

int nts_host_chunk_range(int64_t F, int64_t chunk_frags, int64_t n_chunks, int64_t k, int64_t *q0, int64_t *n)
{
    if (k < 0 || k >= n_chunks) return NTS_EINVAL;
    *q0 = k * chunk_frags;
    *n = F - *q0 < chunk_frags ? F - *q0 : chunk_frags;
    return NTS_OK;
}

int nts_host_alias_sweep(std::vector<NtsByteRange> &ranges, uintptr_t stg, int64_t stg_bytes, const char **why)
{
    // Sort by start and sweep, remembering how far the sources and the destinations seen so far reach.
    std::sort(ranges.begin(), ranges.end(), [](const NtsByteRange &x, const NtsByteRange &y) { return x.lo < y.lo; });
    uintptr_t reach[2] = {0, 0};             // 0: nothing seen yet on that side
    for (const NtsByteRange &r : ranges) {
        if (reach[1 - r.is_dst] && r.lo < reach[1 - r.is_dst]) {
            if (why) *why = "a destination pool of the batch overlaps a source pool of the batch";
            return NTS_EALIAS;
        }
        if (r.lo < stg + uintptr_t(stg_bytes) && stg < r.hi) {
            if (why) *why = "staging area overlaps a pool";
            return NTS_EALIAS;
        }
        if (!reach[r.is_dst] || r.hi > reach[r.is_dst]) reach[r.is_dst] = r.hi;
    }
    return NTS_OK;
}

int64_t nts_host_batch_staging_bytes(const int64_t *chunk_bytes, int n)
{
    int64_t largest = 0;
    for (int i = 0; i < n; ++i)
        if (chunk_bytes[i] > largest) largest = chunk_bytes[i];
    return 2 * align_up(largest, 16);
}
