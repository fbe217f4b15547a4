// C ABI of the KV-migration library: contexts, routing, planning, run calls.
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <new>
#include <vector>

#include "nts_host.h"
#include "nts_internal.h"

// Staging area of nts_run_migrate_static: device memory that exists from the moment the
// library is loaded, one copy per GPU.  Host code never uses this name as an address: each
// context asks the runtime for its device's copy once (nts_init) and passes that pointer on.
static __device__ __align__(256) unsigned char scratch[NTS_STATIC_STAGING_BYTES];

namespace {

struct DeviceGuard {
    int prev = -1;
    bool ok = true;
    explicit DeviceGuard(int dev)
    {
        if (hipGetDevice(&prev) != hipSuccess) prev = -1;
        if (prev != dev) ok = hipSetDevice(dev) == hipSuccess;
    }
    ~DeviceGuard()
    {
        if (prev >= 0) (void)hipSetDevice(prev);
    }
};

int fail(nts_ctx *ctx, int code, const char *what)
{
    if (ctx) ctx->err = what;
    return code;
}

int fail_hip(nts_ctx *ctx, hipError_t e, const char *where)
{
    if (ctx) {
        char buf[256];
        snprintf(buf, sizeof buf, "%s: %s", where, hipGetErrorString(e));
        ctx->err = buf;
    }
    (void)hipGetLastError();
    return NTS_EHIP;
}

#define NTS_HIP(ctx, call)                                         \
    do {                                                           \
        hipError_t e_ = (call);                                    \
        if (e_ != hipSuccess) return fail_hip((ctx), e_, #call);   \
    } while (0)

inline int64_t align_up(int64_t x, int64_t a) { return (x + a - 1) / a * a; }

int fill_tab(const nts_plan *pl, const void *const *ptrs, NtsLayerTab &tab)
{
    const int n = 2 * pl->L;
    for (int i = 0; i < n; ++i) {
        if (!ptrs[i]) return NTS_EINVAL;
        if (reinterpret_cast<uintptr_t>(ptrs[i]) % uintptr_t(pl->vec)) return NTS_EINVAL;
        tab.p[i] = static_cast<char *>(const_cast<void *>(ptrs[i]));
    }
    for (int i = n; i < NTS_MAX_LAYER_PTRS; ++i) tab.p[i] = nullptr;
    return NTS_OK;
}

// Remember that `pl` has work on `st`: nts_plan_free orders that work before any reuse of the plan's block.
void note_stream(nts_plan *pl, hipStream_t st)
{
    for (int i = 0; i < pl->n_used_streams; ++i)
        if (pl->used_streams[i] == st) return;
    if (pl->n_used_streams < nts_plan::kMaxStreams) pl->used_streams[pl->n_used_streams++] = st;
    else pl->more_streams = true;
}

bool overlaps(const char *a, int64_t na, const char *b, int64_t nb)
{
    return a < b + nb && b < a + na;
}

}  // namespace

extern "C" {

const char *nts_strerror(int status)
{
    switch (status) {
    case NTS_OK: return "ok";
    case NTS_EINVAL: return "invalid argument";
    case NTS_ERANGE: return "page id outside its pool";
    case NTS_EDUP: return "duplicate destination slot";
    case NTS_EALIAS: return "source and destination overlap";
    case NTS_ENOMEM: return "out of memory";
    case NTS_EHIP: return "HIP error";
    default: return "unknown status";
    }
}

const char *nts_last_error(const nts_ctx *ctx) { return ctx ? ctx->err.c_str() : "no context"; }

int nts_init(int device_id, nts_ctx **out)
{
    if (!out) return NTS_EINVAL;
    *out = nullptr;
    int n = 0;
    if (hipGetDeviceCount(&n) != hipSuccess || device_id < 0 || device_id >= n) {
        (void)hipGetLastError();
        return NTS_EHIP;
    }
    nts_ctx *ctx = new (std::nothrow) nts_ctx;
    if (!ctx) return NTS_ENOMEM;
    ctx->device = device_id;
    DeviceGuard guard(device_id);
    hipError_t e = guard.ok ? hipSuccess : hipErrorInvalidDevice;
    if (e == hipSuccess) e = hipStreamCreateWithFlags(&ctx->aux, hipStreamNonBlocking);
    for (int i = 0; i < nts_ctx::kSpares && e == hipSuccess; ++i)
        e = hipEventCreateWithFlags(&ctx->spare[i].ev, hipEventDisableTiming);
    // this device's copy of the static staging area (the device is current here)
    if (e == hipSuccess) e = hipGetSymbolAddress(&ctx->static_staging, HIP_SYMBOL(scratch));
    if (e != hipSuccess) {
        nts_free(ctx);
        (void)hipGetLastError();
        return NTS_EHIP;
    }
    *out = ctx;
    return NTS_OK;
}

int nts_free(nts_ctx *ctx)
{
    if (!ctx) return NTS_OK;
    if (ctx->n_plans != 0) return fail(ctx, NTS_EINVAL, "plans of this context are still alive");
    DeviceGuard guard(ctx->device);
    if (ctx->aux) {
        (void)hipStreamSynchronize(ctx->aux);
        (void)hipStreamDestroy(ctx->aux);
    }
    (void)hipDeviceSynchronize();
    for (int i = 0; i < nts_ctx::kSpares; ++i) {
        if (ctx->spare[i].ptr) (void)hipFree(ctx->spare[i].ptr);
        if (ctx->spare[i].ev) (void)hipEventDestroy(ctx->spare[i].ev);
    }
    if (ctx->h_pinned) (void)hipHostFree(ctx->h_pinned);
    delete ctx;
    return NTS_OK;
}

int nts_route(int H, int Ns, int rs, int Nd, int rd, int *src_head_off, int *dst_head_off, int *w)
{
    return nts_host_route(H, Ns, rs, Nd, rd, src_head_off, dst_head_off, w);
}

int nts_plan_create(nts_ctx *ctx, const nts_desc *d, nts_plan **out)
{
    if (!ctx) return NTS_EINVAL;
    if (!d || !out) return fail(ctx, NTS_EINVAL, "null descriptor or output");
    *out = nullptr;
    // validation, prefix sums over requests and chunk geometry: host arithmetic (nts_host.hip)
    NtsGeometry geo;
    const char *why = "";
    const int grc = nts_host_plan_geometry(d, &geo, &why);
    if (grc != NTS_OK) return fail(ctx, grc, why);
    const int p = d->page_size;
    const int64_t T = geo.T, NP = geo.NP;
    const std::vector<int32_t> &tok_off = geo.tok_off, &pg_off = geo.pg_off;

    nts_plan *pl = new (std::nothrow) nts_plan;
    if (!pl) return fail(ctx, NTS_ENOMEM, "host allocation failed");
    pl->ctx = ctx;
    pl->L = d->L; pl->D = d->D; pl->e = d->elem_bytes; pl->p = p;
    pl->Hs = d->Hs; pl->Hd = d->Hd;
    pl->src_head_off = d->src_head_off; pl->dst_head_off = d->dst_head_off; pl->w = d->w;
    pl->S_src = d->S_src; pl->S_dst = d->S_dst;
    pl->src_stride = geo.src_stride; pl->dst_stride = geo.dst_stride;
    pl->T = T;
    pl->has_runs = (d->flags & NTS_DETECT_RUNS) != 0;
    pl->F = geo.F;
    pl->frag_bytes = geo.frag_bytes;
    pl->X = geo.X;
    pl->vec = geo.vec;
    pl->chunk_frags = geo.chunk_frags;
    pl->chunk_bytes = geo.chunk_bytes;
    pl->n_chunks = geo.n_chunks;

    if (T == 0) {
        ++ctx->n_plans;
        *out = pl;
        return NTS_OK;
    }

    DeviceGuard guard(ctx->device);
    // device block: sslot | dslot | meta (tok_off | pg_off | src pages | dst pages) | bitmap | err |
    // run starts | per-block run counts (the last two only with NTS_DETECT_RUNS)
    // pinned host block: err readback (256 B) | meta
    const bool uniq = (d->flags & NTS_VALIDATE_UNIQUE_DST) != 0;
    const int64_t n_off = int64_t(d->n_req) + 1;
    const int64_t b_slots = align_up(T * 4, 256);
    const int64_t b_off = align_up(n_off * 4, 256);
    const int64_t b_pages = align_up(NP * 4, 256);
    const int64_t b_meta = 2 * b_off + 2 * b_pages;
    const int64_t bitmap_words = uniq ? (d->S_dst + 31) / 32 : 0;
    const int64_t b_bitmap = align_up(bitmap_words * 4, 256);
    const bool want_runs = (d->flags & NTS_DETECT_RUNS) != 0;
    const int64_t b_runs = want_runs ? align_up((T + 1) * 4, 256) + align_up(((T + 255) / 256) * 4, 256) : 0;
    // NTS_ORDER_BY_DST: per-word popcount prefix | per-block counts | both slot lists in rank order
    const bool want_order = (d->flags & NTS_ORDER_BY_DST) != 0;
    const int64_t b_wprefix = want_order ? align_up(bitmap_words * 4, 256) : 0;
    const int64_t b_wblocks = want_order ? align_up(((bitmap_words + 255) / 256) * 4, 256) : 0;
    const int64_t b_order = b_wprefix + b_wblocks + (want_order ? 2 * b_slots : 0);
    const int64_t total = 2 * b_slots + b_meta + b_bitmap + 256 + b_runs + b_order;

    hipError_t e = hipSuccess;
    if (ctx->h_pinned_bytes < size_t(b_meta + 256)) {
        if (ctx->h_pinned) (void)hipHostFree(ctx->h_pinned);
        ctx->h_pinned = nullptr;
        ctx->h_pinned_bytes = 0;
        const size_t want = size_t(b_meta + 256) * 2;
        e = hipHostMalloc(&ctx->h_pinned, want, hipHostMallocDefault);
        if (e != hipSuccess) {
            delete pl;
            (void)hipGetLastError();
            return fail(ctx, NTS_ENOMEM, "pinned host allocation failed");
        }
        ctx->h_pinned_bytes = want;
    }
    char *blk = nullptr;
    size_t blk_bytes = 0;
    int take = -1;                                   // oldest spare block that is large enough
    for (int i = 0; i < nts_ctx::kSpares; ++i)
        if (ctx->spare[i].ptr && ctx->spare[i].bytes >= size_t(total) &&
            (take < 0 || ctx->spare[i].age < ctx->spare[take].age))
            take = i;
    if (take >= 0 && ctx->spare[take].pending) {
        // still read by its previous owner's kernels?  Then rather start another block while a
        // slot is free, so that a loop of plans rotates through idle blocks and never waits.
        if (hipEventQuery(ctx->spare[take].ev) == hipSuccess) {
            ctx->spare[take].pending = false;
        } else {
            (void)hipGetLastError();
            for (int i = 0; i < nts_ctx::kSpares; ++i)
                if (!ctx->spare[i].ptr) {
                    take = -1;
                    break;
                }
        }
    }
    if (take >= 0) {
        nts_ctx::Spare &sp = ctx->spare[take];
        // kernels of the plan that owned the block must finish before it is overwritten
        if (sp.pending && (e = hipStreamWaitEvent(ctx->aux, sp.ev, 0)) != hipSuccess) {
            delete pl;
            return fail_hip(ctx, e, "hipStreamWaitEvent");
        }
        blk = static_cast<char *>(sp.ptr);
        blk_bytes = sp.bytes;
        sp.ptr = nullptr;
        sp.bytes = 0;
        sp.pending = false;
    } else {
        e = hipMalloc(reinterpret_cast<void **>(&blk), size_t(total));
        if (e != hipSuccess) {
            delete pl;
            (void)hipGetLastError();
            return fail(ctx, e == hipErrorOutOfMemory ? NTS_ENOMEM : NTS_EHIP, "device allocation of the plan failed");
        }
        blk_bytes = size_t(total);
    }
    pl->d_block = blk;
    pl->d_block_bytes = blk_bytes;
    pl->d_sslot = reinterpret_cast<int32_t *>(blk);
    pl->d_dslot = reinterpret_cast<int32_t *>(blk + b_slots);
    char *d_meta = blk + 2 * b_slots;
    char *h_meta = static_cast<char *>(ctx->h_pinned) + 256;
    volatile int32_t *h_err = static_cast<volatile int32_t *>(ctx->h_pinned);
    memcpy(h_meta, tok_off.data(), size_t(n_off) * 4);
    memcpy(h_meta + b_off, pg_off.data(), size_t(n_off) * 4);
    memcpy(h_meta + 2 * b_off, d->src_pages, size_t(NP) * 4);
    memcpy(h_meta + 2 * b_off + b_pages, d->dst_pages, size_t(NP) * 4);
    h_err[0] = h_err[1] = h_err[2] = 0;
    char *d_bm = d_meta + b_meta;
    int32_t *d_err = reinterpret_cast<int32_t *>(d_bm + b_bitmap);
    NtsFlattenSide fs, fd;
    fs.pages = reinterpret_cast<const int32_t *>(d_meta + 2 * b_off);
    fs.slots = pl->d_sslot;
    fs.bitmap = nullptr;
    fs.n_pool_pages = d->S_src / p;
    fd.pages = reinterpret_cast<const int32_t *>(d_meta + 2 * b_off + b_pages);
    fd.slots = pl->d_dslot;
    fd.bitmap = uniq ? reinterpret_cast<uint32_t *>(d_bm) : nullptr;
    fd.n_pool_pages = d->S_dst / p;

    hipStream_t st = ctx->aux;
    do {
        if ((e = hipMemcpyAsync(d_meta, h_meta, size_t(b_meta), hipMemcpyHostToDevice, st)) != hipSuccess) break;
        if ((e = hipMemsetAsync(d_bm, 0, size_t(b_bitmap + 256), st)) != hipSuccess) break;
        if ((e = nts_launch_flatten(reinterpret_cast<const int32_t *>(d_meta),
                                    reinterpret_cast<const int32_t *>(d_meta + b_off), d->n_req,
                                    uint32_t(T), p, fs, fd, d_err, st)) != hipSuccess) break;
        if (want_runs) {
            pl->d_run_start = reinterpret_cast<int32_t *>(reinterpret_cast<char *>(d_err) + 256);
            int32_t *d_counts = pl->d_run_start + align_up((T + 1) * 4, 256) / 4;
            if ((e = nts_launch_detect_runs(pl->d_sslot, pl->d_dslot, uint32_t(T), d_counts, pl->d_run_start,
                                            d_err + 2, st)) != hipSuccess) break;
        }
        if (want_order) {
            char *at = reinterpret_cast<char *>(d_err) + 256 + b_runs;
            int32_t *d_wprefix = reinterpret_cast<int32_t *>(at);
            int32_t *d_wblocks = reinterpret_cast<int32_t *>(at + b_wprefix);
            pl->d_sslot_by_dst = reinterpret_cast<int32_t *>(at + b_wprefix + b_wblocks);
            pl->d_dslot_by_dst = reinterpret_cast<int32_t *>(at + b_wprefix + b_wblocks + b_slots);
            if ((e = nts_launch_rank_by_dst(pl->d_sslot, pl->d_dslot, uint32_t(T), reinterpret_cast<const uint32_t *>(d_bm),
                                            uint32_t(bitmap_words), d_wprefix, d_wblocks, pl->d_sslot_by_dst,
                                            pl->d_dslot_by_dst, st)) != hipSuccess) break;
        }
        if ((e = hipMemcpyAsync(const_cast<int32_t *>(h_err), d_err, 12, hipMemcpyDeviceToHost, st)) != hipSuccess) break;
        e = hipStreamSynchronize(st);
    } while (0);
    const int err_range = h_err[0], err_dup = h_err[1];
    if (e != hipSuccess || err_range || err_dup) {
        (void)hipFree(blk);
        delete pl;
        if (e != hipSuccess) return fail_hip(ctx, e, "nts_plan_create");
        if (err_range) return fail(ctx, NTS_ERANGE, "a page id lies outside its pool");
        return fail(ctx, NTS_EDUP, "two migrated tokens share a destination slot");
    }
    pl->n_runs = want_runs ? h_err[2] : 0;
    ++ctx->n_plans;
    *out = pl;
    return NTS_OK;
}

int nts_plan_free(nts_plan *pl)
{
    if (!pl) return NTS_OK;
    nts_ctx *ctx = pl->ctx;
    int rc = NTS_OK;
    if (pl->d_block) {
        DeviceGuard guard(ctx->device);
        // Kernels of this plan may still be running and they index through d_block.  The block
        // goes to a spare slot together with an event recorded behind that work; the plan that
        // reuses it makes its own writes wait for the event.
        int slot = -1;
        for (int i = 0; i < nts_ctx::kSpares && slot < 0; ++i)
            if (!ctx->spare[i].ptr) slot = i;
        if (slot < 0) {                              // all slots taken: give the smallest block back
            slot = 0;
            for (int i = 1; i < nts_ctx::kSpares; ++i)
                if (ctx->spare[i].bytes < ctx->spare[slot].bytes) slot = i;
            if (ctx->spare[slot].bytes >= pl->d_block_bytes) slot = -1;   // this one is the smallest
        }
        hipError_t e = hipSuccess;
        if (slot >= 0 && pl->n_used_streams <= 1) {
            nts_ctx::Spare &sp = ctx->spare[slot];
            if (sp.ptr) {                            // evict: the block must be idle before hipFree
                if (sp.pending) e = hipEventSynchronize(sp.ev);
                if (e == hipSuccess) e = hipFree(sp.ptr);
                sp.ptr = nullptr;
                sp.bytes = 0;
                sp.pending = false;
            }
            if (e == hipSuccess && pl->n_used_streams > 0) {
                e = hipEventRecord(sp.ev, pl->used_streams[0]);
                sp.pending = e == hipSuccess;
            }
            if (e == hipSuccess) {
                sp.ptr = pl->d_block;
                sp.bytes = pl->d_block_bytes;
                sp.age = ++ctx->free_count;
                pl->d_block = nullptr;
            }
        }
        if (pl->d_block) {                           // not kept (or several streams): wait, then free
            (void)hipGetLastError();
            if (pl->more_streams) (void)hipDeviceSynchronize();
            else
                for (int i = 0; i < pl->n_used_streams; ++i) (void)hipStreamSynchronize(pl->used_streams[i]);
            e = hipFree(pl->d_block);
        }
        if (e != hipSuccess) rc = fail_hip(ctx, e, "nts_plan_free");
    }
    --ctx->n_plans;
    delete pl;
    return rc;
}

int nts_plan_info(const nts_plan *pl, nts_info *out)
{
    if (!pl || !out) return NTS_EINVAL;
    out->T = pl->T;
    out->F = pl->F;
    out->frag_bytes = pl->frag_bytes;
    out->X = pl->X;
    out->chunk_frags = pl->chunk_frags;
    out->chunk_bytes = pl->chunk_bytes;
    out->n_chunks = pl->n_chunks;
    out->vec_bytes = pl->vec;
    out->n_runs = int32_t(pl->n_runs);
    return NTS_OK;
}

int nts_plan_slots(const nts_plan *pl, int32_t *sslot_host, int32_t *dslot_host)
{
    if (!pl) return NTS_EINVAL;
    if (pl->T == 0) return NTS_OK;
    DeviceGuard guard(pl->ctx->device);
    if (sslot_host) NTS_HIP(pl->ctx, hipMemcpy(sslot_host, pl->d_sslot, size_t(pl->T) * 4, hipMemcpyDeviceToHost));
    if (dslot_host) NTS_HIP(pl->ctx, hipMemcpy(dslot_host, pl->d_dslot, size_t(pl->T) * 4, hipMemcpyDeviceToHost));
    return NTS_OK;
}

int nts_plan_runs(nts_plan *pl, int32_t *run_start_host)
{
    if (!pl || !run_start_host) return NTS_EINVAL;
    if (!pl->has_runs) return fail(pl->ctx, NTS_EINVAL, "the plan was made without NTS_DETECT_RUNS");
    if (pl->T == 0) {
        run_start_host[0] = 0;
        return NTS_OK;
    }
    DeviceGuard guard(pl->ctx->device);
    NTS_HIP(pl->ctx, hipMemcpy(run_start_host, pl->d_run_start, size_t(pl->n_runs + 1) * 4, hipMemcpyDeviceToHost));
    return NTS_OK;
}

static int run_range(nts_plan *pl, NtsMoveMode mode, const void *const *layer_ptrs, int64_t q0,
                     int64_t n_frag, void *linear, bool staging, void *hip_stream)
{
    if (!pl) return NTS_EINVAL;
    nts_ctx *ctx = pl->ctx;
    if (!layer_ptrs) return fail(ctx, NTS_EINVAL, "null layer pointer table");
    if (n_frag <= 0) return NTS_OK;
    if (!linear) return fail(ctx, NTS_EINVAL, "null stream buffer");
    if (reinterpret_cast<uintptr_t>(linear) % uintptr_t(pl->vec)) return fail(ctx, NTS_EINVAL, "stream buffer misaligned");
    NtsLayerTab tab;
    if (fill_tab(pl, layer_ptrs, tab) != NTS_OK) return fail(ctx, NTS_EINVAL, "null or misaligned layer pointer");
    DeviceGuard guard(ctx->device);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    note_stream(pl, st);
    // a launch covers at most chunk-limit fragments; the whole stream may need several
    const int64_t lim = nts_max_frags_per_launch(pl);
    char *lin = static_cast<char *>(linear);
    for (int64_t done = 0; done < n_frag; done += lim) {
        const int64_t n = n_frag - done < lim ? n_frag - done : lim;
        NTS_HIP(ctx, nts_launch_move(mode, pl, q0 + done, n, tab, lin + done * pl->frag_bytes, staging, false, st));
    }
    return NTS_OK;
}

int nts_run_pack(nts_plan *pl, const void *const *src_layer_ptrs, void *stream_out, void *hip_stream)
{
    if (!pl) return NTS_EINVAL;
    return run_range(pl, NTS_MOVE_PACK, src_layer_ptrs, 0, pl->F, stream_out, false, hip_stream);
}

int nts_run_unpack(nts_plan *pl, const void *stream_in, void *const *dst_layer_ptrs, void *hip_stream)
{
    if (!pl) return NTS_EINVAL;
    return run_range(pl, NTS_MOVE_UNPACK, dst_layer_ptrs, 0, pl->F, const_cast<void *>(stream_in), false, hip_stream);
}

static int chunk_range(const nts_plan *pl, int64_t k, int64_t *q0, int64_t *n)
{
    return nts_host_chunk_range(pl->F, pl->chunk_frags, pl->n_chunks, k, q0, n);
}

int nts_run_pack_chunk(nts_plan *pl, const void *const *src_layer_ptrs, int64_t k, void *chunk_out, void *hip_stream)
{
    if (!pl) return NTS_EINVAL;
    int64_t q0, n;
    if (chunk_range(pl, k, &q0, &n) != NTS_OK) return fail(pl->ctx, NTS_EINVAL, "chunk index out of range");
    return run_range(pl, NTS_MOVE_PACK, src_layer_ptrs, q0, n, chunk_out, true, hip_stream);
}

int nts_run_unpack_chunk(nts_plan *pl, const void *chunk_in, int64_t k, void *const *dst_layer_ptrs, void *hip_stream)
{
    if (!pl) return NTS_EINVAL;
    int64_t q0, n;
    if (chunk_range(pl, k, &q0, &n) != NTS_OK) return fail(pl->ctx, NTS_EINVAL, "chunk index out of range");
    return run_range(pl, NTS_MOVE_UNPACK, dst_layer_ptrs, q0, n, const_cast<void *>(chunk_in), true, hip_stream);
}

static int check_pools(nts_plan *pl, const void *const *src_layer_ptrs, void *const *dst_layer_ptrs,
                       NtsLayerTab &stab, NtsLayerTab &dtab)
{
    nts_ctx *ctx = pl->ctx;
    if (!src_layer_ptrs || !dst_layer_ptrs) return fail(ctx, NTS_EINVAL, "null layer pointer table");
    if (fill_tab(pl, src_layer_ptrs, stab) != NTS_OK ||
        fill_tab(pl, reinterpret_cast<const void *const *>(dst_layer_ptrs), dtab) != NTS_OK)
        return fail(ctx, NTS_EINVAL, "null or misaligned layer pointer");
    const int64_t src_span = pl->S_src * pl->src_stride, dst_span = pl->S_dst * pl->dst_stride;
    const int n = 2 * pl->L;
    for (int i = 0; i < n; ++i)
        for (int k = 0; k < n; ++k)
            if (overlaps(stab.p[i], src_span, dtab.p[k], dst_span))
                return fail(ctx, NTS_EALIAS, "source and destination pools overlap");
    return NTS_OK;
}

namespace {

// One pair of a pipeline run: a plan that moves something, with its two pointer tables.
struct PipeItem {
    nts_plan *pl;
    NtsLayerTab stab, dtab;
};

// The double-buffered pipeline of Sec. 3.2.2 over the chunks of `items`, taken as one
// sequence g = 0, 1, ...: stage g packs chunk g into buffer g&1 and unpacks chunk g-1 from
// the other buffer, across pair boundaries too.  The launches go to `st` in order, which
// hands each buffer from its producer to its consumer.  `stride`: distance of the buffers.
int run_pipeline(nts_ctx *ctx, PipeItem *items, size_t n_items, char *staging, int64_t stride, hipStream_t st)
{
    DeviceGuard guard(ctx->device);
    for (size_t i = 0; i < n_items; ++i) note_stream(items[i].pl, st);
    char *buf[2] = {staging, staging + stride};
    size_t pi = 0;              // pair and chunk being packed
    int64_t pk = 0;
    const PipeItem *ui = nullptr;   // pair and chunk packed by the previous stage
    int64_t uk = 0;
    for (int64_t g = 0;; ++g) {
        const PipeItem *ai = pi < n_items ? &items[pi] : nullptr;
        if (!ai && !ui) break;
        int64_t pq = 0, pn = 0, uq = 0, un = 0;
        if (ai) chunk_range(ai->pl, pk, &pq, &pn);
        if (ui) chunk_range(ui->pl, uk, &uq, &un);
        const PipeItem *any = ai ? ai : ui;
        NTS_HIP(ctx, nts_launch_stage(ai ? ai->pl : nullptr, pq, pn, buf[g & 1], ai ? ai->stab : any->stab,
                                      ui ? ui->pl : nullptr, uq, un, buf[(g - 1) & 1],
                                      ui ? ui->dtab : any->dtab, st));
        ui = ai;
        uk = pk;
        if (ai && ++pk == ai->pl->n_chunks) {
            ++pi;
            pk = 0;
        }
    }
    return NTS_OK;
}

}  // namespace

int nts_run_migrate(nts_plan *pl, const void *const *src_layer_ptrs, void *const *dst_layer_ptrs,
                    void *staging, void *hip_stream)
{
    if (!pl) return NTS_EINVAL;
    nts_ctx *ctx = pl->ctx;
    if (!src_layer_ptrs || !dst_layer_ptrs) return fail(ctx, NTS_EINVAL, "null layer pointer table");
    if (pl->F == 0) return NTS_OK;
    PipeItem item;
    item.pl = pl;
    const int rc = check_pools(pl, src_layer_ptrs, dst_layer_ptrs, item.stab, item.dtab);
    if (rc != NTS_OK) return rc;
    if (!staging) return fail(ctx, NTS_EINVAL, "null staging area");
    if (reinterpret_cast<uintptr_t>(staging) % uintptr_t(pl->vec)) return fail(ctx, NTS_EINVAL, "staging area misaligned");
    char *stg = static_cast<char *>(staging);
    const int64_t src_span = pl->S_src * pl->src_stride, dst_span = pl->S_dst * pl->dst_stride;
    for (int i = 0; i < 2 * pl->L; ++i)
        if (overlaps(item.stab.p[i], src_span, stg, 2 * pl->chunk_bytes) ||
            overlaps(item.dtab.p[i], dst_span, stg, 2 * pl->chunk_bytes))
            return fail(ctx, NTS_EALIAS, "staging area overlaps a pool");
    // chunk_bytes is a multiple of the vector width, so the second buffer stays aligned
    return run_pipeline(ctx, &item, 1, stg, pl->chunk_bytes, static_cast<hipStream_t>(hip_stream));
}

int nts_run_migrate_static(nts_plan *pl, const void *const *src_layer_ptrs, void *const *dst_layer_ptrs,
                           void *hip_stream)
{
    if (!pl) return NTS_EINVAL;
    nts_ctx *ctx = pl->ctx;
    if (!src_layer_ptrs || !dst_layer_ptrs) return fail(ctx, NTS_EINVAL, "null layer pointer table");
    if (pl->F == 0) return NTS_OK;                    // nothing to move, whatever the chunk geometry
    if (2 * pl->chunk_bytes > int64_t(NTS_STATIC_STAGING_BYTES))
        return fail(ctx, NTS_EINVAL, "the plan's two staging buffers exceed NTS_STATIC_STAGING_BYTES: "
                                     "create the plan with staging_bytes <= NTS_STATIC_STAGING_BYTES / 2");
    if (!ctx->static_staging) return fail(ctx, NTS_EHIP, "static staging area unavailable");
    return nts_run_migrate(pl, src_layer_ptrs, dst_layer_ptrs, ctx->static_staging, hip_stream);
}

int nts_batch_staging_bytes(int n, nts_plan *const *plans, int64_t *bytes)
{
    if (n < 0 || !bytes || (n > 0 && !plans)) return NTS_EINVAL;
    std::vector<int64_t> cb;
    try {
        for (int i = 0; i < n; ++i) {
            if (!plans[i]) return NTS_EINVAL;
            if (plans[i]->F > 0) cb.push_back(plans[i]->chunk_bytes);
        }
    } catch (...) {
        return NTS_ENOMEM;
    }
    *bytes = nts_host_batch_staging_bytes(cb.data(), int(cb.size()));
    return NTS_OK;
}

int nts_run_migrate_batch(int n, nts_plan *const *plans, const void *const *const *src_layer_ptrs,
                          void *const *const *dst_layer_ptrs, void *staging, void *hip_stream)
{
    if (n < 0 || (n > 0 && (!plans || !src_layer_ptrs || !dst_layer_ptrs))) return NTS_EINVAL;
    nts_ctx *ctx = nullptr;
    for (int i = 0; i < n; ++i) {
        if (!plans[i]) return ctx ? fail(ctx, NTS_EINVAL, "null plan in batch") : NTS_EINVAL;
        if (!ctx) ctx = plans[i]->ctx;
        if (plans[i]->ctx != ctx) return fail(ctx, NTS_EINVAL, "plans of different contexts in one batch");
    }
    if (!ctx) return NTS_OK;

    // the pairs that move something, with their pointer tables
    std::vector<PipeItem> items;
    std::vector<NtsByteRange> ranges;
    try {
        items.reserve(size_t(n));
        for (int i = 0; i < n; ++i) {
            nts_plan *pl = plans[i];
            if (pl->F == 0) continue;
            items.emplace_back();
            PipeItem &it = items.back();
            it.pl = pl;
            const int rc = check_pools(pl, src_layer_ptrs[i], dst_layer_ptrs[i], it.stab, it.dtab);
            if (rc != NTS_OK) return rc;
            const int64_t src_span = pl->S_src * pl->src_stride, dst_span = pl->S_dst * pl->dst_stride;
            for (int k = 0; k < 2 * pl->L; ++k) {
                const uintptr_t sl = reinterpret_cast<uintptr_t>(it.stab.p[k]), dl = reinterpret_cast<uintptr_t>(it.dtab.p[k]);
                ranges.push_back({sl, sl + uintptr_t(src_span), 0});
                ranges.push_back({dl, dl + uintptr_t(dst_span), 1});
            }
        }
    } catch (...) {
        return fail(ctx, NTS_ENOMEM, "host allocation failed");
    }
    if (items.empty()) return NTS_OK;
    if (!staging) return fail(ctx, NTS_EINVAL, "null staging area");
    if (reinterpret_cast<uintptr_t>(staging) % 16u) return fail(ctx, NTS_EINVAL, "staging area misaligned");
    int64_t staging_bytes = 0;
    (void)nts_batch_staging_bytes(n, plans, &staging_bytes);
    char *stg = static_cast<char *>(staging);

    // No destination range may meet a source range of ANY plan, nor the staging area.
    const char *why = "";
    const int arc = nts_host_alias_sweep(ranges, reinterpret_cast<uintptr_t>(stg), staging_bytes, &why);
    if (arc != NTS_OK) return fail(ctx, arc, why);
    // the second buffer starts 16-byte aligned whatever the plans' vector widths
    return run_pipeline(ctx, items.data(), items.size(), stg, staging_bytes / 2, static_cast<hipStream_t>(hip_stream));
}

int nts_run_migrate_direct(nts_plan *pl, const void *const *src_layer_ptrs, void *const *dst_layer_ptrs,
                           void *hip_stream)
{
    if (!pl) return NTS_EINVAL;
    nts_ctx *ctx = pl->ctx;
    if (!src_layer_ptrs || !dst_layer_ptrs) return fail(ctx, NTS_EINVAL, "null layer pointer table");
    if (pl->F == 0) return NTS_OK;
    NtsLayerTab stab, dtab;
    const int rc = check_pools(pl, src_layer_ptrs, dst_layer_ptrs, stab, dtab);
    if (rc != NTS_OK) return rc;
    DeviceGuard guard(ctx->device);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    note_stream(pl, st);
    const int64_t lim = nts_max_frags_per_launch(pl);
    for (int64_t done = 0; done < pl->F; done += lim) {
        const int64_t n = pl->F - done < lim ? pl->F - done : lim;
        NTS_HIP(ctx, nts_launch_direct(pl, done, n, stab, dtab, st));
    }
    return NTS_OK;
}

int nts_run_memcpy_baseline(nts_plan *pl, const void *const *src_layer_ptrs, void *const *dst_layer_ptrs,
                            int merge_runs, void *hip_stream, int64_t *n_copies)
{
    if (!pl) return NTS_EINVAL;
    nts_ctx *ctx = pl->ctx;
    if (n_copies) *n_copies = 0;
    if (!src_layer_ptrs || !dst_layer_ptrs) return fail(ctx, NTS_EINVAL, "null layer pointer table");
    if (pl->F == 0) return NTS_OK;
    NtsLayerTab stab, dtab;
    const int rc = check_pools(pl, src_layer_ptrs, dst_layer_ptrs, stab, dtab);
    if (rc != NTS_OK) return rc;
    DeviceGuard guard(ctx->device);
    if (pl->h_sslot.empty()) {
        try {
            pl->h_sslot.resize(size_t(pl->T));
            pl->h_dslot.resize(size_t(pl->T));
        } catch (...) {
            return fail(ctx, NTS_ENOMEM, "host allocation failed");
        }
        NTS_HIP(ctx, hipMemcpy(pl->h_sslot.data(), pl->d_sslot, size_t(pl->T) * 4, hipMemcpyDeviceToHost));
        NTS_HIP(ctx, hipMemcpy(pl->h_dslot.data(), pl->d_dslot, size_t(pl->T) * 4, hipMemcpyDeviceToHost));
    }
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const int64_t so = int64_t(pl->src_head_off) * pl->D * pl->e, dof = int64_t(pl->dst_head_off) * pl->D * pl->e;
    // a run of tokens in neighbouring slots on both sides is one region when a fragment is a whole row
    const bool can_merge = merge_runs && pl->frag_bytes == pl->src_stride && pl->frag_bytes == pl->dst_stride;
    // the plan's own run list when it has one, else the same rule applied to the host copies
    if (can_merge && pl->has_runs && pl->h_run_start.empty()) {
        try {
            pl->h_run_start.resize(size_t(pl->n_runs) + 1);
        } catch (...) {
            return fail(ctx, NTS_ENOMEM, "host allocation failed");
        }
        NTS_HIP(ctx, hipMemcpy(pl->h_run_start.data(), pl->d_run_start, size_t(pl->n_runs + 1) * 4, hipMemcpyDeviceToHost));
    }
    int64_t copies = 0;
    for (int lc = 0; lc < 2 * pl->L; ++lc) {
        int64_t j = 0, r = 0;
        while (j < pl->T) {
            int64_t len = 1;
            if (can_merge && pl->has_runs) {
                len = int64_t(pl->h_run_start[size_t(r) + 1]) - j;
                ++r;
            } else if (can_merge) {
                while (j + len < pl->T && pl->h_sslot[j + len] == pl->h_sslot[j] + len &&
                       pl->h_dslot[j + len] == pl->h_dslot[j] + len)
                    ++len;
            }
            const char *s = stab.p[lc] + int64_t(pl->h_sslot[j]) * pl->src_stride + so;
            char *d = dtab.p[lc] + int64_t(pl->h_dslot[j]) * pl->dst_stride + dof;
            NTS_HIP(ctx, hipMemcpyAsync(d, s, size_t(len * pl->frag_bytes), hipMemcpyDeviceToDevice, st));
            ++copies;
            j += len;
        }
    }
    if (n_copies) *n_copies = copies;
    return NTS_OK;
}

namespace {
struct LinearGeom {
    int M, Nn, K;
    int64_t ldx, lda, ldy, a_off;   // a_off: element offset of the shard inside W
    int tiled;                       // tile width of the tiled kernel (256 or 128), 0: the streaming / decode kernels
    int tiled_rows;                  // its tile height (256 or 128)
    NtsStreamCfg cfg;                // streaming kernel: tile, prefetch depth, K splits
};

int linear_geom(const nts_linear_desc *d, LinearGeom *g)
{
    if (!d || d->M < 1 || d->n_out < 1 || d->n_in < 1 || d->tp < 1 || d->rank < 0 || d->rank >= d->tp) return NTS_EINVAL;
    if (d->split != NTS_SPLIT_OUT && d->split != NTS_SPLIT_IN) return NTS_EINVAL;
    if (d->dtype != NTS_BF16 && d->dtype != NTS_F16) return NTS_EINVAL;
    const int64_t ldw = d->ldw ? d->ldw : d->n_in;
    if (ldw < d->n_in) return NTS_EINVAL;
    if (d->split == NTS_SPLIT_OUT) {
        if (d->n_out % d->tp) return NTS_EINVAL;
        g->Nn = d->n_out / d->tp;
        g->K = d->n_in;
        g->a_off = int64_t(d->rank) * g->Nn * ldw;
    } else {
        if (d->n_in % d->tp) return NTS_EINVAL;
        g->Nn = d->n_out;
        g->K = d->n_in / d->tp;
        g->a_off = int64_t(d->rank) * g->K;
    }
    g->M = d->M;
    g->lda = ldw;
    g->ldx = d->ldx ? d->ldx : g->K;
    g->ldy = d->ldy ? d->ldy : g->Nn;
    if (g->K % 64 || g->ldx < g->K || g->ldy < g->Nn) return NTS_EINVAL;
    if (g->ldx % 8 || g->lda % 8 || g->ldy % 8 || g->a_off % 8) return NTS_EINVAL;
    // the tiled kernel addresses the 256 rows of a tile with 32-bit byte offsets from the tile's first row
    const int64_t lim = int64_t(1) << 23;
    if (g->ldx >= lim || g->lda >= lim || g->ldy >= lim) return NTS_EINVAL;
    g->tiled = nts_linear_use_tiled(g->M, g->Nn, g->K, &g->tiled_rows);
    g->cfg = nts_linear_stream_config(g->M, g->Nn, g->K);
    if (g->tiled) g->cfg.splits = 1;
    return NTS_OK;
}
}  // namespace

int nts_shard_linear_workspace(const nts_linear_desc *d, size_t *bytes)
{
    LinearGeom g;
    if (!bytes || linear_geom(d, &g) != NTS_OK) return NTS_EINVAL;
    *bytes = g.cfg.splits > 1 ? size_t(g.cfg.splits) * g.M * g.Nn * sizeof(float) : 0;
    return NTS_OK;
}

static void describe_launch(const LinearGeom &g, nts_linear_launch *out)
{
    *out = nts_linear_launch{};
    out->tiled = g.tiled ? 1 : 0;
    const bool decode = !g.tiled && g.cfg.ks > 0;
    out->tile_rows = g.tiled ? g.tiled_rows : decode ? 16 : 32 * g.cfg.mt;
    out->tile_cols = g.tiled ? g.tiled : decode ? 16 * g.cfg.rt : 32 * g.cfg.cw * g.cfg.rt;
    out->k_splits = g.cfg.splits;
    out->slabs_ahead = g.tiled ? 2 : g.cfg.nsets - 1;
    out->k_waves = decode ? g.cfg.ks : 1;
}

static size_t linear_workspace_need(const LinearGeom &g)
{
    return g.cfg.splits > 1 ? size_t(g.cfg.splits) * g.M * g.Nn * sizeof(float) : 0;
}

// Replace the default configuration of `g` by the one nts_shard_linear_tune remembered for this
// shape, when there is one and the workspace at hand is large enough for it.
static void apply_tuned(const nts_ctx *ctx, int dtype, size_t workspace_bytes, bool have_workspace, LinearGeom *g)
{
    const auto it = ctx->tuned_linear.find(std::make_tuple(g->M, g->Nn, g->K, dtype));
    if (it == ctx->tuned_linear.end()) return;
    const nts_ctx::TunedLinear &t = it->second;
    LinearGeom h = *g;
    h.tiled = t.tiled;
    h.tiled_rows = t.tiled_rows;
    h.cfg.mt = t.mt; h.cfg.cw = t.cw; h.cfg.rt = t.rt; h.cfg.nsets = t.nsets; h.cfg.splits = t.splits; h.cfg.ks = t.ks;
    const size_t need = linear_workspace_need(h);
    if (need && (!have_workspace || workspace_bytes < need)) return;
    *g = h;
}

static hipError_t launch_linear(const LinearGeom &g, int dtype, const void *X, const void *W_full, void *Y,
                                void *workspace, hipStream_t st)
{
    const uint16_t *A = static_cast<const uint16_t *>(W_full) + g.a_off;
    if (!g.tiled)
        return nts_launch_linear_stream(static_cast<const uint16_t *>(X), g.ldx, A, g.lda, static_cast<uint16_t *>(Y),
                                        g.ldy, static_cast<float *>(workspace), g.cfg, g.M, g.Nn, g.K,
                                        dtype == NTS_F16, st);
    return nts_launch_linear_tiled(static_cast<const uint16_t *>(X), g.ldx, A, g.lda, static_cast<uint16_t *>(Y),
                                   g.ldy, g.M, g.Nn, g.K, g.tiled_rows, g.tiled, dtype == NTS_F16, st);
}

static int check_linear_operands(nts_ctx *ctx, const void *X, const void *W_full, const void *Y)
{
    if (!X || !W_full || !Y) return fail(ctx, NTS_EINVAL, "null operand");
    if ((reinterpret_cast<uintptr_t>(X) | reinterpret_cast<uintptr_t>(W_full) | reinterpret_cast<uintptr_t>(Y)) % 16)
        return fail(ctx, NTS_EINVAL, "operands must be 16-byte aligned");
    return NTS_OK;
}

// Inverse of describe_launch: the configuration a public launch description names, for the problem in
// `g`.  False when the library has no such kernel instance or the split does not fit the problem.
static bool launch_to_geom(const nts_linear_launch *how, LinearGeom *g)
{
    if (!how) return false;
    const int n_slabs = g->K / 64;
    NtsStreamCfg c;
    c.splits = how->k_splits;
    if (c.splits < 1 || c.splits > 32) return false;
    if (how->tiled) {
        const bool known = (how->tile_rows == 256 && (how->tile_cols == 256 || how->tile_cols == 192 || how->tile_cols == 128)) ||
                           (how->tile_rows == 128 && (how->tile_cols == 192 || how->tile_cols == 128));
        if (!known || c.splits != 1) return false;
        if (g->M < how->tile_rows) return false;         // as in the default choice: a whole batch tile at least
        g->tiled = how->tile_cols;
        g->tiled_rows = how->tile_rows;
        g->cfg.splits = 1;
        return true;
    }
    const int sps = (n_slabs + c.splits - 1) / c.splits;
    if ((n_slabs + sps - 1) / sps != c.splits) return false;                 // would leave an empty split
    c.nsets = how->slabs_ahead + 1;
    if (how->tile_rows == 16) {                                              // decode kernel
        if (g->M > 16 || how->tile_cols % 16) return false;
        c.rt = how->tile_cols / 16;
        c.ks = how->k_waves;
        const bool inst = (c.ks == 2 && c.rt == 1) || (c.ks == 4 && c.rt == 1) || (c.ks == 4 && c.rt == 2);
        if (!inst || c.nsets != (c.rt == 1 ? 8 : 6) || sps / c.ks < 1) return false;
    } else {                                                                 // streaming kernel
        if (how->tile_rows % 32 || how->tile_cols % 32 || how->k_waves != 1) return false;
        c.mt = how->tile_rows / 32;
        c.cw = how->tile_cols / 32;
        c.rt = 1;
        c.ks = 0;
        static const int inst[][3] = {{1, 4, 4}, {2, 4, 4}, {3, 4, 4}, {4, 4, 4}, {6, 4, 3}, {8, 4, 3},
                                      {1, 1, 8}, {2, 1, 4}, {4, 1, 4}, {2, 2, 4}, {4, 2, 4}};
        bool ok = false;
        for (const auto &v : inst) ok = ok || (v[0] == c.mt && v[1] == c.cw && v[2] == c.nsets);
        if (!ok) return false;
    }
    g->tiled = 0;
    g->cfg = c;
    return true;
}

int nts_shard_linear_candidates(const nts_linear_desc *d, nts_linear_launch *out, int max_out, int *n_out)
{
    LinearGeom g;
    if (!out || !n_out || max_out < 1 || linear_geom(d, &g) != NTS_OK) return NTS_EINVAL;
    NtsLinearCand cand[16];
    const int n = nts_linear_candidates(g.M, g.Nn, g.K, 1.4, cand, max_out < 16 ? max_out : 16);
    for (int i = 0; i < n; ++i) {
        LinearGeom h = g;
        h.tiled = cand[i].tiled;
        h.tiled_rows = cand[i].tiled_rows;
        h.cfg = cand[i].cfg;
        describe_launch(h, &out[i]);
    }
    *n_out = n;
    return NTS_OK;
}

int nts_shard_linear_with(nts_ctx *ctx, const nts_linear_desc *d, const nts_linear_launch *how, const void *X,
                          const void *W_full, void *Y, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (!ctx) return NTS_EINVAL;
    LinearGeom g;
    if (linear_geom(d, &g) != NTS_OK) return fail(ctx, NTS_EINVAL, "bad linear-layer descriptor");
    if (!launch_to_geom(how, &g)) return fail(ctx, NTS_EINVAL, "no such kernel configuration for this problem");
    const int rc = check_linear_operands(ctx, X, W_full, Y);
    if (rc != NTS_OK) return rc;
    const size_t need = linear_workspace_need(g);
    if (need && (!workspace || reinterpret_cast<uintptr_t>(workspace) % 16 || workspace_bytes < need))
        return fail(ctx, NTS_EINVAL, "workspace missing, misaligned or too small");
    DeviceGuard guard(ctx->device);
    NTS_HIP(ctx, launch_linear(g, d->dtype, X, W_full, Y, workspace, static_cast<hipStream_t>(hip_stream)));
    return NTS_OK;
}

int nts_shard_linear_remember(nts_ctx *ctx, const nts_linear_desc *d, const nts_linear_launch *how)
{
    if (!ctx) return NTS_EINVAL;
    LinearGeom g;
    if (linear_geom(d, &g) != NTS_OK) return fail(ctx, NTS_EINVAL, "bad linear-layer descriptor");
    const auto key = std::make_tuple(g.M, g.Nn, g.K, int(d->dtype));
    if (!how) {                                       // forget: back to the default
        ctx->tuned_linear.erase(key);
        return NTS_OK;
    }
    if (!launch_to_geom(how, &g)) return fail(ctx, NTS_EINVAL, "no such kernel configuration for this problem");
    nts_ctx::TunedLinear t;
    t.tiled = g.tiled;
    t.tiled_rows = g.tiled_rows;
    t.mt = g.cfg.mt; t.cw = g.cfg.cw; t.rt = g.cfg.rt; t.nsets = g.cfg.nsets; t.splits = g.cfg.splits; t.ks = g.cfg.ks;
    try {
        ctx->tuned_linear[key] = t;
    } catch (...) {
        return fail(ctx, NTS_ENOMEM, "host allocation failed");
    }
    return NTS_OK;
}

int nts_shard_linear_launch(const nts_linear_desc *d, nts_linear_launch *out)
{
    LinearGeom g;
    if (!out || linear_geom(d, &g) != NTS_OK) return NTS_EINVAL;
    describe_launch(g, out);
    return NTS_OK;
}

int nts_shard_linear_view(const nts_linear_desc *d, int64_t *elem_offset, int64_t *rows, int64_t *cols,
                          int64_t *row_stride)
{
    LinearGeom g;
    if (!elem_offset || !rows || !cols || !row_stride || linear_geom(d, &g) != NTS_OK) return NTS_EINVAL;
    *elem_offset = g.a_off;
    *rows = g.Nn;
    *cols = g.K;
    *row_stride = g.lda;
    return NTS_OK;
}

int nts_shard_linear_tuned(const nts_ctx *ctx, const nts_linear_desc *d, nts_linear_launch *out)
{
    LinearGeom g;
    if (!ctx || !out || linear_geom(d, &g) != NTS_OK) return NTS_EINVAL;
    if (ctx->tuned_linear.find(std::make_tuple(g.M, g.Nn, g.K, int(d->dtype))) == ctx->tuned_linear.end()) return NTS_ERANGE;
    apply_tuned(ctx, d->dtype, SIZE_MAX, true, &g);
    describe_launch(g, out);
    return NTS_OK;
}

int nts_shard_linear(nts_ctx *ctx, const nts_linear_desc *d, const void *X, const void *W_full, void *Y,
                     void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (!ctx) return NTS_EINVAL;
    LinearGeom g;
    if (linear_geom(d, &g) != NTS_OK) return fail(ctx, NTS_EINVAL, "bad linear-layer descriptor");
    const int rc = check_linear_operands(ctx, X, W_full, Y);
    if (rc != NTS_OK) return rc;
    const bool ws_ok = workspace && reinterpret_cast<uintptr_t>(workspace) % 16 == 0;
    apply_tuned(ctx, d->dtype, workspace_bytes, ws_ok, &g);
    const size_t need = linear_workspace_need(g);
    if (need && (!ws_ok || workspace_bytes < need))
        return fail(ctx, NTS_EINVAL, "workspace missing, misaligned or too small");
    DeviceGuard guard(ctx->device);
    NTS_HIP(ctx, launch_linear(g, d->dtype, X, W_full, Y, workspace, static_cast<hipStream_t>(hip_stream)));
    return NTS_OK;
}

int nts_shard_linear_tune(nts_ctx *ctx, const nts_linear_desc *d, const void *X, const void *const *W_list, int n_weights,
                          void *Y, void *workspace, size_t workspace_bytes, void *hip_stream, nts_linear_launch *picked)
{
    if (!ctx) return NTS_EINVAL;
    LinearGeom g;
    if (linear_geom(d, &g) != NTS_OK) return fail(ctx, NTS_EINVAL, "bad linear-layer descriptor");
    if (!W_list || n_weights < 1 || n_weights > 4096) return fail(ctx, NTS_EINVAL, "need 1..4096 weight matrices");
    for (int i = 0; i < n_weights; ++i) {
        const int rc = check_linear_operands(ctx, X, W_list[i], Y);
        if (rc != NTS_OK) return rc;
    }
    const bool ws_ok = workspace && reinterpret_cast<uintptr_t>(workspace) % 16 == 0;
    if (linear_workspace_need(g) && (!ws_ok || workspace_bytes < linear_workspace_need(g)))
        return fail(ctx, NTS_EINVAL, "workspace missing, misaligned or too small");
    constexpr int kMaxCand = 8, kReps = 5;
    NtsLinearCand cand[kMaxCand];
    const int n = nts_linear_candidates(g.M, g.Nn, g.K, 1.4, cand, kMaxCand);
    DeviceGuard guard(ctx->device);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    // In service a layer's weights come from HBM every time (a model is far larger than the caches).  A
    // timed pass runs the layer once on each of the given matrices, back to back; when those together are
    // smaller than twice the memory-side cache, a sweep over a buffer of that size comes before each pass.
    constexpr size_t kFlushBytes = size_t(512) << 20;
    const bool need_flush = double(n_weights) * g.Nn * g.K * 2. < double(kFlushBytes);
    void *flush = nullptr;
    if (need_flush && hipMalloc(&flush, kFlushBytes) != hipSuccess) {
        (void)hipGetLastError();
        return fail(ctx, NTS_ENOMEM, "no room for the 512 MiB cache-flush buffer of the tuning run");
    }
    hipEvent_t e0 = nullptr, e1 = nullptr;
    hipError_t e = hipEventCreate(&e0);
    if (e == hipSuccess) e = hipEventCreate(&e1);
    int best = -1;
    float best_ms = 0.f, default_ms = 0.f;
    for (int i = 0; i < n && e == hipSuccess; ++i) {
        LinearGeom h = g;
        h.tiled = cand[i].tiled;
        h.tiled_rows = cand[i].tiled_rows;
        h.cfg = cand[i].cfg;
        const size_t need = linear_workspace_need(h);
        if (need && (!ws_ok || workspace_bytes < need)) continue;       // does not fit the caller's workspace
        // one untimed launch, then the shortest of kReps timed passes
        if ((e = launch_linear(h, d->dtype, X, W_list[0], Y, workspace, st)) != hipSuccess) break;
        float ms_min = 0.f;
        for (int r = 0; r < kReps && e == hipSuccess; ++r) {
            if (flush && (e = hipMemsetAsync(flush, r, kFlushBytes, st)) != hipSuccess) break;
            if ((e = hipEventRecord(e0, st)) != hipSuccess) break;
            for (int k = 0; k < n_weights && e == hipSuccess; ++k)
                e = launch_linear(h, d->dtype, X, W_list[k], Y, workspace, st);
            if (e != hipSuccess) break;
            if ((e = hipEventRecord(e1, st)) != hipSuccess) break;
            if ((e = hipEventSynchronize(e1)) != hipSuccess) break;
            float ms = 0.f;
            if ((e = hipEventElapsedTime(&ms, e0, e1)) != hipSuccess) break;
            if (r == 0 || ms < ms_min) ms_min = ms;
        }
        if (e != hipSuccess) break;
        if (i == 0) default_ms = ms_min;                 // candidate 0 is the default configuration
        // another configuration has to beat the default by 3 % (timing noise), and the best so far at all
        const bool ok = i == 0 || default_ms == 0.f || ms_min < 0.97f * default_ms;
        if (ok && (best < 0 || ms_min < best_ms)) {
            best = i;
            best_ms = ms_min;
        }
    }
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    (void)hipStreamSynchronize(st);
    if (flush) (void)hipFree(flush);
    if (e != hipSuccess) return fail_hip(ctx, e, "nts_shard_linear_tune");
    if (best < 0) return fail(ctx, NTS_EINVAL, "no configuration fits the workspace");
    // leave Y holding the result of the chosen configuration on the first matrix
    {
        LinearGeom h = g;
        h.tiled = cand[best].tiled;
        h.tiled_rows = cand[best].tiled_rows;
        h.cfg = cand[best].cfg;
        NTS_HIP(ctx, launch_linear(h, d->dtype, X, W_list[0], Y, workspace, st));
        if (picked) describe_launch(h, picked);
    }
    nts_ctx::TunedLinear t;
    t.tiled = cand[best].tiled;
    t.tiled_rows = cand[best].tiled_rows;
    t.mt = cand[best].cfg.mt; t.cw = cand[best].cfg.cw; t.rt = cand[best].cfg.rt; t.nsets = cand[best].cfg.nsets;
    t.splits = cand[best].cfg.splits; t.ks = cand[best].cfg.ks;
    try {
        ctx->tuned_linear[std::make_tuple(g.M, g.Nn, g.K, int(d->dtype))] = t;
    } catch (...) {
        return fail(ctx, NTS_ENOMEM, "host allocation failed");
    }
    return NTS_OK;
}

}  // extern "C"
