// Pack / unpack kernels of the KV migration (paper Sec. 3.2.2: the migration
// kernel copies the scattered per-page KV regions of the moved head slice into
// a contiguous buffer; the receiver does the reverse into its own pages).
//
// Both are pure byte movers bound by HBM bandwidth.  Work decomposition: the
// stream range of a launch is cut into vectors of `vec` bytes (16 when
// alignment allows) and every lane moves exactly one vector, so a 64-wide
// wavefront covers 1 KiB of the stream with one load and one store, whatever
// the fragment size: a 2 KiB fragment is two wavefronts, four 256 B fragments
// share one.  Vector index -> (fragment, offset) and fragment -> (slab, token)
// are exact divisions by launch constants, done with a precomputed 64-bit
// reciprocal (Lemire's method) or a shift.  Measured on MI355X this
// one-vector-per-lane shape (1 KiB per single-wavefront workgroup, millions of
// workgroups) sustains more HBM bandwidth than variants that keep several
// loads in flight per lane or that run a persistent grid.
//
// nts_stage_kernel is the double buffer of Sec. 3.2.2 as one launch: runs of
// its workgroups alternate between packing chunk k into one staging buffer
// and unpacking chunk k-1 from the other, so the two copies overlap and
// consecutive launches on one stream hand the buffers over.
//
// Pool accesses are non-temporal everywhere: every pool byte is touched once.
// The whole-stream kernels treat the stream the same way.  The stage kernel
// writes and reads the staging buffers with ordinary stores and loads instead:
// a chunk is read back one launch after it was written, and two buffers that
// fit the memory-side cache (256 MiB) are then served from it, where
// non-temporal accesses go round it.  Measured on the 88 GiB migration with
// 2 x 64 MiB staging: 57.7 ms against 67.2 ms (one box, same run).  The staging
// stores are also written through at agent scope, which leaves the end of a
// launch no dirty L2 lines to flush: another 1 % (57.0 -> 56.5 ms).  The same
// holds for the non-temporal stores (pools, whole streams): with the
// write-through bit as well, 56.5 -> 55.8 ms and a plain copy 6.68 -> 6.75 TB/s.
#include "nts_host.h"
#include "nts_internal.h"

namespace {

constexpr int kThreads = 64;   // one wavefront per workgroup measured best (finer retirement)

template <int BYTES> struct VecOf;
template <> struct VecOf<16> { typedef uint32_t type __attribute__((ext_vector_type(4))); };
template <> struct VecOf<8> { typedef uint32_t type __attribute__((ext_vector_type(2))); };
template <> struct VecOf<4> { typedef uint32_t type; };

// Ordinary (cache-allocating) store that is written through at agent scope: the line goes to the
// memory side at once instead of staying dirty in this XCD's L2 until the end-of-kernel release
// flushes it.  Used for the staging buffers, which the next launch reads from any XCD.
// The compiler does not know that the statement is a store: the wait states a wide store needs
// before its data registers may be overwritten are spelled out (s_nop) instead of left to it.
__device__ __forceinline__ void store_through(const VecOf<16>::type &x, void *p)
{
    asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 1" ::"v"(p), "v"(x) : "memory");
}
__device__ __forceinline__ void store_through(const VecOf<8>::type &x, void *p)
{
    asm volatile("global_store_dwordx2 %0, %1, off sc1\n\ts_nop 1" ::"v"(p), "v"(x) : "memory");
}
__device__ __forceinline__ void store_through(const VecOf<4>::type &x, void *p)
{
    asm volatile("global_store_dword %0, %1, off sc1\n\ts_nop 1" ::"v"(p), "v"(x) : "memory");
}

// Non-temporal store (the line is not kept in any cache: every pool byte is written once) that
// is written through at agent scope as well, for the same reason as above.
__device__ __forceinline__ void store_stream(const VecOf<16>::type &x, void *p)
{
    asm volatile("global_store_dwordx4 %0, %1, off sc1 nt\n\ts_nop 1" ::"v"(p), "v"(x) : "memory");
}
__device__ __forceinline__ void store_stream(const VecOf<8>::type &x, void *p)
{
    asm volatile("global_store_dwordx2 %0, %1, off sc1 nt\n\ts_nop 1" ::"v"(p), "v"(x) : "memory");
}
__device__ __forceinline__ void store_stream(const VecOf<4>::type &x, void *p)
{
    asm volatile("global_store_dword %0, %1, off sc1 nt\n\ts_nop 1" ::"v"(p), "v"(x) : "memory");
}

// n / d for n < 2^32, given m = floor((2^64 - 1) / d) + 1 (exact for every 32-bit n)
__device__ __forceinline__ uint32_t fast_div(uint32_t n, uint64_t m)
{
    return uint32_t(__umul64hi(m, uint64_t(n)));
}

// A full wavefront that covers NF = 2 or 4 whole fragments (V = 64 / NF vectors each), first
// vector gv0: if the fragments lie in one (layer, K|V) slab, the paged address of this lane's
// vector from NF scalar slot loads and one or two selects; false if they straddle two slabs.
template <int BYTES, int NF>
__device__ __forceinline__ bool small_fragments(const NtsMoveJob &job, const NtsLayerTab &tab, uint32_t gv0,
                                                uint32_t lane, char **paged)
{
    constexpr uint32_t V = kThreads / NF, kShift = NF == 2 ? 5 : 4;
    const uint32_t t0 = job.j0 + (gv0 >> kShift);
    const uint32_t ls = job.T_magic ? fast_div(t0, job.T_magic) : t0;
    const uint32_t j = t0 - ls * job.T;
    if (j + NF > job.T) return false;
    int64_t slot;
    if (NF == 2) {
        const int32_t s0 = job.slots[j], s1 = job.slots[j + 1];
        slot = lane < 32u ? s0 : s1;
    } else {
        const int32_t s0 = job.slots[j], s1 = job.slots[j + 1], s2 = job.slots[j + 2], s3 = job.slots[j + 3];
        const int32_t lo = (lane & 16u) ? s1 : s0, hi = (lane & 16u) ? s3 : s2;
        slot = (lane & 32u) ? hi : lo;
    }
    *paged = tab.p[job.lc0 + ls] + slot * job.stride + job.head_off + uint64_t(lane & (V - 1u)) * BYTES;
    return true;
}

// wg: index of the (single-wavefront) workgroup inside the job; lane: threadIdx.x
// LIN_NT: access the stream side with non-temporal instructions too (the paged side always is)
template <int BYTES, bool PACK, bool LIN_NT>
__device__ __forceinline__ void move_vector(const NtsMoveJob &job, const NtsLayerTab &tab, uint32_t wg, uint32_t lane)
{
    typedef typename VecOf<BYTES>::type vec_t;
    const uint32_t gv0 = wg * kThreads;               // first vector of this wavefront: wave-uniform
    char *paged;
    uint32_t gv;
    if (job.wave_in_frag) {
        // V is a multiple of 64: the wavefront lies inside one fragment, so the fragment
        // arithmetic, the slot load and the layer pointer load all run on the scalar unit
        if (gv0 >= job.n_vec) return;
        uint32_t fl, v0;
        if (job.v_shift >= 0) {
            fl = gv0 >> job.v_shift;
            v0 = gv0 & (job.V - 1u);
        } else {
            fl = fast_div(gv0, job.V_magic);
            v0 = gv0 - fl * job.V;
        }
        const uint32_t t = job.j0 + fl;
        const uint32_t ls = job.T_magic ? fast_div(t, job.T_magic) : t;
        const uint32_t j = t - ls * job.T;
        const int64_t slot = job.slots[j];
        gv = gv0 + lane;
        paged = tab.p[job.lc0 + ls] + slot * job.stride + job.head_off + uint64_t(v0 + lane) * BYTES;
    } else {
        gv = gv0 + lane;
        if (gv >= job.n_vec) return;
        bool done = false;
        // V = 32 or 16: a full wavefront covers two or four whole fragments.  When they lie in one
        // (layer, K|V) slab the scalar unit fetches their slots and the one layer pointer, and
        // each lane takes the slot of its own fragment.  Through the pipeline: 512 B fragments
        // 6.09 -> 6.6 TB/s, 256 B fragments 5.92 -> 6.4 TB/s.  (Two blocks with constant shifts:
        // one block with the fragment count as a variable measured 1 % slower.)
        if (job.frags_in_wave == 2 && gv0 + kThreads <= job.n_vec)
            done = small_fragments<BYTES, 2>(job, tab, gv0, lane, &paged);
        if (job.frags_in_wave == 4 && gv0 + kThreads <= job.n_vec)
            done = small_fragments<BYTES, 4>(job, tab, gv0, lane, &paged);
        if (!done) {
            uint32_t fl, v;                           // fragment (launch-local) and vector inside it
            if (job.v_shift >= 0) {
                fl = gv >> job.v_shift;
                v = gv & (job.V - 1u);
            } else {
                fl = fast_div(gv, job.V_magic);
                v = gv - fl * job.V;
            }
            const uint32_t t = job.j0 + fl;
            // slabs crossed since the launch's first one (T == 1 has no 64-bit reciprocal)
            const uint32_t ls = job.T_magic ? fast_div(t, job.T_magic) : t;
            const uint32_t j = t - ls * job.T;
            const int64_t slot = job.slots[j];
            paged = tab.p[job.lc0 + ls] + slot * job.stride + job.head_off + uint64_t(v) * BYTES;
        }
    }
    char *lin = job.linear + uint64_t(gv) * BYTES;
    if (PACK) {
        const vec_t x = __builtin_nontemporal_load(reinterpret_cast<const vec_t *>(paged));
        if (LIN_NT) store_stream(x, lin);
        else store_through(x, lin);
    } else {
        const vec_t x = LIN_NT ? __builtin_nontemporal_load(reinterpret_cast<const vec_t *>(lin))
                               : *reinterpret_cast<const vec_t *>(lin);
        store_stream(x, paged);
    }
}

// Which piece of its job a workgroup takes when the stream side is a staging buffer.
// Consecutive workgroup ids go to the 8 XCDs in turn; taken as they come, every XCD would touch
// every eighth KiB of the staging buffers and of the stream.  Inside aligned groups of
// 8 << kXcdSpanLog2 pieces the low bits are rotated so that the workgroups one XCD receives
// cover 2^kXcdSpanLog2 consecutive pieces (1 MiB): a bijection of each group, the ragged end of
// a job keeps the identity.  Measured on the stage kernel (ms per
// migration, 5 GiB / 88 GiB): none 3.19 / 55.5, 16 KiB per XCD 3.16 / 54.8, 128 KiB 3.15 / 54.6,
// 1 MiB 3.15 / 54.3, 8 MiB 3.18 / 55.0 (runs of 256; with runs of 64: 3.09-3.13 / 53.7-54.0);
// spans of 2-8 KiB lose 3 %.  The chunk calls gain 2 % (6.26 -> 6.40 TB/s through two 64 MiB
// buffers); the whole-stream and pool-to-pool kernels gained nothing and keep the plain order.
constexpr uint32_t kXcdSpanLog2 = 10;

__device__ __forceinline__ uint32_t xcd_contiguous(uint32_t idx, uint32_t n_vec)
{
    constexpr uint32_t G = 8u << kXcdSpanLog2;
    const uint32_t n_wg = (n_vec + kThreads - 1) / kThreads;
    if (idx >= (n_wg & ~(G - 1u))) return idx;
    const uint32_t low = idx & (G - 1u);
    return (idx & ~(G - 1u)) | ((low & 7u) << kXcdSpanLog2) | (low >> 3);
}

// LIN_NT = false: the stream side is a staging buffer that is read back (or was written) a
// moment ago, so it is accessed like the stage kernel's buffers, through the memory-side cache
template <int BYTES, bool PACK, bool LIN_NT>
__global__ __launch_bounds__(kThreads) void nts_move_kernel(NtsMoveJob job, NtsLayerTab tab)
{
    move_vector<BYTES, PACK, LIN_NT>(job, tab, LIN_NT ? blockIdx.x : xcd_contiguous(blockIdx.x, job.n_vec), threadIdx.x);
}

// Workgroups take turns in runs of kStageRun: a run packs (job a), the next run unpacks
// (job b), while both jobs have a full run left; what remains of a, then of b, follows.
// Runs of 64 to 256 single-wavefront workgroups measured 10 % faster than alternating
// workgroup by workgroup or in runs of 16 (fewer read/write turnarounds in HBM) and 7 % faster
// than runs of 8192; with the per-XCD mapping above, 64 is level with or just ahead of 256.
constexpr uint32_t kStageRunLog2 = 6, kStageRun = 1u << kStageRunLog2;

template <int BYTES>
__global__ __launch_bounds__(kThreads) void nts_stage_kernel(NtsMoveJob a, NtsLayerTab atab, NtsMoveJob b,
                                                             NtsLayerTab btab, uint32_t wg_a, uint32_t wg_b)
{
    const uint32_t both = (wg_a < wg_b ? wg_a : wg_b) & ~(kStageRun - 1u);   // whole runs of both jobs
    const uint32_t bid = blockIdx.x;
    bool is_a;
    uint32_t idx;
    if (bid < 2u * both) {
        const uint32_t run = bid >> kStageRunLog2;
        is_a = (run & 1u) == 0u;
        idx = ((run >> 1) << kStageRunLog2) + (bid & (kStageRun - 1u));
    } else {
        const uint32_t rem = bid - 2u * both;
        is_a = rem < wg_a - both;
        idx = is_a ? both + rem : both + rem - (wg_a - both);
    }
    if (is_a)
        move_vector<BYTES, true, false>(a, atab, xcd_contiguous(idx, a.n_vec), threadIdx.x);
    else
        move_vector<BYTES, false, false>(b, btab, xcd_contiguous(idx, b.n_vec), threadIdx.x);
}

// Pool-to-pool variant: the same lane decomposition with a paged address on both
// sides (job a describes the source side, job b the destination side; their
// linear pointers are unused).  This is what a kernel that stores straight into
// a peer-mapped destination pool would look like within one address space.
template <int BYTES>
__global__ __launch_bounds__(kThreads) void nts_direct_kernel(NtsMoveJob a, NtsLayerTab atab, NtsMoveJob b,
                                                              NtsLayerTab btab)
{
    typedef typename VecOf<BYTES>::type vec_t;
    const uint32_t gv0 = blockIdx.x * kThreads;       // first vector of this wavefront: wave-uniform
    const char *src;
    char *dst;
    if (a.wave_in_frag) {
        // the wavefront lies inside one fragment: fragment arithmetic, both slot loads and both
        // layer pointer loads run on the scalar unit (as in move_vector)
        if (gv0 >= a.n_vec) return;
        uint32_t fl, v0;
        if (a.v_shift >= 0) {
            fl = gv0 >> a.v_shift;
            v0 = gv0 & (a.V - 1u);
        } else {
            fl = fast_div(gv0, a.V_magic);
            v0 = gv0 - fl * a.V;
        }
        const uint32_t t = a.j0 + fl;
        const uint32_t ls = a.T_magic ? fast_div(t, a.T_magic) : t;
        const uint32_t j = t - ls * a.T;
        const int64_t ss = a.slots[j], ds = b.slots[j];
        const uint64_t in_frag = uint64_t(v0 + threadIdx.x) * BYTES;
        src = atab.p[a.lc0 + ls] + ss * a.stride + a.head_off + in_frag;
        dst = btab.p[a.lc0 + ls] + ds * b.stride + b.head_off + in_frag;
    } else {
        const uint32_t gv = gv0 + threadIdx.x;
        if (gv >= a.n_vec) return;
        uint32_t fl, v;
        if (a.v_shift >= 0) {
            fl = gv >> a.v_shift;
            v = gv & (a.V - 1u);
        } else {
            fl = fast_div(gv, a.V_magic);
            v = gv - fl * a.V;
        }
        const uint32_t t = a.j0 + fl;
        const uint32_t ls = a.T_magic ? fast_div(t, a.T_magic) : t;
        const uint32_t j = t - ls * a.T;
        const int64_t ss = a.slots[j], ds = b.slots[j];
        src = atab.p[a.lc0 + ls] + ss * a.stride + a.head_off + uint64_t(v) * BYTES;
        dst = btab.p[a.lc0 + ls] + ds * b.stride + b.head_off + uint64_t(v) * BYTES;
    }
    const vec_t x = __builtin_nontemporal_load(reinterpret_cast<const vec_t *>(src));
    store_stream(x, dst);
}

uint64_t magic_of(uint32_t d) { return d > 1 ? UINT64_MAX / d + 1 : 0; }

}  // namespace

// Largest fragment count one launch may cover: lanes = vectors < 2^31.
int64_t nts_max_frags_per_launch(const nts_plan *pl)
{
    static_assert(kThreads == kNtsLanes, "the host geometry assumes single-wavefront workgroups");
    return nts_host_max_frags_per_launch(pl->frag_bytes, pl->vec);
}

void nts_make_job(NtsMoveMode mode, const nts_plan *pl, int64_t q0, int64_t n_frag, char *linear,
                  NtsMoveJob *job)
{
    const bool pack = mode == NTS_MOVE_PACK;
    const uint32_t V = uint32_t(pl->frag_bytes / pl->vec);
    job->slots = pack ? pl->d_sslot : pl->d_dslot;
    job->linear = linear;
    job->stride = pack ? pl->src_stride : pl->dst_stride;
    job->head_off = int64_t(pack ? pl->src_head_off : pl->dst_head_off) * pl->D * pl->e;
    job->T = uint32_t(pl->T);
    job->T_magic = magic_of(job->T);
    job->V = V;
    job->V_magic = magic_of(V);
    job->v_shift = -1;
    if ((V & (V - 1)) == 0) {
        int s = 0;
        while ((1u << s) < V) ++s;
        job->v_shift = s;
    }
    job->lc0 = uint32_t(q0 / pl->T);
    job->j0 = uint32_t(q0 % pl->T);
    job->n_vec = uint32_t(n_frag * V);
    job->wave_in_frag = (V % kThreads) == 0 ? 1 : 0;
    job->frags_in_wave = (V == 32 || V == 16) ? kThreads / V : 0;
}

// A plan ranked by destination slot is packed and unpacked in that order inside the pipeline:
// what lies in the staging buffers is no output, and the unpack half then writes upwards.
// Both halves of a chunk must agree, so every pipeline-internal job goes through here.
static void use_rank_order(NtsMoveMode mode, const nts_plan *pl, NtsMoveJob *job)
{
    if (!pl->d_sslot_by_dst) return;
    job->slots = mode == NTS_MOVE_PACK ? pl->d_sslot_by_dst : pl->d_dslot_by_dst;
}

hipError_t nts_launch_move(NtsMoveMode mode, const nts_plan *pl, int64_t q0, int64_t n_frag,
                           const NtsLayerTab &tab, char *linear, bool linear_is_staging, bool rank_order,
                           hipStream_t st)
{
    if (n_frag <= 0) return hipSuccess;
    NtsMoveJob job;
    nts_make_job(mode, pl, q0, n_frag, linear, &job);
    if (rank_order) use_rank_order(mode, pl, &job);
    const dim3 grid((job.n_vec + kThreads - 1) / kThreads), block(kThreads);
#define NTS_LAUNCH(B, P)                                                                              \
    {                                                                                                 \
        if (linear_is_staging) hipLaunchKernelGGL((nts_move_kernel<B, P, false>), grid, block, 0, st, job, tab); \
        else hipLaunchKernelGGL((nts_move_kernel<B, P, true>), grid, block, 0, st, job, tab);         \
    }
    if (mode == NTS_MOVE_PACK) {
        if (pl->vec == 16) NTS_LAUNCH(16, true)
        else if (pl->vec == 8) NTS_LAUNCH(8, true)
        else NTS_LAUNCH(4, true)
    } else {
        if (pl->vec == 16) NTS_LAUNCH(16, false)
        else if (pl->vec == 8) NTS_LAUNCH(8, false)
        else NTS_LAUNCH(4, false)
    }
#undef NTS_LAUNCH
    return hipGetLastError();
}

hipError_t nts_launch_stage(const nts_plan *ppl, int64_t pack_q0, int64_t pack_n, char *pack_buf,
                            const NtsLayerTab &stab, const nts_plan *upl, int64_t unpack_q0,
                            int64_t unpack_n, char *unpack_buf, const NtsLayerTab &dtab, hipStream_t st)
{
    const bool has_a = ppl && pack_n > 0, has_b = upl && unpack_n > 0;
    if (!has_a && !has_b) return hipSuccess;
    if (has_a && has_b && ppl->vec != upl->vec) {
        // two plans whose vector widths differ cannot share the kernel instance
        const hipError_t e = nts_launch_move(NTS_MOVE_UNPACK, upl, unpack_q0, unpack_n, dtab, unpack_buf, true, true, st);
        if (e != hipSuccess) return e;
        return nts_launch_move(NTS_MOVE_PACK, ppl, pack_q0, pack_n, stab, pack_buf, true, true, st);
    }
    NtsMoveJob a = {}, b = {};   // an absent side is a job of zero vectors
    if (has_a) nts_make_job(NTS_MOVE_PACK, ppl, pack_q0, pack_n, pack_buf, &a);
    if (has_b) nts_make_job(NTS_MOVE_UNPACK, upl, unpack_q0, unpack_n, unpack_buf, &b);
    if (has_a) use_rank_order(NTS_MOVE_PACK, ppl, &a);
    if (has_b) use_rank_order(NTS_MOVE_UNPACK, upl, &b);
    const int vec = has_a ? ppl->vec : upl->vec;
    const uint32_t wg_a = (a.n_vec + kThreads - 1) / kThreads, wg_b = (b.n_vec + kThreads - 1) / kThreads;
    const dim3 grid(wg_a + wg_b), block(kThreads);
    if (vec == 16) hipLaunchKernelGGL((nts_stage_kernel<16>), grid, block, 0, st, a, stab, b, dtab, wg_a, wg_b);
    else if (vec == 8) hipLaunchKernelGGL((nts_stage_kernel<8>), grid, block, 0, st, a, stab, b, dtab, wg_a, wg_b);
    else hipLaunchKernelGGL((nts_stage_kernel<4>), grid, block, 0, st, a, stab, b, dtab, wg_a, wg_b);
    return hipGetLastError();
}

hipError_t nts_launch_direct(const nts_plan *pl, int64_t q0, int64_t n_frag, const NtsLayerTab &stab,
                             const NtsLayerTab &dtab, hipStream_t st)
{
    if (n_frag <= 0) return hipSuccess;
    NtsMoveJob a, b;
    nts_make_job(NTS_MOVE_PACK, pl, q0, n_frag, nullptr, &a);
    nts_make_job(NTS_MOVE_UNPACK, pl, q0, n_frag, nullptr, &b);
    if (pl->d_sslot_by_dst) {                // walk the tokens in ascending destination-slot order
        a.slots = pl->d_sslot_by_dst;
        b.slots = pl->d_dslot_by_dst;
    }
    const dim3 grid((a.n_vec + kThreads - 1) / kThreads), block(kThreads);
    if (pl->vec == 16) hipLaunchKernelGGL((nts_direct_kernel<16>), grid, block, 0, st, a, stab, b, dtab);
    else if (pl->vec == 8) hipLaunchKernelGGL((nts_direct_kernel<8>), grid, block, 0, st, a, stab, b, dtab);
    else hipLaunchKernelGGL((nts_direct_kernel<4>), grid, block, 0, st, a, stab, b, dtab);
    return hipGetLastError();
}
