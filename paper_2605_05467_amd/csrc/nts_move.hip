// Pack / unpack kernels of the KV migration (paper Sec. 3.2.2: the migration
// kernel copies the scattered per-page KV regions of the moved head slice into
// a contiguous buffer; the receiver does the reverse into its own pages).
//
// Both are pure byte movers bound by HBM bandwidth.  Work decomposition for
// 64-wide wavefronts: a fragment (w*D*elem_bytes contiguous bytes) is cut into
// V vectors of `vec` bytes.  LPF = min(64, next power of two >= V) lanes share
// one fragment, so a wavefront covers 64/LPF fragments per row and walks a
// fragment wider than 64 vectors in `cols` column steps.  A 256-thread
// workgroup owns tile_f = ROWS*4*(64/LPF) consecutive fragments of the stream
// (32..64 KiB), which makes the linear side of the copy one long contiguous
// burst per workgroup while the paged side touches whole fragments.  Each lane
// keeps ROWS independent vector loads in flight before the first store.
#include "nts_internal.h"

namespace {

constexpr int kRows = 8;     // fragments rows per wavefront, all in flight at once
constexpr int kWaves = 4;    // wavefronts per workgroup
constexpr int kThreads = 64 * kWaves;

template <int BYTES> struct VecOf;
template <> struct VecOf<16> { typedef uint32_t type __attribute__((ext_vector_type(4))); };
template <> struct VecOf<8> { typedef uint32_t type __attribute__((ext_vector_type(2))); };
template <> struct VecOf<4> { typedef uint32_t type; };

template <int BYTES, bool PACK>
__global__ __launch_bounds__(kThreads) void nts_move_kernel(NtsMoveGeom g, NtsPagedSide pg,
                                                            NtsLayerTab tab, char *linear)
{
    typedef typename VecOf<BYTES>::type vec_t;
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wv = threadIdx.x >> 6;
    const uint32_t lpf = 1u << g.lpf_log2;
    const uint32_t fpw = 64u >> g.lpf_log2;          // fragments per wavefront row
    const uint32_t sub = lane >> g.lpf_log2;          // which fragment of the row
    const uint32_t vl = lane & (lpf - 1u);            // vector lane inside the fragment

    const uint32_t tile0 = blockIdx.x * g.tile_f;     // first fragment of this tile, launch-local
    // slab / token of the tile's first fragment: one division per workgroup
    const uint32_t t0 = g.j0 + tile0;
    const uint32_t lc_t = g.lc0 + t0 / g.T;
    const uint32_t j_t = t0 % g.T;

    const char *paged[kRows];
    char *lin[kRows];
    bool ok[kRows];
#pragma unroll
    for (int r = 0; r < kRows; ++r) {
        const uint32_t f_tile = (uint32_t(r) * kWaves + wv) * fpw + sub;   // fragment inside the tile
        const uint32_t fl = tile0 + f_tile;
        ok[r] = fl < g.n_frag;
        uint32_t lc = lc_t, j = j_t + f_tile;
        while (j >= g.T) { j -= g.T; ++lc; }
        int64_t slot = 0;
        const char *base = nullptr;
        if (ok[r]) {
            slot = pg.slots[j];
            base = tab.p[lc];
        }
        paged[r] = base + slot * pg.stride + pg.head_off;
        lin[r] = linear + uint64_t(fl) * g.frag_bytes;
    }

    for (uint32_t col = 0; col < g.cols; ++col) {
        const uint32_t v = col * lpf + vl;
        const bool inb = v < g.V;
        const uint64_t off = uint64_t(v) * BYTES;
        vec_t buf[kRows];
#pragma unroll
        for (int r = 0; r < kRows; ++r) {
            if (ok[r] && inb) {
                const vec_t *s = reinterpret_cast<const vec_t *>((PACK ? paged[r] : lin[r]) + off);
                buf[r] = __builtin_nontemporal_load(s);
            }
        }
#pragma unroll
        for (int r = 0; r < kRows; ++r) {
            if (ok[r] && inb) {
                vec_t *d = reinterpret_cast<vec_t *>(const_cast<char *>(PACK ? lin[r] : paged[r]) + off);
                __builtin_nontemporal_store(buf[r], d);
            }
        }
    }
}

}  // namespace

hipError_t nts_launch_move(NtsMoveMode mode, const nts_plan *pl, int64_t q0, int64_t n_frag,
                           const NtsLayerTab &tab, char *linear, hipStream_t st)
{
    if (n_frag <= 0) return hipSuccess;
    NtsMoveGeom g;
    g.T = uint32_t(pl->T);
    g.lc0 = uint32_t(q0 / pl->T);
    g.j0 = uint32_t(q0 % pl->T);
    g.n_frag = uint32_t(n_frag);
    g.V = uint32_t(pl->frag_bytes / pl->vec);
    uint32_t lg = 0;
    while (lg < 6 && (1u << lg) < g.V) ++lg;
    g.lpf_log2 = lg;
    const uint32_t lpf = 1u << lg;
    g.cols = (g.V + lpf - 1) / lpf;
    g.tile_f = uint32_t(kRows * kWaves) * (64u >> lg);
    g.frag_bytes = uint64_t(pl->frag_bytes);

    NtsPagedSide pg;
    const bool pack = mode == NTS_MOVE_PACK;
    pg.slots = pack ? pl->d_sslot : pl->d_dslot;
    pg.stride = pack ? pl->src_stride : pl->dst_stride;
    pg.head_off = int64_t(pack ? pl->src_head_off : pl->dst_head_off) * pl->D * pl->e;

    const uint64_t tiles = (uint64_t(n_frag) + g.tile_f - 1) / g.tile_f;
    const dim3 grid((unsigned)tiles), block(kThreads);
#define NTS_LAUNCH(B, P) hipLaunchKernelGGL((nts_move_kernel<B, P>), grid, block, 0, st, g, pg, tab, linear)
    if (pack) {
        if (pl->vec == 16) NTS_LAUNCH(16, true);
        else if (pl->vec == 8) NTS_LAUNCH(8, true);
        else NTS_LAUNCH(4, true);
    } else {
        if (pl->vec == 16) NTS_LAUNCH(16, false);
        else if (pl->vec == 8) NTS_LAUNCH(8, false);
        else NTS_LAUNCH(4, false);
    }
#undef NTS_LAUNCH
    return hipGetLastError();
}
