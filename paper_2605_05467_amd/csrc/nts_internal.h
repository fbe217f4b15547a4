// Internal declarations shared by the library's translation units.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>

#include "nitsum_kvmig.h"

#define NTS_MAX_LAYER_PTRS (2 * NTS_MAX_LAYERS)

struct nts_ctx {
    int device = 0;
    hipStream_t aux = nullptr;          // unpack side of the double buffer
    hipEvent_t ev_fork = nullptr;
    hipEvent_t ev_packed[2] = {nullptr, nullptr};
    hipEvent_t ev_unpacked[2] = {nullptr, nullptr};
    int n_plans = 0;
    std::string err;
};

struct nts_plan {
    nts_ctx *ctx = nullptr;
    // geometry
    int32_t L = 0, D = 0, e = 0, p = 1, Hs = 0, Hd = 0, src_head_off = 0, dst_head_off = 0, w = 0;
    int64_t S_src = 0, S_dst = 0, src_stride = 0, dst_stride = 0;
    int64_t T = 0, F = 0, frag_bytes = 0, X = 0, chunk_frags = 0, chunk_bytes = 0, n_chunks = 0;
    int32_t vec = 16;
    // device index arrays, one allocation
    void *d_block = nullptr;
    int32_t *d_sslot = nullptr;
    int32_t *d_dslot = nullptr;
};

// Base pointers of the 2L per-(layer, K|V) arrays of one pool; passed by value
// as a kernel argument so that a run needs no device-side table.
struct NtsLayerTab {
    char *p[NTS_MAX_LAYER_PTRS];
};

// One launch of the mover covers fragments [q0, q0 + n_frag) of the stream,
// q = (l*2+c)*T + j.
struct NtsMoveGeom {
    uint32_t T;         // tokens per (layer, K|V) slab
    uint32_t lc0, j0;   // q0 split into slab index and token index
    uint32_t n_frag;    // fragments in this launch (< 2^31)
    uint32_t V;         // vectors per fragment
    uint32_t lpf_log2;  // log2 of the lanes that share one fragment (<= 6)
    uint32_t cols;      // ceil(V / lanes per fragment)
    uint32_t tile_f;    // fragments per workgroup
    uint64_t frag_bytes;
};

struct NtsPagedSide {
    const int32_t *slots;  // device [T]
    int64_t stride;        // bytes between token slots
    int64_t head_off;      // byte offset of the moved slice inside a token row
};

enum NtsMoveMode { NTS_MOVE_PACK = 0, NTS_MOVE_UNPACK = 1 };

// nts_move.hip
hipError_t nts_launch_move(NtsMoveMode mode, const nts_plan *pl, int64_t q0, int64_t n_frag,
                           const NtsLayerTab &tab, char *linear, hipStream_t st);

// nts_plan.hip
hipError_t nts_launch_flatten(const int32_t *d_tok_off, const int32_t *d_pg_off,
                              const int32_t *d_pages, int n_req, uint32_t T, int p,
                              int64_t n_pool_pages, int32_t *d_slots, uint32_t *d_bitmap,
                              int32_t *d_err, hipStream_t st);
