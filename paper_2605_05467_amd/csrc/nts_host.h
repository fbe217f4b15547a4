// Host-side integer arithmetic of the KV-migration library: routing, the
// validation, prefix sums and chunk geometry of a plan, and the overlap checks
// of a batch.  Plain C++ with no GPU runtime behind it, so that the same code
// can also be compiled for the CPU alone and run under AddressSanitizer /
// UndefinedBehaviorSanitizer (tests/host_sanitize).
#pragma once

#include <stdint.h>

#include <vector>

#include "nitsum_kvmig.h"

// lanes of one (single-wavefront) workgroup of the movers; a launch covers fewer than 2^31 lanes
constexpr int kNtsLanes = 64;

// What nts_plan_create derives from a descriptor before anything touches the GPU.
struct NtsGeometry {
    int64_t src_stride = 0, dst_stride = 0;   // bytes between token slots
    int64_t frag_bytes = 0;                   // w * D * elem_bytes
    int32_t vec = 16;                         // bytes per lane access: 16, 8 or 4
    int64_t T = 0, NP = 0;                    // tokens and pages over all requests
    int64_t F = 0, X = 0;                     // fragments and payload bytes
    int64_t chunk_frags = 0, chunk_bytes = 0, n_chunks = 0;
    std::vector<int32_t> tok_off, pg_off;     // exclusive prefix sums over requests, n_req + 1 each
};

// Sec. 3.2.2: heads [r*H/N, (r+1)*H/N) per rank; the slice to move is the intersection.
int nts_host_route(int H, int Ns, int rs, int Nd, int rd, int *src_head_off, int *dst_head_off, int *w);

// Largest fragment count one launch may cover (one lane per vector, lanes < 2^31).
int64_t nts_host_max_frags_per_launch(int64_t frag_bytes, int32_t vec);

// Validates `d` and fills `g`.  NTS_OK, or NTS_EINVAL / NTS_ENOMEM with *why set to a
// static message.  Reads d->ctx_len (host) but neither page table.
int nts_host_plan_geometry(const nts_desc *d, NtsGeometry *g, const char **why);

// Fragment range [*q0, *q0 + *n) of chunk k.  NTS_EINVAL when k is not a chunk.
int nts_host_chunk_range(int64_t F, int64_t chunk_frags, int64_t n_chunks, int64_t k, int64_t *q0, int64_t *n);

// Byte range [lo, hi) of one (layer, K|V) array of a pool of a batch, as integers.
struct NtsByteRange {
    uintptr_t lo, hi;
    int is_dst;
};

// NTS_EALIAS when any destination range meets any source range or when any range meets the
// staging area [stg, stg + stg_bytes); sorts `ranges` by start.  *why: static message.
int nts_host_alias_sweep(std::vector<NtsByteRange> &ranges, uintptr_t stg, int64_t stg_bytes, const char **why);

// 2 * (largest chunk_bytes rounded up to 16): staging area of a batch.
int64_t nts_host_batch_staging_bytes(const int64_t *chunk_bytes, int n);
