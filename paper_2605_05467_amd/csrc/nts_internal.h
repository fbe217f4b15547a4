// Internal declarations shared by the library's translation units.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <map>
#include <string>
#include <tuple>
#include <vector>

#include "nitsum_kvmig.h"

#define NTS_MAX_LAYER_PTRS (2 * NTS_MAX_LAYERS)

struct nts_ctx {
    int device = 0;
    hipStream_t aux = nullptr;          // planning work (copies, flatten kernel)
    void *static_staging = nullptr;     // this device's copy of the library's static staging array
    void *h_pinned = nullptr;           // pinned host staging for plan metadata
    size_t h_pinned_bytes = 0;
    // Device blocks of freed plans, kept for reuse.  A block may still be read by kernels of
    // the plan that owned it; `ev` (recorded when it was freed) orders them before reuse.
    // Blocks are reused oldest first, so in a steady loop the wait is already over.
    struct Spare {
        void *ptr = nullptr;
        size_t bytes = 0;
        hipEvent_t ev = nullptr;
        bool pending = false;           // ev was recorded and has not been waited on by `aux`
        uint64_t age = 0;               // order of freeing
    };
    static constexpr int kSpares = 16;          // a TP switch of eight GPUs has up to 15 pairs per GPU
    Spare spare[kSpares];
    uint64_t free_count = 0;
    int n_plans = 0;
    std::string err;
    // configurations nts_shard_linear_tune found fastest, by (M, shard rows, reduction length, format)
    struct TunedLinear {
        int tiled;      // tile width of the tiled kernel (256, 192 or 128), 0: streaming / decode kernel
        int tiled_rows; // its tile height (256 or 128)
        int mt, cw, rt, nsets, splits, ks;
    };
    std::map<std::tuple<int, int, int, int>, TunedLinear> tuned_linear;
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
    size_t d_block_bytes = 0;
    int32_t *d_sslot = nullptr;
    int32_t *d_dslot = nullptr;
    // both slot lists in ascending destination-slot order (plan flag NTS_ORDER_BY_DST), else null
    int32_t *d_sslot_by_dst = nullptr;
    int32_t *d_dslot_by_dst = nullptr;
    // run list (plan flag NTS_DETECT_RUNS): n_runs + 1 token indices, the last one T
    bool has_runs = false;
    int32_t *d_run_start = nullptr;
    int64_t n_runs = 0;
    // host copies of the slot lists, fetched on first use by the per-fragment memcpy baseline
    std::vector<int32_t> h_sslot, h_dslot, h_run_start;
    // streams this plan's run calls have launched on; their pending work reads d_block.  A fixed
    // array, so that a run call never allocates; with more streams than it holds, nts_plan_free
    // waits for the whole device instead.
    static constexpr int kMaxStreams = 8;
    hipStream_t used_streams[kMaxStreams] = {};
    int n_used_streams = 0;
    bool more_streams = false;
};

// Base pointers of the 2L per-(layer, K|V) arrays of one pool; passed by value
// as a kernel argument so that a run needs no device-side table.
struct NtsLayerTab {
    char *p[NTS_MAX_LAYER_PTRS];
};

// One job of the mover: fragments [q0, q0 + n_frag) of the stream,
// q = (l*2+c)*T + j, against a linear buffer that starts at fragment q0.
// Every lane moves one vector; n_vec = n_frag * V < 2^31.
struct NtsMoveJob {
    const int32_t *slots;  // device [T]: slot of every migrated token on the paged side
    char *linear;          // stream / staging side
    int64_t stride;        // bytes between token slots of the paged side
    int64_t head_off;      // byte offset of the moved slice inside a token row
    uint64_t T_magic;      // reciprocal of T for exact division; 0 when T == 1
    uint64_t V_magic;      // reciprocal of V (used when V is not a power of two)
    uint32_t T;            // tokens per (layer, K|V) slab
    uint32_t V;            // vectors per fragment
    int32_t v_shift;       // log2(V) if V is a power of two, else -1
    uint32_t lc0, j0;      // q0 split into slab index and token index
    uint32_t n_vec;        // vectors (= lanes) of this job
    uint32_t wave_in_frag; // 1 when V is a multiple of 64: a wavefront never straddles fragments
    uint32_t frags_in_wave; // 2 or 4 when V is 32 or 16: whole fragments per full wavefront; else 0
};

enum NtsMoveMode { NTS_MOVE_PACK = 0, NTS_MOVE_UNPACK = 1 };

// nts_move.hip
int64_t nts_max_frags_per_launch(const nts_plan *pl);
// linear_is_staging: the stream side is a small buffer reused within moments (a chunk), not the whole stream;
// rank_order: pipeline-internal move that follows the plan's destination ranking if it has one (the
// stream handed out by pack / unpack and their chunk calls always keeps the caller's token order)
hipError_t nts_launch_move(NtsMoveMode mode, const nts_plan *pl, int64_t q0, int64_t n_frag,
                           const NtsLayerTab &tab, char *linear, bool linear_is_staging, bool rank_order,
                           hipStream_t st);
// pack fragments [pack_q0, +pack_n) of plan `ppl` into pack_buf and unpack fragments
// [unpack_q0, +unpack_n) of plan `upl` from unpack_buf in one launch (either count may be
// zero, and then its plan may be null; the two plans may differ)
hipError_t nts_launch_stage(const nts_plan *ppl, int64_t pack_q0, int64_t pack_n, char *pack_buf,
                            const NtsLayerTab &stab, const nts_plan *upl, int64_t unpack_q0,
                            int64_t unpack_n, char *unpack_buf, const NtsLayerTab &dtab, hipStream_t st);
// pool-to-pool move of fragments [q0, q0 + n_frag) with no stream in between
hipError_t nts_launch_direct(const nts_plan *pl, int64_t q0, int64_t n_frag, const NtsLayerTab &stab,
                             const NtsLayerTab &dtab, hipStream_t st);

// nts_plan.hip
struct NtsFlattenSide {
    const int32_t *pages;   // device: page ids, CSR by request
    int32_t *slots;         // device [T]: out
    uint32_t *bitmap;       // device, one bit per pool slot, zeroed; nullptr = no uniqueness check
    int64_t n_pool_pages;
};
hipError_t nts_launch_flatten(const int32_t *d_tok_off, const int32_t *d_pg_off, int n_req, uint32_t T,
                              int p, const NtsFlattenSide &src, const NtsFlattenSide &dst,
                              int32_t *d_err, hipStream_t st);
// run_start[0 .. n) = first token of every run in token order, run_start[n] = T, *d_n_runs = n;
// d_block_count: scratch of ceil(T / 256) entries
hipError_t nts_launch_detect_runs(const int32_t *d_sslot, const int32_t *d_dslot, uint32_t T,
                                  int32_t *d_block_count, int32_t *d_run_start, int32_t *d_n_runs,
                                  hipStream_t st);

// tokens in ascending destination-slot order (plan flag NTS_ORDER_BY_DST): both slot lists scattered
// into rank order; d_word_prefix: n_words entries, d_block_count: ceil(n_words / 256) entries of scratch
hipError_t nts_launch_rank_by_dst(const int32_t *d_sslot, const int32_t *d_dslot, uint32_t T,
                                  const uint32_t *d_bitmap, uint32_t n_words, int32_t *d_word_prefix,
                                  int32_t *d_block_count, int32_t *d_ss_sorted, int32_t *d_ds_sorted, hipStream_t st);

// nts_linear.hip: Y[M][Nn] = X[M][K] . A[Nn][K]^T, bf16 or f16 in, fp32 accumulate, same format out
struct NtsStreamCfg {
    int mt = 1;       // batch rows per workgroup / 32
    int cw = 4;       // consumer wavefronts per workgroup
    int rt = 1;       // 32-row weight tiles per consumer (decode kernel: 16-row blocks per wavefront)
    int nsets = 4;    // weight register sets in rotation (nsets - 1 slabs in flight per wavefront)
    int splits = 1;   // K splits (> 1: fp32 partial sums in the workspace, reduced in split order)
    int ks = 0;       // > 0: the decode kernel (16 weight rows per workgroup, ks wavefronts sharing K) instead
};
NtsStreamCfg nts_linear_stream_config(int M, int Nn, int K);
int nts_linear_use_tiled(int M, int Nn, int K, int *rows);   // tile width (and height) of the tiled kernel, 0: not tiled
// one way of running a problem: the tiled kernel, or the streaming / decode kernel with `cfg`
struct NtsLinearCand {
    int tiled = 0;          // tile width of the tiled kernel (256, 192 or 128), 0: streaming / decode kernel
    int tiled_rows = 256;   // its tile height (256 or 128)
    NtsStreamCfg cfg;
    double est_us = 0.;
};
int nts_linear_candidates(int M, int Nn, int K, double slack, NtsLinearCand *out, int max_out);
hipError_t nts_launch_linear_stream(const uint16_t *X, int64_t ldx, const uint16_t *A, int64_t lda, uint16_t *Y,
                                    int64_t ldy, float *part, const NtsStreamCfg &c, int M, int Nn, int K,
                                    bool f16, hipStream_t st);
hipError_t nts_launch_linear_tiled(const uint16_t *X, int64_t ldx, const uint16_t *A, int64_t lda,
                                   uint16_t *Y, int64_t ldy, int M, int Nn, int K, int tile_rows, int tile_cols,
                                   bool f16, hipStream_t st);
