/*
 * nitsum_kvmig.h: C ABI of the MI355X KV-cache migration library.
 *
 * The operation is the "aggregated and pipelined KV migration" of the Nitsum
 * paper, Sec. 3.2.2: when the tensor-parallel (TP) level of a serving group
 * changes, every GPU must hand the KV heads it no longer owns to the GPUs that
 * own them under the new level.  KV lives in a paged pool, so the bytes of one
 * request are scattered; the method gathers the moved head slice of every
 * token into a contiguous stream ("pack"), moves the stream in chunks through
 * two staging buffers so that copying and transmission overlap, and the
 * receiver scatters the stream into its own paged pool ("unpack").
 *
 * Conventions
 *   - All functions return NTS_OK (0) or a negative nts_status.  Nothing throws
 *     or aborts across this boundary.  nts_last_error() gives the text of the
 *     last failure on a context.
 *   - "host" / "device" on a pointer says where the memory lives.  The caller
 *     owns every buffer it passes in (pools, stream, staging) and the HIP
 *     stream; the library owns only the device index arrays inside a plan.
 *   - run calls only enqueue work on the given HIP stream (a hipStream_t passed
 *     as void*, NULL = the default stream), allocate nothing and never block
 *     the host.  A context and its plans may be used by one host thread at a time.
 *     A context keeps a pinned host buffer and up to sixteen spare device blocks between
 *     plans so that planning in a steady loop allocates nothing.
 *
 * Data layout (the paper fixes none; this is the layout of this library)
 *   pool      per GPU and per (layer l, c = 0 for K / 1 for V) one array
 *             [S slots][H_local heads][D elements] of elem_bytes each, given by
 *             its device base pointer: 2L pointers, index l*2+c.  Consecutive
 *             slots are token_stride bytes apart (0 means H_local*D*elem_bytes).
 *             One allocation [L][2][S][H_local][D] is the common special case.
 *   fragment  the w*D*elem_bytes contiguous bytes that one (layer, K|V, token)
 *             contributes: heads [head_off, head_off+w) of that token's row.
 *   stream    fragments in the order [l][c][j], j = 0..T-1 the flattened token
 *             index (requests in the order given, tokens by position).  Chunk k
 *             is bytes [k*chunk_bytes, (k+1)*chunk_bytes) of the stream, with
 *             chunk_bytes a multiple of the fragment size, so the stream does
 *             not depend on the staging size.
 */
#ifndef NITSUM_KVMIG_H
#define NITSUM_KVMIG_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct nts_ctx nts_ctx;
typedef struct nts_plan nts_plan;

typedef enum nts_status {
    NTS_OK = 0,
    NTS_EINVAL = -1,  /* null pointer, bad geometry, head slice outside a pool's heads */
    NTS_ERANGE = -2,  /* a page id lies outside its pool */
    NTS_EDUP = -3,    /* two migrated tokens share a destination slot */
    NTS_EALIAS = -4,  /* source and destination byte ranges overlap */
    NTS_ENOMEM = -5,  /* host or device allocation failed */
    NTS_EHIP = -6     /* a HIP call failed; see nts_last_error() */
} nts_status;

enum {
    NTS_MAX_LAYERS = 96,          /* 2*L base pointers travel as kernel arguments */
    NTS_VALIDATE_UNIQUE_DST = 1u, /* plan flag: check destination slots are distinct */
    NTS_DETECT_RUNS = 2u,         /* plan flag: also find the runs of neighbouring slots */
    NTS_ORDER_BY_DST = 4u,        /* plan flag: also rank the tokens by destination slot; nts_run_migrate[_batch, _static]
                                     and nts_run_migrate_direct then move them in that order */
    NTS_DEFAULT_STAGING_BYTES = 64 << 20,
    NTS_STATIC_STAGING_BYTES = 32 << 20   /* both buffers of nts_run_migrate_static together */
};

/*
 * One (source GPU -> destination GPU) migration: the metadata the paper's
 * handshake exchanges (request, KV heads, context length; Sec. 3.2.2) plus the
 * page tables of both ends.
 */
typedef struct nts_desc {
    int32_t L;             /* layers */
    int32_t D;             /* head dimension in elements */
    int32_t elem_bytes;    /* 1, 2 or 4 */
    int32_t page_size;     /* p >= 1 tokens per page */
    int32_t Hs;            /* heads held per token by the source GPU (H / Ns) */
    int32_t Hd;            /* heads held per token by the destination GPU (H / Nd) */
    int32_t src_head_off;  /* first moved head, local to the source's Hs */
    int32_t dst_head_off;  /* first moved head, local to the destination's Hd */
    int32_t w;             /* heads moved, > 0 (see nts_route) */
    int32_t n_req;         /* requests to migrate, >= 0 */
    int64_t S_src;         /* source pool capacity in token slots (multiple of p) */
    int64_t S_dst;         /* destination pool capacity in token slots */
    const int32_t *ctx_len;   /* host [n_req]: tokens of each request, >= 0 */
    const int32_t *src_pages; /* host: page ids, CSR by request, ceil(ctx_len/p) each */
    const int32_t *dst_pages; /* host: same shape; destination pages must be distinct */
    int64_t src_token_stride; /* bytes between source slots; 0 = Hs*D*elem_bytes; at most 2^30 */
    int64_t dst_token_stride; /* bytes between destination slots; 0 = Hd*D*elem_bytes */
    int64_t staging_bytes;    /* B: size of ONE staging buffer; 0 = 64 MiB.  Rounded
                                 down to a whole number of fragments (at least one). */
    uint32_t flags;           /* NTS_VALIDATE_UNIQUE_DST | NTS_DETECT_RUNS | NTS_ORDER_BY_DST */
    uint32_t reserved;
} nts_desc;

typedef struct nts_info {
    int64_t T;            /* tokens migrated */
    int64_t F;            /* fragments = T * L * 2 */
    int64_t frag_bytes;   /* w * D * elem_bytes */
    int64_t X;            /* payload bytes = F * frag_bytes = stream size */
    int64_t chunk_frags;  /* fragments per chunk */
    int64_t chunk_bytes;  /* chunk_frags * frag_bytes <= staging_bytes */
    int64_t n_chunks;     /* ceil(F / chunk_frags); 0 for an empty plan */
    int32_t vec_bytes;    /* bytes each lane moves per access (16, 8 or 4) */
    int32_t n_runs;       /* runs found with NTS_DETECT_RUNS; 0 without the flag */
} nts_info;

/* Create a context on HIP device `device_id`.  *out is owned by the caller
 * until nts_free.  Fails with NTS_EHIP when no such device exists. */
int nts_init(int device_id, nts_ctx **out);

/* Destroy a context.  Plans made from it must be freed first. */
int nts_free(nts_ctx *ctx);

/* Text of the last failure on `ctx` (host string owned by the context, valid
 * until the next failing call); never NULL. */
const char *nts_last_error(const nts_ctx *ctx);

/* Name of a status code; never NULL. */
const char *nts_strerror(int status);

/*
 * Routing step (host only, integer).  KV heads are split evenly over the GPUs
 * of a TP group (Sec. 3.2.2); rank r of a group at level N holds heads
 * [r*H/N, (r+1)*H/N).  The heads to move from source rank rs (level Ns) to
 * destination rank rd (level Nd) are the intersection of the two intervals.
 * Outputs are local to each side's own range; *w == 0 means nothing moves.
 * NTS_EINVAL if H is not a multiple of Ns and Nd or a rank is out of range.
 */
int nts_route(int H, int Ns, int rs, int Nd, int rd,
              int *src_head_off, int *dst_head_off, int *w);

/*
 * Planning step.  Flattens the request list and page tables of `d` into one
 * source slot and one destination slot per migrated token (token t of a
 * request sits in slot pages[t / p] * p + t % p; only the ctx_len valid tokens
 * of a last partial page move), validates them on the GPU and fixes the chunk
 * geometry.  Host arrays in `d` are copied and may be freed on return.  The
 * call synchronises with the device.  Errors: NTS_EINVAL (null pointers, w <= 0,
 * head slice outside Hs / Hd, elem_bytes not 1/2/4, fragment size or strides
 * not a multiple of 4 bytes, L > NTS_MAX_LAYERS, negative ctx_len, more than
 * 2^31-1 tokens, D > 2^20, more than 65536 heads, a token stride above 2^30
 * bytes, NTS_ORDER_BY_DST without NTS_VALIDATE_UNIQUE_DST), NTS_ERANGE, NTS_EDUP (only with NTS_VALIDATE_UNIQUE_DST),
 * NTS_ENOMEM, NTS_EHIP.  A plan with zero tokens is legal; its run calls do nothing.
 */
int nts_plan_create(nts_ctx *ctx, const nts_desc *d, nts_plan **out);

/*
 * Frees a plan (NULL is allowed).  Run calls of the plan that are still queued
 * or running stay valid: the plan's device arrays are kept until that work has
 * finished.  With work on one stream the call does not wait (the arrays are
 * handed to the next plan of the context, which orders itself behind that work);
 * with work on several streams it waits for them, beyond eight streams for the
 * whole device.  NTS_EHIP if the runtime reports an error; the plan is gone
 * either way.
 */
int nts_plan_free(nts_plan *plan);
int nts_plan_info(const nts_plan *plan, nts_info *out);

/*
 * Runs (plan flag NTS_DETECT_RUNS).  With small pages a request's KV lies in
 * many scattered regions, with a contiguous per-request layout in few (paper
 * Sec. 3.2.2).  Token j continues the run of token j-1 when it sits in the next
 * slot on the source side and in the next slot on the destination side; the
 * plan then holds, on the device, the first token of every run in token order.
 * When a fragment is a whole token row on both sides a run is one contiguous
 * region per (layer, K|V); nts_run_memcpy_baseline's merge_runs uses the list.
 * The kernels' results do not depend on the flag.
 * nts_plan_runs copies the list to the host: run_start_host receives
 * n_runs + 1 int32 (n_runs from nts_plan_info), the last one T.  Synchronises.
 * Errors: NTS_EINVAL (null, or the plan was made without the flag).
 */
int nts_plan_runs(nts_plan *plan, int32_t *run_start_host);

/* Copy the flattened slot lists back to the host (each int32 [T], either may
 * be NULL).  Synchronises; meant for tests and debugging. */
int nts_plan_slots(const nts_plan *plan, int32_t *sslot_host, int32_t *dslot_host);

/*
 * Pack (aggregate): stream_out[l][c][j][0:w][0:D] =
 *     src[l][c][sslot[j]][src_head_off : src_head_off+w][0:D]   for all l, c, j.
 * src_layer_ptrs: host array of 2L device pointers.  stream_out: device, X bytes.
 * Pointers must be aligned to vec_bytes.
 */
int nts_run_pack(nts_plan *plan, const void *const *src_layer_ptrs, void *stream_out,
                 void *hip_stream);

/* Pack chunk k only, into a device buffer of chunk_bytes (the last chunk may
 * be shorter).  This is what a sender calls once per staging buffer.  The chunk
 * calls treat their buffer as staging that is consumed (or was produced) moments
 * later: ordinary, cache-allocating accesses on that side, where nts_run_pack /
 * nts_run_unpack stream past the caches (pack -> unpack through two 64 MiB
 * buffers on one GPU: 6.3 against 5.4 TB/s). */
int nts_run_pack_chunk(nts_plan *plan, const void *const *src_layer_ptrs, int64_t k,
                       void *chunk_out, void *hip_stream);

/*
 * Unpack: dst[l][c][dslot[j]][dst_head_off : dst_head_off+w][0:D] =
 *     stream_in[l][c][j][0:w][0:D]; every other byte of dst keeps its value.
 * The paper does not describe the receiving side; this is the mirror of pack.
 */
int nts_run_unpack(nts_plan *plan, const void *stream_in, void *const *dst_layer_ptrs,
                   void *hip_stream);
int nts_run_unpack_chunk(nts_plan *plan, const void *chunk_in, int64_t k,
                         void *const *dst_layer_ptrs, void *hip_stream);

/*
 * The whole migration on one GPU with the wire left out: the double buffering
 * of Sec. 3.2.2 with the unpack as the consumer instead of the interconnect.
 * staging: device, 2 * chunk_bytes (two buffers).  Stage k is ONE kernel launch
 * whose workgroups alternate between packing chunk k into buffer k&1 and
 * unpacking chunk k-1 from the other buffer, so the two copies overlap; the
 * n_chunks + 1 launches go to hip_stream in order, which hands each buffer
 * from its producer to its consumer.  The kernels access the pools with
 * non-temporal loads and stores and the staging buffers with ordinary ones, so
 * that buffers which together fit the GPU's memory-side cache (256 MiB on
 * MI355X) are served from it.  The order of the fragments inside the staging
 * buffers is not defined (see NTS_ORDER_BY_DST); only the destination pool is
 * an output.  NTS_EALIAS if a source layer range overlaps a destination layer
 * range or the staging area.
 */
int nts_run_migrate(nts_plan *plan, const void *const *src_layer_ptrs,
                    void *const *dst_layer_ptrs, void *staging, void *hip_stream);

/*
 * nts_run_migrate for callers that cannot allocate device memory or pass a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  The two staging buffers live in a static device array of
 * NTS_STATIC_STAGING_BYTES that the library holds on every GPU it runs on from
 * load until the process ends; the call itself allocates nothing and frees
 * nothing on the device.  The plan must have been created with staging_bytes <=
 * NTS_STATIC_STAGING_BYTES / 2 (so that 2 * chunk_bytes fits): NTS_EINVAL with an
 * explanatory message otherwise.  Result, other errors and stream semantics
 * as nts_run_migrate.  All calls on one GPU share the one array, whatever their
 * context or stream, and it keeps the bytes of the last call (nothing in it
 * needs to start at zero): calls that overlap in time on one GPU race on it and
 * must be ordered by the caller (one stream, or events).
 */
int nts_run_migrate_static(nts_plan *plan, const void *const *src_layer_ptrs,
                           void *const *dst_layer_ptrs, void *hip_stream);

/*
 * Several (source, destination) pairs as ONE pipeline.  A TP switch moves KV
 * from every GPU of the old group to every GPU of the new one whose head
 * interval meets its own (Sec. 3.2.2: GPU 1 sends heads to GPU 2, GPU 3 to GPUs
 * 1 and 2, and so on), so a switch is a list of pairs, each with its own plan.
 * The chunks of plans[0], plans[1], ... form one chunk sequence through the two
 * staging buffers: stage g packs chunk g of that sequence and unpacks chunk
 * g-1, so the last unpack of a pair shares a launch with the first pack of the
 * next pair and short pairs do not drain the pipeline.  The result equals
 * nts_run_migrate on each plan in turn.
 *   plans           host array of n plans of one context (zero-token plans are skipped)
 *   src_layer_ptrs  host array of n host arrays of 2L device pointers (plan i's source pool)
 *   dst_layer_ptrs  likewise, plan i's destination pool; several plans may share a pool
 *   staging         device, 16-byte aligned, nts_batch_staging_bytes() bytes: twice the
 *                   largest chunk_bytes among the plans rounded up to a multiple of 16
 * Every plan reads its source pool as it was before the call: NTS_EALIAS if any
 * plan's destination layer range overlaps any plan's source layer range or the
 * staging area.  Destinations of different plans that overlap each other are
 * written in plan order.  NTS_EINVAL for n < 0, null entries or plans of
 * different contexts.  Enqueues only; no allocation on the device.
 */
int nts_run_migrate_batch(int n, nts_plan *const *plans, const void *const *const *src_layer_ptrs,
                          void *const *const *dst_layer_ptrs, void *staging, void *hip_stream);

/* Size in bytes of the staging area nts_run_migrate_batch needs for these plans
 * (host arithmetic only): 2 * (largest chunk_bytes, rounded up to 16).  The
 * rounding keeps the second buffer aligned for plans of every vector width. */
int nts_batch_staging_bytes(int n, nts_plan *const *plans, int64_t *bytes);

/*
 * The same migration as one kernel from pool to pool, never forming the stream:
 * dst[l][c][dslot[j]][dst_head_off+h][x] = src[l][c][sslot[j]][src_head_off+h][x].
 * Within one address space this is what the direct transfer to the new group's
 * GPUs (Sec. 3.2.2) becomes when the destination pool is mapped into the
 * sender; it moves each payload byte once instead of twice.  The order in which
 * tokens are moved is invisible in the result; a plan made with NTS_ORDER_BY_DST
 * (which needs NTS_VALIDATE_UNIQUE_DST: the plan ranks the tokens by counting the
 * bits of the uniqueness bitmap below each destination slot) lets this call walk
 * them in ascending destination-slot order, so that its writes sweep the pool
 * upwards: 10-14 % faster on fully fragmented pools.  nts_run_migrate and its
 * batch and static variants use the same order inside their staging buffers,
 * whose contents are no output (1-2 %); pack, unpack and the chunk calls, whose
 * stream is an output, never look at the flag.  NTS_EALIAS if the pools overlap.
 */
int nts_run_migrate_direct(nts_plan *plan, const void *const *src_layer_ptrs,
                           void *const *dst_layer_ptrs, void *hip_stream);

/*
 * Comparison baseline of the paper's microbenchmark (Sec. 3.2.2, Fig.
 * "KV-Migration Latency Comparison"): one asynchronous device-to-device memcpy
 * per fragmented region, issued by the host.  With merge_runs != 0, tokens that
 * sit in neighbouring slots on both sides and whose fragment is a whole row are
 * copied as one region (the "contiguous per-request layout" case).  The first
 * call on a plan copies the slot lists to the host (synchronises once).
 * *n_copies (may be NULL) receives the number of memcpy calls issued.
 */
int nts_run_memcpy_baseline(nts_plan *plan, const void *const *src_layer_ptrs,
                            void *const *dst_layer_ptrs, int merge_runs, void *hip_stream,
                            int64_t *n_copies);

/* ------------------------------------------------------------------------
 * TP-shard-selecting linear layer (paper Sec. 3.2.1, "Zero-Overhead TP Weight
 * Switching"): each GPU keeps one full copy of a weight matrix W[n_out][n_in]
 * (row-major, 16-bit) and rank `rank` of a group at TP level `tp` computes with
 * its 1/tp of it, selected at execution time; nothing is copied or reloaded
 * when tp changes.
 *   NTS_SPLIT_OUT  Y[M][n_out/tp] = X[M][n_in]    . W[rank*n_out/tp : +n_out/tp, :]^T
 *   NTS_SPLIT_IN   Y[M][n_out]    = X[M][n_in/tp] . W[:, rank*n_in/tp : +n_in/tp]^T
 *                  (a partial sum; the all-reduce over ranks is the caller's)
 * X, W, Y: device, all bfloat16 (NTS_BF16) or all IEEE float16 (NTS_F16);
 * products are accumulated in fp32 and Y is rounded to nearest even once.  ldx / ldw / ldy: row strides in elements, 0 = dense
 * (n_in or n_in/tp for X, n_in for W, the output width for Y); all strides
 * multiples of 8 and below 2^23 elements, all pointers 16-byte aligned.  The shard's reduction length
 * (n_in or n_in/tp) must be a multiple of 64.  workspace: device scratch of at
 * least nts_shard_linear_workspace() bytes (may be NULL when that is 0); it
 * holds fp32 partial sums when the reduction is split over workgroups, which
 * are then added in a fixed order, so results are reproducible.  Y must not
 * overlap X, W or the workspace (not checked).  The call only enqueues work on
 * hip_stream and allocates nothing.
 * Errors: NTS_EINVAL (null pointer, bad split / rank / sizes / alignment,
 * workspace too small), NTS_EHIP.
 */
enum { NTS_SPLIT_OUT = 0, NTS_SPLIT_IN = 1 };
enum { NTS_BF16 = 0, NTS_F16 = 1 };

typedef struct nts_linear_desc {
    int32_t M;      /* rows of X: tokens in the batch, >= 1 */
    int32_t n_out;  /* rows of the FULL weight matrix */
    int32_t n_in;   /* columns of the FULL weight matrix */
    int32_t tp;     /* TP level N */
    int32_t rank;   /* this GPU's rank in its TP group */
    int32_t split;  /* NTS_SPLIT_OUT or NTS_SPLIT_IN */
    int32_t dtype;  /* NTS_BF16 or NTS_F16 */
    int32_t reserved;
    int64_t ldx, ldw, ldy;
} nts_linear_desc;

int nts_shard_linear_workspace(const nts_linear_desc *d, size_t *bytes);

/*
 * Which kernel and launch shape nts_shard_linear uses for a descriptor (host
 * arithmetic only, no GPU needed; the choice depends on M, the shard's size
 * and nothing else).  For callers that log or tune around it and for tests
 * that must reach every kernel variant.  Errors: NTS_EINVAL as above.
 */
typedef struct nts_linear_launch {
    int32_t tiled;       /* 1: matrix-core tiles of tile_rows x tile_cols (256 or 128 rows by 256, 192 or 128 columns, not 128 x 256);
                            0: weight-streaming kernel, or, with tile_rows == 16, the decode kernel */
    int32_t tile_rows;   /* batch rows per workgroup */
    int32_t tile_cols;   /* output columns (weight rows) per workgroup */
    int32_t k_splits;    /* parts the reduction is cut into; > 1 uses the workspace */
    int32_t slabs_ahead; /* 64-wide weight slabs a wavefront keeps in flight */
    int32_t k_waves;     /* wavefronts of a workgroup that share its reduction range (decode kernel), else 1 */
    int32_t reserved[2];
} nts_linear_launch;

int nts_shard_linear_launch(const nts_linear_desc *d, nts_linear_launch *out);

/*
 * The shard of a descriptor as a view into the full weight matrix (host
 * arithmetic only).  A GPU keeps the whole matrix and every TP level works on
 * its part of it in place (Sec. 3.2.1), so a shard is nothing but an element
 * offset, a row count, a column count and the full matrix's row stride:
 *   shard[i][k] = W_full[*elem_offset + i * *row_stride + k],  i < *rows, k < *cols
 * (rows = output features of the shard, cols = its reduction length).  This is
 * what nts_shard_linear computes with; a caller can hand the same view to a GEMM
 * library, which on this GPU is the faster route for prefill batches of a
 * thousand rows and more.  Errors: NTS_EINVAL as for nts_shard_linear_workspace.
 */
int nts_shard_linear_view(const nts_linear_desc *d, int64_t *elem_offset, int64_t *rows, int64_t *cols,
                          int64_t *row_stride);
int nts_shard_linear(nts_ctx *ctx, const nts_linear_desc *d, const void *X, const void *W_full,
                     void *Y, void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Opt-in tuning of nts_shard_linear for one shape.  The default choice of kernel
 * and launch shape comes from a cost estimate fitted on one MI355X and is good to
 * about 10 %; this call instead runs, on the caller's operands, every
 * configuration whose estimate is within 1.4 x of the best (at most eight, the
 * default first; those that need more workspace than given are skipped), times
 * each with HIP events and remembers the fastest in the context; a configuration
 * other than the default has to beat it by 3 %.
 *   W_list, n_weights  host array of device pointers to full weight matrices of
 *        the descriptor's shape: typically the same layer of every transformer
 *        block.  A timed pass runs the layer once on each, back to back (one
 *        untimed launch, then the shortest of five passes).  In service weights
 *        come from HBM every time; when the given matrices' shards together are
 *        smaller than 512 MiB the call allocates a buffer of that size, sweeps
 *        it before every pass and frees it.  More matrices give a measurement
 *        closer to service; one is enough.
 * Later nts_shard_linear calls on this context with the same M, shard shape
 * (rows and reduction length after the TP cut) and element format use the
 * remembered configuration whenever their workspace is large enough for it, and
 * the default otherwise; strides, rank and split axis do not enter the key.
 * Other arguments as nts_shard_linear; on return Y holds the layer's result on
 * W_list[0].  *picked (may be NULL) receives the chosen configuration.  The call
 * synchronises with hip_stream several times: it is meant for set-up, not for a
 * captured or latency-critical path.  Every configuration is held to the same
 * parity bar, so tuning changes speed only.  nts_shard_linear_tuned reports the
 * remembered configuration for a descriptor (NTS_ERANGE when there is none);
 * nts_shard_linear_workspace stays the size the default needs: give
 * nts_shard_linear_tune the largest workspace you are willing to keep (M * rows
 * * 4 bytes per K split, at most 32 splits).
 * Errors: as nts_shard_linear; NTS_ENOMEM when the flush buffer cannot be allocated.
 */
int nts_shard_linear_tune(nts_ctx *ctx, const nts_linear_desc *d, const void *X,
                          const void *const *W_list, int n_weights, void *Y, void *workspace,
                          size_t workspace_bytes, void *hip_stream, nts_linear_launch *picked);
int nts_shard_linear_tuned(const nts_ctx *ctx, const nts_linear_desc *d, nts_linear_launch *out);

/*
 * The pieces nts_shard_linear_tune is made of, for callers that want to time the
 * candidates their own way (inside their graph, on their real activations):
 *   nts_shard_linear_candidates  host arithmetic: the configurations the tuner would
 *       try for this descriptor, out[0] the default, at most max_out (16 at most);
 *   nts_shard_linear_with        nts_shard_linear with exactly the configuration `how`
 *       (workspace: k_splits * M * rows * 4 bytes when k_splits > 1; enqueues only);
 *       NTS_EINVAL when the library has no such kernel instance for this problem;
 *   nts_shard_linear_remember    makes `how` the context's choice for this shape, as
 *       the tuner does with its winner; how == NULL forgets the shape again.
 * Every configuration computes the same layer to the same parity bar.
 */
int nts_shard_linear_candidates(const nts_linear_desc *d, nts_linear_launch *out, int max_out, int *n_out);
int nts_shard_linear_with(nts_ctx *ctx, const nts_linear_desc *d, const nts_linear_launch *how,
                          const void *X, const void *W_full, void *Y, void *workspace,
                          size_t workspace_bytes, void *hip_stream);
int nts_shard_linear_remember(nts_ctx *ctx, const nts_linear_desc *d, const nts_linear_launch *how);

/* ------------------------------------------------------------------------
 * Goodput-efficiency planner (paper Sec. 3.3.1; host only, no GPU needed).
 * For SLO tier k, thp[i] / thd[i] are the profiled maximum prefill / decode
 * request rates (req/s) of ONE instance at TP level {1,2,4,8}[i] under the
 * tier's TTFT / TPOT SLO; 0 marks a level that cannot meet the SLO.  A
 * configuration (tier, prefill TP, decode TP) is scored on a balanced block of
 * P prefill and D decode instances (P*THP ~ D*THD) with the paper's Eq. 1,
 *     GE = min(P*THP, rps) / (P*TPi + D*TPj),
 * and nts_plan_cluster assigns the pool greedily by GE * rps / served_rps.
 * Where the paper is silent: a block is the (P, D) in 1..max_inst with the
 * smallest |P*THP - D*THD| / max (ties: fewer instances, then smaller P) and
 * serves min(P*THP, D*THD); Eq. 1 is evaluated as printed (prefill rate only;
 * thd does not enter nts_goodput_efficiency) with the tier's unmet rate, so with
 * an inexact integer balance a block's score can exceed what it serves; a tier served
 * nothing yet outranks the others; ties: larger GE, then lower tier, prefill
 * TP, decode TP; one block per step until no demand is unmet or nothing fits.
 * out: host array of max_out entries in assignment order; *n_out is the number
 * of steps taken (NTS_ERANGE if it exceeds max_out; the first max_out are
 * valid), *gpus_left the GPUs no block could use.
 */
enum { NTS_TP_LEVELS = 4 };

typedef struct nts_tier {
    double rps;                 /* incoming request rate of the tier in the last window */
    double thp[NTS_TP_LEVELS];  /* prefill req/s of one instance at TP 1, 2, 4, 8 */
    double thd[NTS_TP_LEVELS];  /* decode req/s of one instance at TP 1, 2, 4, 8 */
} nts_tier;

typedef struct nts_alloc {
    int32_t tier, tp_prefill, tp_decode, P, D, gpus;
    double served_rps;          /* goodput this block adds to its tier */
} nts_alloc;

int nts_balanced_block(double thp, double thd, int max_inst, int *P, int *D);
int nts_goodput_efficiency(double thp, int tpi, double thd, int tpj, int P, int D, double rps,
                           double *ge);
int nts_plan_cluster(int n_gpus, int n_tiers, const nts_tier *tiers, int max_inst, nts_alloc *out,
                     int max_out, int *n_out, int *gpus_left);

#ifdef __cplusplus
}
#endif
#endif /* NITSUM_KVMIG_H */
