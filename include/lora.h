/*
 * liblora — batched heterogeneous-adapter LoRA delta for one MI355X (gfx950).
 *
 * Every row of a batch carries its own adapter id and, in MoE layers, its routed expert
 * id, and receives  y[row] += scale[adapter] * (x[row] * A) * B  with the A and B of its
 * (adapter, layer, expert) unit.
 *
 * Conventions that hold for every call:
 *   - returns LORA_OK (0) or a negative lora_status; never throws, never exits;
 *   - "device" pointers are HIP device memory owned by the caller; "host" pointers are
 *     ordinary process memory; the library allocates no device memory at all: the pool
 *     lives in a caller-provided slab, intermediates in caller-provided workspaces;
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream); all device
 *     work is enqueued on it and nothing synchronises, so outputs are ready when the
 *     stream reaches that point;
 *   - activations and outputs are row-major; bf16 is passed as 16-bit patterns;
 *   - device pointers to activations, outputs and workspaces must be 16-byte aligned and
 *     leading dimensions (in elements) multiples of 8;
 *   - host-detectable mistakes (NULL, negative sizes, bad rank, misalignment, short
 *     buffers, out-of-range layer/projection) are reported before any device work is
 *     enqueued; data-dependent ones (an id outside the pool) cannot be, so they raise a
 *     bit in the device status word of lora_segments and the row is treated as id -1.
 */
#ifndef LORA_H
#define LORA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum lora_status {
    LORA_OK = 0,
    LORA_ERR_INVALID_ARG = -1,      /* NULL where a pointer is required, negative count, bad enum */
    LORA_ERR_BAD_SHAPE = -2,        /* widths not multiples of 8, ld < width, layer/proj out of range */
    LORA_ERR_UNSUPPORTED_RANK = -3, /* rank not in {8, 16, 32, 64} */
    LORA_ERR_BUFFER_TOO_SMALL = -4, /* slab or workspace smaller than the size query says */
    LORA_ERR_NOT_REGISTERED = -5,   /* pool handle NULL or destroyed, segments not built */
    LORA_ERR_HIP = -6,              /* a HIP runtime call failed; see lora_last_hip_error */
    LORA_ERR_MISALIGNED = -7,       /* pointer not 16-byte (slab: 256-byte) aligned */
    LORA_ERR_TOO_LARGE = -8         /* P or key space beyond what the segment builder handles */
} lora_status;

enum { LORA_DTYPE_BF16 = 0, LORA_DTYPE_F32 = 1 };
enum { LORA_MOE_UPGATE = 0, LORA_MOE_DOWN = 1 };
enum {
    LORA_MAX_PROJ = 8,
    LORA_MAX_ROWS = 1 << 14,        /* rows of a batch that one workgroup sorts (small workspace) */
    LORA_MAX_ROWS_LONG = 1 << 20    /* rows of a batch, any pool */
};

/* where a pool's calls expect the activations (input rows, output rows) when a call starts */
enum {
    LORA_ACT_AUTO = 0,       /* in a cache unless a call's rows are too many to be (default) */
    LORA_ACT_RESIDENT = 1,   /* always in a cache: no streaming hints on activations */
    LORA_ACT_STREAMING = 2   /* in HBM only: activations are read and written with streaming hints */
};

/* bits of the device status word written by lora_build_segments */
enum { LORA_STATUS_BAD_ADAPTER = 1u, LORA_STATUS_BAD_EXPERT = 2u };

const char *lora_strerror(int status);
/* Text of the last HIP error seen by this thread's calls ("" if none). */
const char *lora_last_hip_error(void);

/* ------------------------------------------------------------------------------------
 * Adapter pool and pointer table.
 *
 * Sec. 4.1 abstracts the adapters as an n x l x e tensor of units, one unit holding the
 * LoRA matrices of one expert at one layer of one adapter; Sec. 4.2 keeps a working set
 * of adapters resident in GPU memory.  Here a unit carries, for each of n_proj
 * projections, A (h_in x rank) and B (rank x h_out) in bf16 (Sec. 2.2), and the pool is
 * the resident set: one slab in HBM plus a device table with one entry per
 * (layer, adapter, expert, projection) giving the addresses of that unit's A and B, its
 * rank and its adapter's scale.
 *
 * The slab stores A and B re-tiled for the kernels (see lora_pool_unit_layout); callers
 * hand over plain row-major matrices and the library repacks them on the device.
 * An adapter whose own rank is below the pool rank is zero-padded, which is exact.
 * MoE pools used with lora_moe_apply have n_proj = 3 in the order gate, up, down.
 * ------------------------------------------------------------------------------------ */
typedef struct lora_proj_desc {
    int32_t h_in;   /* input width of the projection, multiple of 8 */
    int32_t h_out;  /* output width, multiple of 8 */
} lora_proj_desc;

typedef struct lora_pool_desc {
    int32_t n_adapters;            /* n >= 1 */
    int32_t n_layers;              /* l >= 1 */
    int32_t n_experts;             /* e >= 1 (1 = dense layer) */
    int32_t n_proj;                /* 1 .. LORA_MAX_PROJ */
    int32_t rank;                  /* pool rank: 8, 16, 32 or 64 */
    int32_t dtype;                 /* LORA_DTYPE_BF16 */
    lora_proj_desc proj[LORA_MAX_PROJ];
    const float *scale;            /* host, [n_adapters]; NULL = 1.0 for all */
    const int32_t *adapter_rank;   /* host, [n_adapters], each 1..rank; NULL = pool rank */
} lora_pool_desc;

typedef struct lora_pool lora_pool; /* opaque host handle */

/* Bytes the slab must have for this description (table + all units), 0 if invalid. */
size_t lora_pool_bytes(const lora_pool_desc *d);

/*
 * Lay the pool out inside `slab` (device, 256-byte aligned, >= lora_pool_bytes) and write
 * the device table.  A_src / B_src: host arrays of n_adapters*n_layers*n_experts*n_proj
 * device pointers in the order [adapter][layer][expert][proj], each to a row-major bf16
 * A[h_in][adapter_rank] / B[adapter_rank][h_out]; both NULL = leave every unit zero (load
 * later with lora_pool_load_*).  The slab must stay alive and untouched by the caller until
 * lora_pool_destroy.  On success *out receives the handle.
 */
int lora_register_pool(const lora_pool_desc *d, void *slab, size_t slab_bytes,
                       const void *const *A_src, const void *const *B_src,
                       void *stream, lora_pool **out);

/* Repack one unit's projection from row-major device matrices (bf16). */
int lora_pool_load_unit(lora_pool *pool, int adapter, int layer, int expert, int proj,
                        const void *A, const void *B, void *stream);

/*
 * Repack all experts and projections of one (adapter, layer) from one contiguous device
 * buffer laid out [expert][proj]{ A[h_in][r], B[r][h_out] } with r = that adapter's rank
 * (Sec. 5.3 loads adapters layer by layer; this is the unit of such a load).
 */
int lora_pool_load_adapter_layer(lora_pool *pool, int adapter, int layer, const void *src,
                                 void *stream);

/*
 * Layer-wise loading of a whole adapter into its slot of the pool (Sec. 5.3: transfer and
 * computation are pipelined at layer granularity, so the first layer can compute as soon
 * as its weights have arrived while later layers are still on their way).
 *
 * lora_pool_adapter_layer_bytes: bytes of one (adapter, layer) source window, laid out as
 *   lora_pool_load_adapter_layer expects it; 0 on a bad argument.
 * lora_pool_load_adapter_async: host_src = pinned host memory holding the n_layers windows
 *   of the adapter back to back, layer 0 first.  For every layer in order, on load_stream:
 *   copy the window to `staging` (device, 16-byte aligned, at least one window), repack it
 *   into the pool, record the layer's ready event.  Returns after enqueueing; host_src and
 *   staging must stay untouched until the last layer is ready.  The source windows are read
 *   with the slot's current rank and the slot keeps its current scale: when the incoming
 *   adapter differs in either, call lora_pool_set_adapter on load_stream first.  Work that
 *   was launched earlier may still be reading the slot's old contents; ordering the load
 *   behind that work is the caller's job (make load_stream wait for it first).
 * lora_pool_wait_layer: make `stream` wait (on the device, without blocking the host) until
 *   the latest load of (adapter, layer) enqueued before this call has landed; a no-op for a
 *   layer that was never loaded asynchronously.
 * lora_pool_layer_ready: 1 if that load has completed (or none was ever enqueued), 0 if it
 *   is still in flight, a negative lora_status on error.  Never blocks.
 * These four calls and lora_pool_destroy on one pool must not race with each other.
 */
size_t lora_pool_adapter_layer_bytes(const lora_pool *pool, int adapter);

/*
 * Give a slot of the pool another rank (1 .. pool rank) and scale, as when the cache of
 * Sec. 4.2 replaces one resident adapter by another: rewrites the scale and rank of the slot's
 * table entries of every layer on `stream` (a small kernel, ordered like any other work on that
 * stream) and makes later loads into the slot read their source with the new rank.  The packed
 * matrices themselves are left alone; load the new adapter afterwards (loads zero-pad a rank
 * below the pool rank, which is exact).
 */
int lora_pool_set_adapter(lora_pool *pool, int adapter, int rank, float scale, void *stream);

/*
 * Cache hints for the activations of this pool's compute calls (Sec. 5.2: the kernels are bound
 * by memory traffic, so where the rows come from decides their speed).  The adapter weights are
 * always read with streaming hints (each is read once per call).  Activations, by `policy`:
 *   LORA_ACT_AUTO (default)  input and output rows go through the caches, as suits rows that
 *       the kernel before the call has just written and the kernel after it will read; input
 *       rows that every pair reads for itself (no src_row / token_of_pair gather) are streamed
 *       once they reach 64 MiB per call, output rows once a call's outputs reach 256 MiB (the
 *       memory-side cache holds 256 MiB).
 *   LORA_ACT_RESIDENT        no streaming hint on any activation, whatever its size.
 *   LORA_ACT_STREAMING       for callers whose activations are in HBM only when a call starts
 *       (arrived over a link, or written long ago): output rows are read and written with
 *       streaming hints at every size, and so are input rows that every pair reads for itself.
 * Results are bit-identical under all three; only the decode kernels (tiles of at most 16 rows)
 * look at the policy, the long-segment kernels always stream their outputs.  Host state only:
 * takes effect from the next call on, must not race with calls on the same pool.  Errors:
 * LORA_ERR_NOT_REGISTERED, LORA_ERR_INVALID_ARG (unknown policy).
 */
int lora_pool_set_activation_policy(lora_pool *pool, int policy);
int lora_pool_activation_policy(const lora_pool *pool);   /* the current policy, negative on error */
int lora_pool_load_adapter_async(lora_pool *pool, int adapter, const void *host_src,
                                 void *staging, size_t staging_bytes, void *load_stream);
int lora_pool_wait_layer(const lora_pool *pool, int adapter, int layer, void *stream);
int lora_pool_layer_ready(const lora_pool *pool, int adapter, int layer);

/* Inverse of the repacking: write one unit's projection back as row-major bf16
 * A[h_in][rank] and B[rank][h_out] (pool rank, zero padding included). */
int lora_pool_read_unit(const lora_pool *pool, int adapter, int layer, int expert, int proj,
                        void *A_out, void *B_out, void *stream);

/* Host view of one table entry: byte offsets of the packed A and B inside the slab,
 * their sizes, the unit's rank and scale. Any out pointer may be NULL. */
int lora_pool_unit_layout(const lora_pool *pool, int adapter, int layer, int expert, int proj,
                          size_t *A_offset, size_t *A_bytes, size_t *B_offset, size_t *B_bytes,
                          int32_t *rank, float *scale);

/* Device address of the table (entries of 32 bytes: A*, B*, float scale, int32 rank, pad),
 * ordered [layer][adapter][expert][proj]. */
const void *lora_pool_device_table(const lora_pool *pool);

int lora_pool_destroy(lora_pool *pool);

/* ------------------------------------------------------------------------------------
 * Segments.
 *
 * App. A.2.2: rows that share an adapter are aggregated into one GEMM so that the
 * adapter's weights are read once; with expert-specific matrices (Sec. 2.3) the rows that
 * share (adapter, expert).  lora_build_segments produces the one canonical grouping:
 *   key = adapter * n_experts + expert;
 *   rows with adapter -1 (no LoRA) or an out-of-range id are left out;
 *   perm[0 .. P_act) lists the remaining row indices by ascending key, original order
 *   kept inside a key (a stable counting sort);
 *   seg_key[s], s < S: key of the s-th non-empty group; seg_start[s] its first position
 *   in perm; seg_start[S] = P_act;
 *   counts = { S, P_act, n_tiles, 0 }.
 * Results are deterministic and bit-identical run to run.  Entries of perm, seg_start,
 * seg_key beyond the stated ranges are unspecified.  tiles (row blocks of at most
 * tile_rows rows that never cross a segment) are what the compute kernels iterate over.
 * ------------------------------------------------------------------------------------ */
typedef struct lora_tile {   /* device record, 16 bytes */
    int32_t key;             /* segment key of the tile */
    int32_t row0;            /* first position in perm */
    int32_t n_rows;          /* 1 .. tile_rows */
    int32_t seg;             /* index of the segment */
} lora_tile;

typedef struct lora_segments {
    int32_t P;               /* host: rows the ids describe; set by lora_build_segments */
    int32_t tile_rows;       /* host: set by lora_build_segments */
    int32_t n_keys;          /* host: n_adapters * n_experts of the pool the segments were built
                                for; set by lora_build_segments.  Every call that takes segments
                                returns LORA_ERR_NOT_REGISTERED for a pool with another key count */
    int32_t reserved;        /* host: set to 0 by lora_build_segments */
    int32_t *perm;           /* device [P] */
    int32_t *seg_start;      /* device [P + 1] */
    int32_t *seg_key;        /* device [P] */
    lora_tile *tiles;        /* device [P] */
    int32_t *counts;         /* device [4] */
    uint32_t *status;        /* device [1]: 0 or LORA_STATUS_* bits of this call */
} lora_segments;

size_t lora_segments_ws_bytes(int P);

/*
 * adapter_id: device int32 [P], -1 = no adapter.  expert_id: device int32 [P] or NULL for a
 * dense layer.  P = 0 is a valid no-op that writes counts = 0.  P <= LORA_MAX_ROWS_LONG, beyond
 * that LORA_ERR_TOO_LARGE.
 * `seg`: the caller fills the six device pointers; the call fills P, tile_rows and n_keys.
 * ws: device scratch of lora_segments_ws_bytes(P).  Batches of up to LORA_MAX_ROWS rows are
 * sorted in LDS by one workgroup; longer ones, and long ones of at most 256 keys
 * (n_adapters * n_experts), by several workgroups, which keep per-chunk counts and (beyond
 * LORA_MAX_ROWS rows) the rows' keys and two intermediate orders there: 12 bytes per row.
 */
/* Kernel launches lora_build_segments enqueues for a batch of P rows on this pool: 1 (one
 * workgroup), 2 (several workgroups, at most 256 keys) or 2 per 8 key bits + 2 (several
 * workgroups, larger key spaces); negative on a bad argument.  A host-side query; it enqueues
 * nothing. */
int lora_segments_launches(const lora_pool *pool, int P);

int lora_build_segments(const lora_pool *pool, const int32_t *adapter_id,
                        const int32_t *expert_id, int P, lora_segments *seg,
                        void *ws, size_t ws_bytes, void *stream);

/* ------------------------------------------------------------------------------------
 * Shrink and expand (App. A.2.2 names the two phases; Sec. 2.2 defines the product).
 *
 * lora_shrink:  v = gather(x) * A.   Row i of the sorted order reads x row
 *   src_row[perm[i]] (src_row NULL: perm[i]) — Sec. 5.2: activations are scattered and
 *   must be gathered.  x: device bf16, row stride ldx elements.
 *   v: device workspace of lora_v_bytes(pool, proj, P) bytes; it holds per-K-slice fp32
 *   partial sums in sorted-row order (and room that lora_expand uses for itself) and is
 *   meant only to be passed to lora_expand with the same pool, layer, proj and segments.
 * lora_expand:  y[perm[i]] += scale * v_i * B   (Sec. 2.2: the update is added to the base
 *   output; Fig. 7b: final addition of the two outputs).  y: device, row stride ldy
 *   elements, bf16 (read, add in fp32, round to nearest even, write) or fp32.  Rows that
 *   are not in perm are never read or written.  x and y must not overlap.
 * ------------------------------------------------------------------------------------ */
size_t lora_v_bytes(const lora_pool *pool, int proj, int P);

int lora_shrink(const lora_pool *pool, int layer, int proj, const void *x, int64_t ldx,
                const int32_t *src_row, const lora_segments *seg, float *v, void *stream);

/* v is not const in lora_expand: for batches of long segments the call keeps the bf16 operand
 * images of the summed, scaled v in the tail of the same workspace. */
int lora_expand(const lora_pool *pool, int layer, int proj, float *v,
                const lora_segments *seg, void *y, int64_t ldy, int out_dtype, void *stream);

/*
 * lora_apply: the whole delta of one projection, y[row] += scale * (x[row] * A) * B (Sec. 2.2):
 * exactly lora_shrink followed by lora_expand on the workspace v (lora_v_bytes(pool, proj, P)
 * bytes, contents unspecified afterwards), with the arguments of the two.
 */
int lora_apply(const lora_pool *pool, int layer, int proj, const void *x, int64_t ldx,
               const int32_t *src_row, const lora_segments *seg, void *y, int64_t ldy,
               int out_dtype, float *v, void *stream);

/*
 * lora_apply_group: the deltas of n_proj (1 .. 3) consecutive projections proj0 .. proj0+n_proj-1
 * that read the same input x (equal h_in; their h_out may differ): the query/key/value
 * projections of an attention block, or gate and up (Sec. 2.3 lists the per-expert matrices
 * that share the expert's input).  Results are bit-identical to n_proj lora_apply calls; x is
 * read once per row tile for all of them and each phase is one launch for the group when the
 * batch is a decode batch.  y[j], ldy[j]: output and row stride of projection proj0 + j (host
 * arrays of n_proj entries).  ws: device scratch of lora_group_ws_bytes(pool, proj0, n_proj, P).
 */
size_t lora_group_ws_bytes(const lora_pool *pool, int proj0, int n_proj, int P);

/* How many kernel launches lora_apply_group (lora_apply: n_proj = 1; lora_moe_apply: up/gate is
 * proj0 = 0, n_proj = 2, down is proj0 = 2, n_proj = 1) enqueues for these segments: 1 when shrink
 * and expand run as one launch (small decode batches with short inputs), else 2 or more; 0 for an empty
 * batch; a negative lora_status on a bad argument.  A host-side query for schedulers and
 * benchmarks; it enqueues nothing. */
int lora_group_launches(const lora_pool *pool, int proj0, int n_proj, int out_dtype,
                        const lora_segments *seg);

int lora_apply_group(const lora_pool *pool, int layer, int proj0, int n_proj, const void *x,
                     int64_t ldx, const int32_t *src_row, const lora_segments *seg,
                     void *const *y, const int64_t *ldy, int out_dtype, void *ws,
                     size_t ws_bytes, void *stream);

/* ------------------------------------------------------------------------------------
 * Segment build and first application of a layer call in one entry point (App. A.2.2: the
 * rows of a batch are aggregated by adapter before shrink and expand; Sec. 5.2: scheduling
 * the LoRA computation with few launches).
 *
 * lora_build_apply_group = lora_build_segments(adapter_id, expert_id, P, seg, seg_ws) followed by
 * lora_apply_group(..., seg, ...), with the same arguments, results (segments and outputs, bit
 * for bit) and errors; lora_moe_build_apply likewise for lora_moe_apply.  For decode batches of
 * at most 2048 rows on pools of at most 256 (adapter, expert) keys the first shrink kernel
 * sorts the batch itself and writes `seg` out for the calls that follow, so the launch of the
 * segment builder, which such a short layer call feels, goes away; otherwise the two are
 * launched one after the other.  `seg` is complete when the call's kernels have run and is
 * then used like any other (the down projection of the same MoE layer, later groups of a
 * dense layer).  A call that returns an error has enqueued nothing.
 * lora_build_apply_launches: kernels such a call enqueues for P rows (host-side query).
 * ------------------------------------------------------------------------------------ */
int lora_build_apply_group(const lora_pool *pool, int layer, int proj0, int n_proj, const void *x,
                           int64_t ldx, const int32_t *src_row, const int32_t *adapter_id,
                           const int32_t *expert_id, int P, lora_segments *seg, void *seg_ws,
                           size_t seg_ws_bytes, void *const *y, const int64_t *ldy, int out_dtype,
                           void *ws, size_t ws_bytes, void *stream);

int lora_build_apply_launches(const lora_pool *pool, int proj0, int n_proj, int out_dtype, int P);

/* ------------------------------------------------------------------------------------
 * MoE application (Sec. 3: the LoRA computation runs twice per MoE layer, for the
 * up/gate and for the down projection; Sec. 4.1: a batch of b requests with top-k routing
 * activates b*k units per layer).  Rows are (token, expert) pairs.
 *
 * LORA_MOE_UPGATE: in = token activations x[T][ld_in] (bf16); pair p reads row
 *   token_of_pair[p]; y0[P][ldy] += delta of projection 0 (gate), y1[P][ldy] += delta of
 *   projection 1 (up).  Both projections share one pass over x.
 * LORA_MOE_DOWN: in = per-pair activations hmid[P][ld_in]; token_of_pair ignored;
 *   y0[P][ldy] += delta of projection 2 (down); y1 ignored.
 * Outputs are bf16, one row per pair (routing weights are applied by the caller after).
 * ws: device scratch of lora_moe_ws_bytes(pool, P).
 * ------------------------------------------------------------------------------------ */
size_t lora_moe_ws_bytes(const lora_pool *pool, int P);

int lora_moe_apply(const lora_pool *pool, int layer, int which, const void *in, int64_t ld_in,
                   const int32_t *token_of_pair, const lora_segments *seg,
                   void *y0, void *y1, int64_t ldy, void *ws, size_t ws_bytes, void *stream);

/* lora_build_segments + lora_moe_apply in one entry point; see lora_build_apply_group. */
int lora_moe_build_apply(const lora_pool *pool, int layer, int which, const void *in,
                         int64_t ld_in, const int32_t *token_of_pair, const int32_t *adapter_id,
                         const int32_t *expert_id, int P, lora_segments *seg, void *seg_ws,
                         size_t seg_ws_bytes, void *y0, void *y1, int64_t ldy, void *ws,
                         size_t ws_bytes, void *stream);

/*
 * lora_moe_apply for callers that cannot allocate device memory and have no workspace to hand
 * over: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments, checks, kernels and results as lora_moe_apply, but the intermediate lives in
 * a device array of LORA_STATIC_WS_BYTES that is part of the library's code object (every GPU
 * the library runs on holds its own copy until the process ends).  The call allocates nothing.
 *   - LORA_ERR_TOO_LARGE if lora_moe_ws_bytes(pool, seg->P) exceeds LORA_STATIC_WS_BYTES;
 *     nothing is enqueued then.
 *   - All calls on one GPU share the one array: two calls whose device work can overlap (two
 *     streams, two threads) race; keep them on one stream or order them with events.  The array
 *     keeps the previous call's contents; nothing in it needs clearing, because the shrink
 *     writes every value the expand reads.
 *   - The array's device address is looked up once per device, in lora_register_pool (or in the
 *     first call here on a device that registered no pool); that lookup is a runtime query, so
 *     let it happen before a graph capture starts.
 */
enum { LORA_STATIC_WS_BYTES = 16 << 20 };

int lora_moe_apply_static(const lora_pool *pool, int layer, int which, const void *in, int64_t ld_in,
                          const int32_t *token_of_pair, const lora_segments *seg,
                          void *y0, void *y1, int64_t ldy, void *stream);

/*
 * The two phases of lora_moe_apply as separate calls (App. A.2.2 reports shrink and expand
 * separately): lora_moe_shrink leaves the intermediate in ws, lora_moe_expand consumes it.
 * lora_moe_apply(...) is exactly lora_moe_shrink(...) followed by lora_moe_expand(...) with
 * the same pool, layer, which, segments and ws.
 */
int lora_moe_shrink(const lora_pool *pool, int layer, int which, const void *in, int64_t ld_in,
                    const int32_t *token_of_pair, const lora_segments *seg,
                    void *ws, size_t ws_bytes, void *stream);

int lora_moe_expand(const lora_pool *pool, int layer, int which, const lora_segments *seg,
                    void *y0, void *y1, int64_t ldy, void *ws, size_t ws_bytes, void *stream);

/* ------------------------------------------------------------------------------------
 * Down projection with the routing-weighted combine into token rows.
 *
 * Sec. 4.1: a token activates its top-k experts, so rows are pairs p = t * top_k + j;
 * Sec. 3 / Fig. 7b: the update is added to the base output.  A MoE layer's base output of a
 * token is the routing-weighted sum of its experts' outputs, so the token row gains
 *   y_tok[t] += sum over j = 0 .. top_k-1 (ascending) of route_w[t*top_k + j] * delta[t*top_k + j]
 * with delta the update of the down projection (projection 2) of pair p, over the pairs that
 * have a valid adapter and expert; a token without such a pair is never read or written.  (The
 * paper does not spell the routing weights out; with top_k = 1 and route_w = 1 this is
 * lora_moe_apply(LORA_MOE_DOWN) on token rows.)
 *
 * hmid: device bf16 [P][ld_in] per-pair inputs.  adapter_id, expert_id: the device arrays the
 * segments were built from.  route_w: device fp32 [P].  y_tok: device bf16 [P / top_k][ldy],
 * updated in place: one fp32 sum in the fixed order above, added to the row in fp32, rounded
 * to nearest even once; results are bit-identical run to run.  The per-pair updates pass
 * through bf16 rows inside ws.  ws: device scratch of lora_moe_combine_ws_bytes(pool, P).
 * seg->P must be a multiple of top_k (1 .. 16).
 * ------------------------------------------------------------------------------------ */
size_t lora_moe_combine_ws_bytes(const lora_pool *pool, int P);

int lora_moe_down_combine(const lora_pool *pool, int layer, const void *hmid, int64_t ld_in,
                          const int32_t *adapter_id, const int32_t *expert_id,
                          const lora_segments *seg, const float *route_w, int top_k,
                          void *y_tok, int64_t ldy, void *ws, size_t ws_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* LORA_H */
