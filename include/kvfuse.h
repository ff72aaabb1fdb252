/*
 * kvfuse.h -- C ABI of the MI355X (gfx950) Fast Fusion library.
 *
 * Fast Fusion ("Joint Encoding of KV-Cache Blocks for Scalable LLM Serving", method section and
 * Algorithm 1) fuses similar paged KV-cache blocks of different requests (BFF) or of different chunks of
 * one request (CFF) into one shared unit-direction block, keeps a norm per logical block, and rewrites the
 * block table so that several logical blocks point at one physical block.  This library is the
 * data-parallel hot path of that method for ONE GPU:
 *
 *   a1 block norms -> a2 similarity -> a3 assignment -> a4 merge -> a5 block-table rewrite,
 *   driven level by level over Algorithm 1's binary tree (a6), and a7 paged decode attention that reads
 *   the cache through the fused table.
 *
 * Conventions
 *   - Plain C.  Every call returns an int status (KVFUSE_OK = 0, else an error code below); the text of
 *     the last error of a context is available from kvfuse_last_error().  Nothing throws or aborts.
 *   - "device" pointers are HIP device memory owned by the caller (typically PyTorch tensors); the library
 *     borrows them for the duration of a call and never frees them.  "host" pointers are ordinary host
 *     memory read during the call only.  The library allocates no device memory: scratch comes from the
 *     workspace handed to kvfuse_plan_create / kvfuse_paged_decode_attn, sized by the *_bytes queries.
 *   - All work is enqueued on the context's stream and is asynchronous unless stated otherwise.
 *   - A group g is one (layer, KV head): g = layer * kv_heads + kv_head.  Groups are independent.
 *   - Pool layout: [G][P][t][d] elements, one block (r = t*d elements) contiguous.  dtype bf16 or f32.
 *     r * sizeof(element) must be a multiple of 128 bytes and at most 32 KiB (KVFUSE_ESHAPE otherwise).
 *     The fusion steps never look inside a block, so the paper's own vector -- one per block over all KV heads
 *     of a layer (method section: r = t*h*d, one table per layer) -- is the same call with G = layers,
 *     d := h*d and the pool laid out [layers][P][t][h][d]; kvfuse_paged_decode_attn_all_heads decodes through such a
 *     cache, the other attention entry points need the per-head layout.
 *   - Representation (method section: one unit vector and one scalar norm per block): logical block
 *     x of group g stands for  scale[g][x] * stored(bt[g][x]).  Blocks that were never fused stay as they
 *     were written (scale exactly 1); a fused representative is stored as a unit vector rounded to the
 *     pool dtype, and scale = ||original x|| / ||stored representative||.
 *   - Decisions (which block fuses into which) are taken on cosines evaluated in fp64 on the stored values.
 *     The MFMA similarity kernel is a screen whose error is bounded by `band`; every candidate that the
 *     screen cannot decide (within 2*band of the threshold or of the column maximum) is re-evaluated in
 *     fp64 by kvfuse_assign, so the result does not depend on MFMA rounding.
 */
#ifndef KVFUSE_H
#define KVFUSE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    KVFUSE_OK = 0,
    KVFUSE_EINVAL = 1,    /* bad argument (null pointer, negative size, overlapping leaves, ...) */
    KVFUSE_ESHAPE = 2,    /* unsupported dtype / block size / head size */
    KVFUSE_EOVERFLOW = 3, /* a caller-sized output is too small */
    KVFUSE_ENOMEM = 4,    /* workspace too small */
    KVFUSE_EHIP = 5       /* HIP runtime error; see kvfuse_last_error */
};

enum { KVFUSE_F32 = 0, KVFUSE_BF16 = 1 };

typedef struct kvfuse_ctx kvfuse_ctx;   /* opaque; holds device id, stream, last error; no KV data */
typedef struct kvfuse_plan kvfuse_plan; /* opaque; Algorithm 1's tree cut into heights + workspace layout */

/* The paged KV cache of all groups (method section: cache laid out as blocks of t tokens). */
typedef struct kvfuse_pool {
    void *k;            /* device [G][P][t*d] dtype, keys   (fused rows are overwritten in place) */
    void *v;            /* device [G][P][t*d] dtype, values (same) */
    int32_t dtype;      /* KVFUSE_F32 or KVFUSE_BF16 */
    int32_t G, P, t, d; /* groups, physical blocks per group, tokens per block, head size */
    double *norm_k;     /* device [G][P] out: ||stored block||_2 in fp64 (method section: the norm of every block vector is kept) */
    double *norm_v;     /* device [G][P] out */
    float *inv_norm_k;  /* device [G][P] out: (float)(1/norm_k), 0 for a zero block; similarity epilogue operand */
} kvfuse_pool;

/* Per-group block tables and the per-logical-block rescale. */
typedef struct kvfuse_table {
    int32_t n;           /* logical blocks per group */
    int32_t *bt;         /* device [G][n] in/out: logical -> physical.  Must be injective per group on entry
                            (Algorithm 1 starts from unshared blocks); kvfuse_fuse_tree reports a table that is not */
    float *scale_k;      /* device [G][n] out */
    float *scale_v;      /* device [G][n] out */
    double *orig_norm_k; /* device [G][n] out: norm of the block each logical entry had before fusion */
    double *orig_norm_v; /* device [G][n] out */
    int32_t *refcount;   /* device [G][P] out: logical blocks pointing at each physical block */
    int32_t *remap;      /* device [G][P] out: -1 = live, else the physical block this one was fused into */
} kvfuse_table;

/* Algorithm 1's inputs as index lists (host memory).  A leaf is a run of consecutive logical entries (the
 * full blocks of one request for BFF, of one chunk for CFF); a unit is a run of consecutive leaves (one
 * request).  The recursion splits the unit list at len/2 (left first); a unit with several leaves is first
 * fused over its own leaves the same way.  With one unit this is CFF over its chunks; with one leaf per
 * unit it is BFF.  group_size > 0 applies the method's "every N requests or chunks": consecutive runs of
 * N units (N leaves when there is a single unit) form independent trees; <= 0 means one tree.
 * Leaves must not overlap; the order of the lists is the order of the tree, whatever the logical positions (see
 * kvfuse_tree_spec_shortest_first). */
typedef struct kvfuse_tree_spec {
    int32_t n_leaves;
    const int32_t *leaf_start;    /* host [n_leaves] */
    const int32_t *leaf_count;    /* host [n_leaves] */
    int32_t n_units;
    const int32_t *unit_leaf_ptr; /* host [n_units + 1] */
    int32_t group_size;
} kvfuse_tree_spec;

/* Counters of one kvfuse_fuse_tree run, summed over groups unless noted. */
typedef struct kvfuse_stats {
    int64_t logical_blocks;   /* G * n */
    int64_t physical_blocks;  /* blocks still referenced after fusion */
    int64_t fused;            /* right blocks fused into a left block, all heights */
    int64_t near_threshold;   /* decisions whose best cosine lies within `band` of thr (reported separately) */
    int64_t refined;          /* decisions re-evaluated in fp64 */
    int64_t cand_overflow;    /* columns with more screen candidates than slots (full fp64 rescan) */
    double compression_ratio; /* logical / physical (analysis section, corollary) */
    double sim_flops;         /* sum over nodes of 2 * m_l * m_r * r with the actual set sizes */
    /* stage times in ms from HIP events on the context's stream; filled only when timing was requested */
    float ms_norms, ms_similarity, ms_assign, ms_merge, ms_rewrite, ms_total;
    int32_t n_heights;
    int32_t merge_targets;    /* left blocks rebuilt by kvfuse_merge, all heights (each reads itself and its members, is written once) */
} kvfuse_stats;

/* Device views of one height's intermediate results, for tests and tools.  Column c of a height is right
 * block j = c - r_base[node] of that node; row index i addresses the node's left set. */
typedef struct kvfuse_height_view {
    int32_t n_nodes, total_l_cap, total_r_cap, cand_cap;
    int64_t total_s;           /* sum over nodes of l_cap * r_cap: per-group stride of a dense S buffer */
    const int32_t *l_off, *r_off, *l_slot, *r_slot, *out_slot, *l_cap, *r_cap, *l_base, *r_base; /* device [n_nodes(+1)] */
    const int64_t *s_base;     /* device [n_nodes + 1] */
    const int32_t *set_ids;    /* device [G][n]: surviving physical ids, node sets at their offsets */
    const int32_t *set_cnt;    /* device [G][n_slots] */
    const int32_t *assign;     /* device [G][r_stride]: target row i or -1 */
    const unsigned long long *best_packed; /* device [G][r_stride]: a diagnostic, filled only by a kvfuse_similarity
                                  call that asked for the dense matrix (0 otherwise): column maximum of the screen, packed as
                                  (ordered cosine bits << 32) | (0xFFFFFFFF - row); ordered bits = ~b if the float's
                                  sign bit is set, else b | 0x80000000; 0 = no left row */
    const int32_t *cand_cnt;   /* device [G][r_stride] */
    int32_t n_slots, r_stride, l_stride, reserved;
} kvfuse_height_view;

/* ---- context ------------------------------------------------------------------------------------- */

/* Create a context bound to HIP device `device` and to `hip_stream` (a hipStream_t; NULL = default stream). */
int kvfuse_create(kvfuse_ctx **ctx, int device, void *hip_stream);
int kvfuse_destroy(kvfuse_ctx *ctx);
/* Text of the last error recorded on this context ("" if none).  Valid until the next failing call. */
const char *kvfuse_last_error(const kvfuse_ctx *ctx);

/* ---- a6: tree schedule (Algorithm 1's recursion, host side) ----------------------------------------- */

/* Bytes of device workspace a plan needs.  cand_cap = screen-candidate slots per right block (>= 1). */
int kvfuse_workspace_bytes(int32_t G, int32_t n, const kvfuse_tree_spec *spec, int32_t cand_cap, size_t *bytes);

/* Build the recursion tree of Algorithm 1, cut it into heights (nodes of equal height are independent and
 * are processed by one batched launch per step), lay the intermediate arrays out in `workspace` (device,
 * 256-byte aligned, kept by the caller until kvfuse_plan_destroy) and upload the node tables.
 * pool / table descriptors are copied; the arrays they point at must stay valid while the plan is used. */
int kvfuse_plan_create(kvfuse_ctx *ctx, const kvfuse_pool *pool, const kvfuse_table *table,
                       const kvfuse_tree_spec *spec, int32_t cand_cap, void *workspace, size_t workspace_bytes,
                       kvfuse_plan **plan);
int kvfuse_plan_destroy(kvfuse_plan *plan);
int kvfuse_plan_heights(const kvfuse_plan *plan, int32_t *n_heights);
int kvfuse_plan_view(const kvfuse_plan *plan, int32_t height, kvfuse_height_view *view);

/* ---- a1: norms, leaf step of Algorithm 1 ("normalize") ---------------------------------------------- */

/* Method section: the norm of every block vector is kept.  Computes norm_k, norm_v, inv_norm_k for all G*P blocks
 * (fp64 accumulation), and initialises the table: orig_norm_* from the block each entry points at,
 * scale = 1, refcount = entries per block, remap = -1. */
int kvfuse_block_norms(kvfuse_ctx *ctx, const kvfuse_pool *pool, const kvfuse_table *table);

/* Leaf sets of the plan: every leaf's surviving set = the physical ids of its logical entries. */
int kvfuse_leaf_sets(kvfuse_ctx *ctx, kvfuse_plan *plan);

/* ---- a2: similarity (Algorithm 1: sim <- k_l k_r^T, keys only) ------------------------------------- */

/* For every node of `height` and every group: cosine of each left block with each right block on the
 * MFMA units (bf16 x bf16 -> fp32, or f32), normalised with inv_norm_k.  Per right block it records the
 * list of rows whose screened cosine exceeds thr - 2*band (at most cand_cap kept; the count is exact) and, when
 * the dense matrix is asked for, the column maximum and its row.  dense_s, if not NULL, is device [G][total_s] float and receives
 * every screened cosine: node k's matrix at s_base[k], row-major [l_cap][r_cap], entries beyond the
 * current set sizes untouched.  band must be >= r * 2^-22 (the bound assumed on the screen's error). */
int kvfuse_similarity(kvfuse_ctx *ctx, kvfuse_plan *plan, int32_t height, double thr, double band, float *dense_s);

/* ---- a3: assignment (Algorithm 1: indices where sim > thr, one target per right block) ---------- */

/* Right block j fuses into the left row with the largest cosine, lowest row on exact ties, iff that cosine
 * is > thr (strict); under KVFUSE_RULE_FIRST_ROW (kvfuse_plan_set_assign_rule) into the lowest row whose cosine
 * is > thr.  Cosines that decide are fp64.  Then, per node: members grouped by target (ascending j),
 * evicted blocks entered in table.remap, the surviving set cat(left, non-fused right in order) written in
 * place, and the list of targets to rebuild handed to kvfuse_merge. */
int kvfuse_assign(kvfuse_ctx *ctx, kvfuse_plan *plan, int32_t height, double thr, double band);

/* ---- a4: merge (Algorithm 1: k_l(row) <- normalize(k_l(row) + sum k_r(i)), same for v) --------- */

/* For every target chosen by kvfuse_assign at this height: unit-vector sum of the target and its members
 * (fp64), renormalised, rounded to the pool dtype (nearest even) and written in place at the target's
 * physical block, for K and, with the same members, V; norm_k, norm_v, inv_norm_k of the target are
 * recomputed from the rounded values. */
int kvfuse_merge(kvfuse_ctx *ctx, kvfuse_plan *plan, int32_t height);

/* ---- a5: block-table rewrite (Algorithm 1: evict, update block-table) ---------------------------- */

/* Repoints every logical entry whose physical block was evicted (following table.remap to a live block),
 * recounts references, refreshes scale_k / scale_v of entries that point at a fused representative, and
 * lists the freed physical ids.  free_list: device [G][P] int32 (ascending ids per group), n_free, n_phys:
 * device [G] int32.  Any of the three may be NULL. */
int kvfuse_rewrite_block_table(kvfuse_ctx *ctx, const kvfuse_pool *pool, const kvfuse_table *table,
                               int32_t *free_list, int32_t *n_free, int32_t *n_phys);

/* ---- whole pipeline ---------------------------------------------------------------------------------- */

/* a1 .. a5 over all heights of the plan.  If stats is not NULL the call synchronises the stream at the end
 * and fills it; want_timing additionally brackets the stages with HIP events on the stream.  With stats the call
 * also reports caller errors found on the device: ids outside [0, P), a table that shares blocks on entry
 * (fused before, or a prefix cache), and key blocks whose norm is not finite or, unless zero, outside [2^-40, 2^40]
 * (the similarity screen multiplies stored values in binary32; products of such blocks leave its range and a pair
 * above the threshold could be missed) -- KVFUSE_EINVAL, the pool and table are then undefined. */
int kvfuse_fuse_tree(kvfuse_ctx *ctx, kvfuse_plan *plan, double thr, double band, int32_t *free_list,
                     int32_t *n_free, int32_t *n_phys, kvfuse_stats *stats, int32_t want_timing);

/* The counters of the last tree run on this plan, group by group (the results section reports that layers fuse very
 * different numbers of blocks; kvfuse_stats holds the sums).  out: host [G][4] int32: right blocks fused, decisions within
 * `band` of thr, decisions re-evaluated in fp64, columns whose candidate list overflowed.  Waits for the context's
 * stream.  n_groups must be the plan's G. */
int kvfuse_plan_group_counters(kvfuse_ctx *ctx, const kvfuse_plan *plan, int32_t *out, int32_t n_groups);

/* ---- a7: paged decode attention through the (fused) table -------------------------------------------- */

/* Workspace bytes for a decode call over n_layers layers, B requests, Hq query heads, kv_heads KV heads. */
int kvfuse_decode_workspace_bytes(int32_t n_layers, int32_t B, int32_t Hq, int32_t kv_heads, int32_t d,
                                  int32_t max_blocks, size_t *bytes);

/* One decode step of softmax attention (analysis section: logits q.k/sqrt(d)) for layers
 * [layer_begin, layer_begin + n_layers): request b, query head h reads KV head h / (Hq / kv_heads) of the
 * layer's groups through table.bt, each logical block rescaled by scale_k / scale_v.
 *   q        device [n_layers][B][Hq][d] pool dtype
 *   req_start device [B] int32: first logical entry of request b;  ctx_len device [B] int32 tokens
 *   max_blocks = max over b of ceil(ctx_len[b] / t) (host value, sizes the launch)
 *   out      device [n_layers][B][Hq][d] float
 * Supported: t a multiple of 16, d in {64, 128}, Hq / kv_heads <= 16.  A request with ctx_len 0 gets zeros;
 * B == 0 or n_layers == 0 returns at once. */
int kvfuse_paged_decode_attn(kvfuse_ctx *ctx, const kvfuse_pool *pool, const kvfuse_table *table, int32_t kv_heads,
                             int32_t layer_begin, int32_t n_layers, const void *q, const int32_t *req_start,
                             const int32_t *ctx_len, int32_t B, int32_t Hq, int32_t max_blocks, float sm_scale,
                             void *workspace, size_t workspace_bytes, float *out);

/* The same decode step over the paper's own block vector (method section: r = t * h * d, one vector per block over
 * all KV heads of a layer, one block table per layer).  The pool is laid out [layers][P][t][kv_heads][head size]
 * (pool.G = layers, pool.d = kv_heads * head size), the table and the scales are [layers][n]: every KV head of a layer
 * reads its head-size slice of the token rows of the same blocks, through the same table entry and the same pair of
 * scales.  q, out, req_start, ctx_len, the workspace (kvfuse_decode_workspace_bytes with d = head size) and the limits
 * are those of kvfuse_paged_decode_attn; head size in {64, 128}. */
int kvfuse_paged_decode_attn_all_heads(kvfuse_ctx *ctx, const kvfuse_pool *pool, const kvfuse_table *table, int32_t kv_heads,
                                       int32_t layer_begin, int32_t n_layers, const void *q, const int32_t *req_start,
                                       const int32_t *ctx_len, int32_t B, int32_t Hq, int32_t max_blocks, float sm_scale,
                                       void *workspace, size_t workspace_bytes, float *out);

/* The same decode step for callers that cannot allocate device memory or provide a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid allocation).  The split-KV partial states live in a static
 * device array of KVFUSE_DECODE_STATIC_SCRATCH_BYTES inside the library (one copy per GPU, held until the process
 * ends) instead of a workspace; the call allocates nothing and is otherwise kvfuse_paged_decode_attn, with the same
 * arguments, limits and results.  A call whose partial states would not fit (kvfuse_decode_workspace_bytes greater
 * than the constant) fails with KVFUSE_ENOMEM and a message that names both sizes.  All calls on one GPU share the
 * array: two such calls that overlap in time on one GPU (different streams or threads) race; calls that follow each
 * other on one stream do not, and nothing needs clearing between them. */
#define KVFUSE_DECODE_STATIC_SCRATCH_BYTES (8u << 20)
int kvfuse_paged_decode_attn_static(kvfuse_ctx *ctx, const kvfuse_pool *pool, const kvfuse_table *table, int32_t kv_heads,
                                    int32_t layer_begin, int32_t n_layers, const void *q, const int32_t *req_start,
                                    const int32_t *ctx_len, int32_t B, int32_t Hq, int32_t max_blocks, float sm_scale,
                                    float *out);

/* ---- shared-block decode attention -------------------------------------------------------------------- */

/* The same attention as kvfuse_paged_decode_attn, organised around the blocks that fusion made common
 * (motivation section: a fused representation allows one matrix-matrix product where there were several
 * matrix-vector products; Algorithm 1 marks shared blocks for that purpose; the result for a request is the
 * merge of the attention over its fused part and over its unique part, rescaled).
 *
 * A decode plan is built on the host from the current block table: within each group, physical blocks that are
 * referenced by exactly the same set of requests form a cluster; a cluster of at least min_cluster_blocks blocks
 * is walked once per tile of up to 16 / (Hq / kv_heads) sharing requests, whose query heads fill the rows of one
 * MFMA tile, so its K and V blocks are read once per tile instead of once per request.  What is left of every
 * request (unshared blocks, small clusters, the partial last block) is walked per request as before.  Partial
 * softmax states (maximum, sum, weighted values) of all pieces of a request are merged at the end.  Where a
 * request's blocks sit in its context does not matter, so clusters need not be prefixes or aligned.
 *
 * The plan depends on the table contents: rebuild it after every fusion or table edit.  Building copies the
 * table of the covered groups to the host and synchronises the stream (milliseconds to a fraction of a second,
 * a few times per fusion, never per decode step). */
typedef struct kvfuse_decode_plan kvfuse_decode_plan;

typedef struct kvfuse_decode_plan_info {
    int64_t device_bytes;      /* workspace the plan needs on the device (tables + partial states) */
    int64_t clusters;          /* clusters used, all groups */
    int64_t shared_instances;  /* logical blocks served through clusters */
    int64_t logical_blocks;    /* logical blocks in the contexts, all groups */
    int64_t cluster_block_reads; /* K+V block reads of the cluster pass (blocks x request tiles) */
    int64_t residual_block_reads; /* block reads of the per-request pass */
    int64_t items_cluster, items_residual;
} kvfuse_decode_plan_info;

/* Step 1 (host only plus one device-to-host copy): analyse the table.  req_start, ctx_len: HOST arrays [B].
 * min_cluster_blocks >= 1 (4 is a sensible value).  On success *plan is a host object to be finished by
 * kvfuse_shared_decode_plan_upload and released with kvfuse_shared_decode_plan_destroy. */
int kvfuse_shared_decode_plan_build(kvfuse_ctx *ctx, const kvfuse_pool *pool, const kvfuse_table *table, int32_t kv_heads,
                                    int32_t layer_begin, int32_t n_layers, const int32_t *req_start, const int32_t *ctx_len,
                                    int32_t B, int32_t Hq, int32_t min_cluster_blocks, kvfuse_decode_plan **plan,
                                    kvfuse_decode_plan_info *info);

/* Step 2: place the plan's tables in workspace (device, >= info.device_bytes, owned by the caller, must stay
 * alive and untouched while the plan is used).  Synchronises the stream. */
int kvfuse_shared_decode_plan_upload(kvfuse_ctx *ctx, kvfuse_decode_plan *plan, void *workspace, size_t workspace_bytes);

int kvfuse_shared_decode_plan_destroy(kvfuse_decode_plan *plan);

/* One decode step through an uploaded plan; q and out as in kvfuse_paged_decode_attn, for the plan's layers,
 * requests and context lengths.  Asynchronous on the context's stream. */
int kvfuse_paged_decode_attn_shared(kvfuse_ctx *ctx, const kvfuse_pool *pool, const kvfuse_table *table,
                                    const kvfuse_decode_plan *plan, const void *q, float sm_scale, float *out);

/* ---- chunked-prefill attention with reuse on fused blocks ----------------------------------------------- */

/* Causal softmax attention of a run of query tokens of ONE request over its paged, fused context (motivation
 * section: with chunked prefill, a softmax-attention computation that involves a fused block is reused for the
 * later instances of that block; the result merges the fused part and the unique part with rescaling).
 * The queries are the tokens [q_begin, q_end) of the chunk that starts at token chunk_begin (a multiple of t);
 * the query at position pos sees tokens 0 .. pos.  Logical blocks that end before the chunk and point at the same
 * stored block share one Q K^T product and one product with V; only the exponentials are per instance.  The blocks
 * of the chunk itself are walked one by one with the causal mask.  reuse = 0 builds the same plan without merging
 * instances (every logical block its own entry): the baseline the reuse is measured against; both give the
 * same result up to summation order.  bfloat16 pools, d in {64, 128}, t a multiple of 16, Hq / kv_heads <= 16.
 * The plan reads the table (ids and scales of the blocks before the chunk) once, on the host: rebuild it when the
 * table changes.  Tokens at and after q_end are never read as visible; tokens of the last block beyond q_end may
 * hold anything. */
typedef struct kvfuse_prefill_plan kvfuse_prefill_plan;

typedef struct kvfuse_prefill_plan_info {
    int64_t device_bytes;                 /* workspace the plan needs on the device */
    int64_t logical_blocks_before_chunk;  /* over all groups of the plan */
    int64_t stored_blocks_before_chunk;   /* distinct stored blocks among them (= logical if reuse is off) */
} kvfuse_prefill_plan_info;

int kvfuse_prefill_plan_build(kvfuse_ctx *ctx, const kvfuse_pool *pool, const kvfuse_table *table, int32_t kv_heads,
                              int32_t layer_begin, int32_t n_layers, int32_t req_start, int32_t chunk_begin, int32_t q_begin,
                              int32_t q_end, int32_t Hq, int32_t reuse, kvfuse_prefill_plan **plan,
                              kvfuse_prefill_plan_info *info);
/* workspace: device, >= info.device_bytes, 256-byte aligned, owned by the caller, alive while the plan is used. */
int kvfuse_prefill_plan_upload(kvfuse_ctx *ctx, kvfuse_prefill_plan *plan, void *workspace, size_t workspace_bytes);
int kvfuse_prefill_plan_destroy(kvfuse_prefill_plan *plan);

/* q: device [n_layers][q_end - q_begin][Hq][d] bfloat16;  out: device, same shape, float.  Asynchronous. */
int kvfuse_prefill_attn(kvfuse_ctx *ctx, const kvfuse_pool *pool, const kvfuse_table *table, const kvfuse_prefill_plan *plan,
                        const void *q, float sm_scale, float *out);

/* ---- threshold control ------------------------------------------------------------------------------- */

/* Analysis section: with a layer's block similarities approximately Gaussian (mean mu_l and variance sigma_l^2 =
 * the sample moments of n similarities), the number of similarities above a threshold u is approximately Poisson
 * with rate Lambda_l(u) = n (1 - Phi((u - mu_l) / sigma_l)); the corollary gives the compression ratio over L
 * layers, L m / (L m - sum_l Lambda_l(u)) with m blocks per layer, and the probability that a layer fuses
 * nothing, exp(-Lambda_l(u)), which allows skipping such layers.  Method section, remark on self-adjusting
 * thresholds: feedback on the observed compression. */

/* Cosines of sampled pairs of logical blocks (keys), through the block table, for every group of the pool.
 *   pairs   device [n_pairs][2] int32 logical indices in [0, table.n), the same list for all groups (the caller
 *           draws them; out-of-range indices are clamped)
 *   cos_out device [G][n_pairs] double;  a pair with a zero block gives 0
 * Needs pool.norm_k to be current (kvfuse_block_norms, or a finished fusion).  Asynchronous. */
int kvfuse_pair_cosines(kvfuse_ctx *ctx, const kvfuse_pool *pool, const kvfuse_table *table, const int32_t *pairs,
                        int32_t n_pairs, double *cos_out);

/* Per group, mean and (population) variance of its n_pairs cosines: moments device [G][2] double.  Fixed summation
 * order.  Average the groups of a layer on the host for the per-layer figures of the paper.  Asynchronous. */
int kvfuse_cosine_moments(kvfuse_ctx *ctx, const double *cos_in, int32_t G, int32_t n_pairs, double *moments);

/* Host-only closed forms (no context, no device).  Lambda(u) for n similarities; the u that gives a wanted rate
 * (NaN unless 0 < rate < n and sigma > 0); the corollary (p_no_fusion: host [n_layers] or NULL); one step of
 * target-compression feedback, thr + gain * (observed - target) / target clamped to [lo, hi]: compression above
 * the target raises the threshold.  The paper fixes only that direction (remark on self-adjusting thresholds); the
 * proportional gain law and the clamp are this library's choice, not the paper's. */
double kvfuse_exceedance_rate(double n, double mu, double sigma, double u);
double kvfuse_threshold_for_rate(double n, double mu, double sigma, double rate);
int kvfuse_predict_compression(const double *rates, int32_t n_layers, double blocks_per_layer, double *compression_ratio,
                               double *p_no_fusion);
double kvfuse_threshold_feedback(double thr, double observed_cr, double target_cr, double gain, double lo, double hi);

/* Switch groups off for the following kvfuse_similarity / kvfuse_fuse_tree calls on this plan: enable is a device
 * array [G] of bytes (0 = skip: the group's similarity work items exit at once, its candidate lists stay empty and
 * nothing in it fuses; the other steps run and leave the group as it is), or NULL for all groups.  The array is
 * read during those calls and must stay alive; it is also copied to the host here for the statistics (this call
 * waits for the stream). */
int kvfuse_plan_set_group_mask(kvfuse_ctx *ctx, kvfuse_plan *plan, const uint8_t *enable);

/* ---- prefix screen ------------------------------------------------------------------------------------------ */

/* An exact shortcut for Algorithm 1's product sim <- k_l k_r^T when only the entries above a threshold matter.  With a
 * prefix of p elements, cos(a, b) <= <a[0:p], b[0:p]> / (|a| |b|) + tail(a) * tail(b), where tail(x) = |x[p:]| / |x|
 * (Cauchy-Schwarz on the two tails).  The similarity step then multiplies only the first prefix_elements of every key
 * block and lists a pair as a candidate when this upper bound clears thr - 2 * band; the assignment step evaluates every
 * candidate in full, in fp64, exactly as it does for the undecided candidates of the full-length screen, so targets,
 * tables and fused blocks are the same as without the shortcut.  What changes is the work: on caches whose unrelated
 * blocks spread their energy over the whole block a quarter of the block rejects practically every unrelated pair
 * (tail product about 0.75 against a threshold of 0.9) and the matrix product shrinks fourfold; a prefix that is too
 * short for the data (tail product near or above the threshold) only produces more candidates, up to a full fp64 rescan
 * of the overflowing columns -- slower, never wrong.
 *   prefix_elements  0 switches the shortcut off (the default); otherwise a multiple of 64 bytes worth of elements, at
 *                    least 128 bytes and shorter than a block
 *   tail_share       device [G][P] float, owned by the caller, alive while the plan is used: tail(x) of every key block,
 *                    rounded up; written by kvfuse_leaf_sets / kvfuse_fuse_tree and after every merge
 * Applies to the following kvfuse_leaf_sets, kvfuse_similarity (without a dense matrix), kvfuse_assign, kvfuse_merge
 * and kvfuse_fuse_tree calls on this plan. */
int kvfuse_plan_set_screen_prefix(kvfuse_ctx *ctx, kvfuse_plan *plan, int32_t prefix_elements, float *tail_share);

/* ---- fp8 screen --------------------------------------------------------------------------------------------- */

/* A second exact shortcut for the same product (Algorithm 1, sim <- k_l k_r^T), for the same reason: only entries above
 * the threshold matter, and every one of those is evaluated again in fp64.  Every key block is kept a second time as
 * bytes.  With u = x / |x| the unit block, m a direction of the group (see `centre`; without one alpha = 0 below),
 *     alpha(x) = <m, u> in binary32,  u_c = u - alpha(x) m,  q(x) = e4m3(u_c * 256 / |u_c|),  scale(x) = |u_c| / 256
 * (OCP 8-bit float, 4 exponent and 3 mantissa bits), together with err(x) = | u_c - q(x) scale(x) | (Euclidean norm,
 * fp64, measured on the bytes actually written) plus what the roundings of alpha and of |m| cost, rounded up.  For two
 * blocks
 *     | cos(a, b) - ( <q(a), q(b)> scale(a) scale(b) + alpha(a) alpha(b) ) |  <=  err(a) + err(b) + err(a) * err(b)
 * (the identity <u, v> = <u_c, v_c> + alpha alpha' for a unit m, and Cauchy-Schwarz twice), so the similarity step
 * multiplies the byte copies on the fp8 matrix cores (twice the rate of bfloat16 and half the bytes through LDS and L2)
 * and lists a pair when that value plus this bound clears thr - 2 * band.  The assignment step takes a listed value as
 * the centre of an interval of radius band + bound: a column is settled from the intervals when one row's lower end
 * clears thr + band and every other listed row's upper end (or, under the row-order rule, when no undecided row comes
 * before the first certain one); every other column is evaluated in fp64 on the pool itself, exactly as the undecided
 * columns of the full-length screen are.  Targets, tables and fused blocks are therefore the same as without the
 * shortcut, whatever the data and whatever m; blocks that quantise badly (err is measured, not assumed: typically
 * 0.02 - 0.03) only get wider intervals.
 *   centre  non-zero: before the copies are written, kvfuse_leaf_sets / kvfuse_fuse_tree take as m of each group the
 *           normalised sum of up to 64 of its unit key blocks (even steps through the pool).  Keys of real caches share
 *           a direction (a common offset, a few heavy channels), so that unrelated blocks have cosines of 0.5 and more;
 *           uncentred, err is then too coarse to tell 0.8 from 0.9 and most columns go to the fp64 evaluation.  With the
 *           shared part taken out and carried exactly by alpha, the bytes describe what tells the blocks apart and the
 *           intervals shrink by |u_c| / |u|.  Costs one small kernel per pass and two more sweeps over registers per
 *           block.  Ignored (copies uncentred) while the prefix screen is on and for blocks of more than 8192 elements.
 * Combines with the prefix screen: the product then runs over the first prefix_elements bytes, which must be a multiple
 * of 64 and at least 128 (set the prefix after this call, or switch it off first); the assignment step then first
 * multiplies the whole copies of the listed pairs to get such intervals back.
 *   k8       device, G * P * t * d bytes, block b of group g at (g * P + b) * t * d; owned by the caller, alive while the
 *            plan is used; written by kvfuse_leaf_sets / kvfuse_fuse_tree (all key blocks) and after every merge (the
 *            rebuilt targets)
 *   k8_side  device, 3 * G * P + G * t * d floats, owned by the caller likewise: [G][P] err, then [G][P] scale, then
 *            [G][P] alpha, written along with k8, then [G][t * d] the directions m (unused without `centre`)
 *   k8_bytes, k8_side_floats   what the caller allocated; smaller than stated above -> KVFUSE_EINVAL, nothing changes
 * Two NULLs switch the shortcut off (the default).  Blocks must have a multiple of 64 and at least 128 elements.
 * Applies to the following kvfuse_leaf_sets, kvfuse_similarity, kvfuse_assign, kvfuse_merge and kvfuse_fuse_tree calls
 * on this plan; with a dense matrix kvfuse_similarity then writes the value above instead of the cosine. */
int kvfuse_plan_set_screen_fp8(kvfuse_ctx *ctx, kvfuse_plan *plan, void *k8, size_t k8_bytes, float *k8_side, size_t k8_side_floats,
                               int32_t centre);

/* ---- variants of the method ---------------------------------------------------------------------------- */

/* Algorithm 1 loops over the rows of sim, collects for each row the right blocks above the threshold and evicts
 * them.  A right block that clears the threshold for several rows can go to one of them only.
 * KVFUSE_RULE_ARGMAX (the default) gives it to the most similar row; KVFUSE_RULE_FIRST_ROW follows the loop
 * literally: the block is gone once the first such row has taken it, so the lowest row with cosine > thr wins.
 * Applies to the following kvfuse_assign / kvfuse_fuse_tree calls on this plan.  Under FIRST_ROW the
 * near_threshold statistic counts columns whose deciding cosine (the taker's; the column maximum when no row
 * takes the block) lies within band of thr. */
enum { KVFUSE_RULE_ARGMAX = 0, KVFUSE_RULE_FIRST_ROW = 1 };
int kvfuse_plan_set_assign_rule(kvfuse_ctx *ctx, kvfuse_plan *plan, int32_t rule);

/* Method section, remark on the order of requests: requests with fewer blocks are better placed on the left of
 * the tree.  Host only.  Writes the spec's lists reordered so that units come in ascending number of blocks
 * (stable; the leaves of a unit keep their order); with a single unit its leaves are sorted instead.
 *   leaf_start, leaf_count host [n_leaves] out;  unit_leaf_ptr host [n_units + 1] out (may alias the inputs)
 *   order  host [n_units] (or [n_leaves] when n_units == 1) out, may be NULL: position k holds the unit (leaf)
 *          that was at index order[k]
 * The logical layout of the table is untouched: only the tree changes. */
int kvfuse_tree_spec_shortest_first(const kvfuse_tree_spec *spec, int32_t *leaf_start, int32_t *leaf_count,
                                    int32_t *unit_leaf_ptr, int32_t *order);

/* Results section, first evaluation mode (the fused, rescaled cache is copied back into every fused block and no
 * block is freed): every logical entry x gets the block it had before fusion back, orig_bt[x], filled with
 * scale[x] * stored(bt[x]) rounded once to the pool dtype (K with scale_k, V with scale_v), so that an attention
 * kernel that knows nothing of fusion sees what the fused cache stands for.  On return the table is orig_bt again
 * with unit scales, one reference per block, nothing evicted, and the pool's norms are those of the rewritten
 * blocks, exactly as after kvfuse_block_norms on the new contents.
 *   orig_bt  device [G][n] int32: the table as it was before kvfuse_fuse_tree (injective per group; the caller
 *            keeps a copy, the library does not).  Entries with an id outside [0, P) are left alone.
 * Asynchronous. */
int kvfuse_replicate_rescaled(kvfuse_ctx *ctx, const kvfuse_pool *pool, const kvfuse_table *table, const int32_t *orig_bt);

/* Results section, second evaluation mode (blocks are fused and freed, nothing is rescaled): the fused table and
 * the freed blocks stay as they are and every scale_k / scale_v becomes 1, so each logical block reads its shared
 * representative as stored.  Asynchronous. */
int kvfuse_drop_rescale(kvfuse_ctx *ctx, const kvfuse_pool *pool, const kvfuse_table *table);

#ifdef __cplusplus
}
#endif
#endif /* KVFUSE_H */
