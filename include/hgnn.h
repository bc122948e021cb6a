/*
 * hgnn.h -- C ABI of the MI355X (gfx950) mini-batch HGNN layer library.
 *
 * The library runs the per-layer compute of mini-batch heterogeneous-GNN training
 * -- the four stages the HiFuse paper (arXiv 2408.08490) lists in Section 2.2:
 * semantic graph build, feature projection, neighbour aggregation, semantic fusion,
 * forward and backward -- over ONE type-first merged feature matrix and ONE merged,
 * relation-segmented CSR, so that every stage is a single kernel launch instead of
 * one short launch per vertex type or relation (Section 4.2, Algorithm 1), with the
 * integer-only semantic graph build done by host threads and uploaded on a side
 * stream (Section 4.3, Algorithm 2 and "Pipelining").
 *
 * Conventions
 *  - T vertex types, R relations (semantic graphs); relation r goes from type
 *    rel_src_type[r] to type rel_dst_type[r].  Limits: T <= 32, R <= 128.
 *  - "device" pointers are HIP device memory owned by the CALLER (the Python binding
 *    uses PyTorch tensors); "host" pointers are ordinary host memory.  The library
 *    owns only what hangs off hgnn_ctx / hgnn_graph.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Compute
 *    entry points only enqueue work; they do not synchronise the stream.
 *  - Feature matrices are row-major.  dtype (hgnn_schema.dtype) is the storage type
 *    of features, weights, activations and feature gradients; all sums accumulate in
 *    fp32; weight and bias gradients are always fp32.
 *  - Every feature width (in_dim[t]) must be a multiple of 16 bytes / sizeof(dtype)
 *    (4 for fp32, 8 for bf16); out_dim may be any positive value.
 *  - Device buffers handed to the layer entry points (x_merged, h_out, saved, scratch,
 *    grad_h, grad_x_merged, feature_cat) must be 16-byte aligned (HGNN_EINVAL otherwise).
 *  - Every function returns HGNN_OK or a negative hgnn_status; hgnn_last_error gives
 *    the text of the calling thread's most recent failure.  On failure no caller
 *    output buffer has been handed to a kernel by that call.
 */
#ifndef HGNN_H
#define HGNN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define HGNN_MAX_TYPES 32
#define HGNN_MAX_RELS 128

typedef struct hgnn_ctx hgnn_ctx;     /* thread pool, pinned staging, side stream, buffer pool   */
typedef struct hgnn_graph hgnn_graph; /* one mini-batch: merged CSR + transpose for every layer  */

typedef enum {
  HGNN_OK = 0,
  HGNN_EINVAL = -1,       /* NULL pointer, bad size, index or edge type out of range            */
  HGNN_ENOMEM = -2,       /* host or device allocation failed                                   */
  HGNN_EHIP = -3,         /* a HIP runtime call failed (text in hgnn_last_error)                */
  HGNN_EOVERFLOW = -4,    /* a row / edge / element count does not fit the int32 index outputs  */
  HGNN_ENOTREADY = -5,    /* graph build failed or was never started                            */
  HGNN_EUNSUPPORTED = -6  /* valid request outside what this build implements                   */
} hgnn_status;

typedef enum { HGNN_F32 = 0, HGNN_BF16 = 1 } hgnn_dtype;
typedef enum { HGNN_AGG_MEAN = 0, HGNN_AGG_ATTN = 1 } hgnn_agg;
typedef enum { HGNN_FUSE_SUM = 0, HGNN_FUSE_SEMATTN = 1 } hgnn_fuse;

typedef struct {
  int32_t num_types, num_rels;
  const int32_t *rel_src_type; /* host [R] */
  const int32_t *rel_dst_type; /* host [R] */
  int32_t heads;               /* 1 for mean aggregation */
  int32_t agg;                 /* hgnn_agg   */
  int32_t fuse;                /* hgnn_fuse  */
  int32_t dtype;               /* hgnn_dtype */
} hgnn_schema;

/* Create a context bound to HIP device `device` (< 0: host-only, for the graph build alone)
 * with `host_threads` builder threads (<= 0: one per online core, at most 16), split evenly
 * over `concurrent_builds` builders that each work on one queued graph at a time (<= 0: a
 * quarter of the threads, at most 4 builders: lowest latency for one build; == host_threads:
 * single-threaded builds, the highest rate when many mini-batches are queued ahead).
 * The schema is copied. */
hgnn_status hgnn_create(hgnn_ctx **out, const hgnn_schema *schema, int device, int host_threads,
                        int concurrent_builds);
void hgnn_destroy(hgnn_ctx *ctx);
/* Message of the calling thread's last failed call; never NULL. */
const char *hgnn_last_error(void);

/* ---- Stage 0: type-first feature layout (Section 4.2 "Reorganizing Features") ------------
 * Gathers the mini-batch's rows out of T device-resident per-type feature stores into one
 * buffer ordered by vertex type first, by position in ids[t] second:
 *     x_merged[elem_off[t] + i*feat_dim[t] + c] = store[t][ids[t][i]*feat_dim[t] + c].
 * One kernel launch for all types.
 *   store    host array [T] of device pointers, store[t] is [num_vertices_t x feat_dim[t]] (dtype)
 *   ids      host array [T] of device pointers to int64 [n_rows[t]] (may be NULL when n_rows[t]==0);
 *            every id must be a valid row of store[t] (not checked on the device)
 *   x_merged device, at least elem_off[T] elements (caller computes the size the same way)
 *   row_off  host out int32 [T+1]: rows before type t;  elem_off host out int64 [T+1]: scalars before type t
 * Errors: EINVAL (NULL, negative count, bad feat_dim), EOVERFLOW (more than 2^31-1 rows). */
hgnn_status hgnn_merge_features(hgnn_ctx *ctx, void *stream, const void *const *store,
                                const int32_t *feat_dim, const int64_t *const *ids,
                                const int64_t *n_rows, void *x_merged, int32_t *row_off,
                                int64_t *elem_off);

/* Index-first baseline of the same stage (what Section 4.2's reorganisation replaces; kept for the ablation): the
 * mini-batch's rows of ALL types in one buffer in an interleaved order, as a framework that keeps features by global
 * vertex index has them.  pos: host array [T] of device int32 arrays, pos[t][i] = row of the interleaved buffer
 * that holds row i of type t (together a permutation of 0 .. sum n_rows - 1; positions outside are clamped into
 * the buffer).  One width for all types (HGNN_EUNSUPPORTED otherwise).  hgnn_merge_features_index_first gathers
 * the store rows into that order; hgnn_select_type_first then copies them into the type-first x_merged the
 * layer calls read -- the per-type selection pass that the type-first merge makes unnecessary -- and returns the
 * same offsets as hgnn_merge_features.  Both enqueue on `stream` and return. */
hgnn_status hgnn_merge_features_index_first(hgnn_ctx *ctx, void *stream, const void *const *store,
                                            const int32_t *feat_dim, const int64_t *const *ids,
                                            const int64_t *n_rows, const int32_t *const *pos,
                                            void *x_interleaved);
hgnn_status hgnn_select_type_first(hgnn_ctx *ctx, void *stream, const void *x_interleaved,
                                   const int32_t *feat_dim, const int32_t *const *pos,
                                   const int64_t *n_rows, void *x_merged, int32_t *row_off,
                                   int64_t *elem_off);

/* ---- Stage 1: semantic graph build on the host (Section 4.3, Algorithm 2) ----------------
 * One mini-batch layer as the sampler hands it over: a COO edge list mixing all relations. */
typedef struct {
  int64_t num_edges;
  const void *edge_index;          /* host [2 x num_edges]: row 0 = local source index within its type,
                                      row 1 = local destination index within its type */
  int32_t index_is_i64;            /* 1: int64 entries, 0: int32 entries */
  const int32_t *edge_type;        /* host [num_edges] relation of each edge, or NULL, then: */
  const int64_t *edge_id;          /* host [num_edges] ids into global_edge_type (Algorithm 2's EdgeID) */
  const int32_t *global_edge_type; /* host [num_global_edges] (Algorithm 2's EdgeType); NULL with edge_id given =
                                      the table registered with hgnn_set_edge_types */
  int64_t num_global_edges;
  const int64_t *n_src;            /* host [T] source-side rows per type (rows of this layer's x_merged) */
  const int64_t *n_dst;            /* host [T] destination rows per type; the destinations of type t are
                                      the FIRST n_dst[t] of its n_src[t] source rows */
  const int32_t *transpose_types;  /* host [T] or NULL (= all 1): 0 = source rows of type t get no transpose
                                      entries (their input gradient will not be asked for; see
                                      hgnn_layer_params.input_grad, which must then be 0 for t as well) */
} hgnn_coo_layer;

/* The same build done by device kernels on `stream` instead of by host threads (the arrangement Section 4.3
 * moves away from; kept as the baseline to measure the host build against): edge-type matching, a stable radix
 * sort by (relation, destination), a second one for the transpose.  Same inputs (host arrays), same index arrays
 * bit for bit, same graph object.  Synchronous: returns when the graph is complete (no hgnn_graph_wait needed);
 * allocates device scratch that the context keeps.  gpu_ms (may be NULL): device time of the build between two
 * events on `stream`, uploads of the inputs included, the copy of the results back to the host views excluded.
 * Errors as for hgnn_build_semantic_csr, except that a bad edge is reported by kind, not by position. */
hgnn_status hgnn_build_semantic_csr_device(hgnn_ctx *ctx, void *stream, int32_t num_layers,
                                           const hgnn_coo_layer *layers, hgnn_graph **out, float *gpu_ms);

/* Registers the graph's global edge-type table (Algorithm 2's EdgeType, one entry per edge of the whole graph):
 * the context keeps a compact copy (one byte per edge), so that later hgnn_coo_layer entries may pass edge_id
 * alone.  The look-up EdgeType[EdgeID] is a random access per sampled edge; the compact table keeps most of it
 * in the host caches (and a table made of a few runs of equal type is searched by its run boundaries
 * instead).  Host array, copied (may be freed afterwards); entries outside [0, num_rels) are an
 * error.  Replaces an earlier table; must not be called while builds are in flight. */
hgnn_status hgnn_set_edge_types(hgnn_ctx *ctx, const int32_t *global_edge_type, int64_t num_global_edges);

/* Starts the build of all `num_layers` layers (execution order) on the context's host threads
 * and returns; the threads select edges by relation (Algorithm 2), sort them stably into one
 * merged CSR per layer plus its transpose, stage the arrays in pinned memory and upload them on
 * the context's side stream.  The input arrays must stay valid and unchanged until
 * hgnn_graph_wait returns (or until the first hgnn_layer_fwd/bwd on the graph returns).
 * Validation errors (edge type outside [0,R), endpoint outside [0,n_src)/[0,n_dst),
 * n_dst[t] > n_src[t], counts >= 2^31) are reported by hgnn_graph_wait / hgnn_layer_* as the
 * status of the build.  Argument errors (NULL, num_layers outside 1..8) are reported here. */
hgnn_status hgnn_build_semantic_csr(hgnn_ctx *ctx, int32_t num_layers, const hgnn_coo_layer *layers,
                                    hgnn_graph **out);
/* Whether later builds (hgnn_build_semantic_csr, hgnn_sample_and_build) produce the two permutations
 * `perm` and `cperm` (default: they do).  The mean-aggregation layers read neither; without them the sorts
 * carry one int per edge instead of two and write half as much, which shortens the build by about a
 * tenth.  With enabled = 0 the host view returns NULL for perm and cperm; every other array is unchanged.
 * Ignored by a context of the attention variant (its backward needs cperm).  Must not be called while
 * builds are in flight. */
hgnn_status hgnn_set_build_permutation(hgnn_ctx *ctx, int32_t enabled);
/* Blocks the calling host thread until the build and the upload have finished; returns the
 * build's status. */
hgnn_status hgnn_graph_wait(hgnn_ctx *ctx, hgnn_graph *g);

/* Host-side view of one layer's index arrays (valid until hgnn_graph_release; waits for the
 * build first).  All arrays int32:
 *   rel_row_off [R+1]   merged row range of relation r: one row per destination vertex of type
 *                       rel_dst_type[r], i.e. merged row = rel_row_off[r] + local destination
 *   rel_edge_off[R+1]   CSR position range of relation r's edges
 *   rowptr [rows+1], colidx [edges]  merged CSR; colidx = row of the source in x_merged
 *                       (= row_off[src type] + local source); inside a row, input order is kept
 *   perm   [edges]      input position of the CSR edge (NULL after hgnn_set_build_permutation(ctx, 0), as is cperm)
 *   cptr [src_rows+1], crow [edges], cperm [edges]  transpose: for every x_merged row the edges
 *                       that read it, ascending CSR position; crow = merged CSR row, cperm = CSR position
 * Any output pointer may be NULL. */
typedef struct {
  int64_t rows, edges, src_rows;
  int64_t transpose_edges; /* entries of crow/cperm (= edges unless transpose_types masks some types) */
  const int32_t *rel_row_off, *rel_edge_off, *rowptr, *colidx, *perm, *cptr, *crow, *cperm;
} hgnn_csr_view;
hgnn_status hgnn_graph_host_view(hgnn_ctx *ctx, hgnn_graph *g, int32_t layer, hgnn_csr_view *view);
/* Returns the graph's buffers to the context's pool.  Work already enqueued that reads the
 * graph must have been ordered before the next build on a stream the caller synchronises, or
 * simply finished. */
void hgnn_graph_release(hgnn_ctx *ctx, hgnn_graph *g);

/* ---- Sampling in the loop (Section 2.3 step 1; Fig. 6: one CPU thread samples the mini-batch
 * and selects its edge indices, the side stream uploads, the compute stream trains) -----------
 * The whole graph, as host arrays that the caller keeps alive and unchanged until
 * hgnn_sampler_destroy.  In-neighbour lists per relation: the sources of destination vertex v of
 * relation r are in_nbr[r][in_indptr[r][v] .. in_indptr[r][v+1]); position p of in_nbr[r] is the
 * edge with global id edge_off[r] + p. */
typedef struct hgnn_sampler hgnn_sampler;
typedef struct {
  const int64_t *num_nodes;        /* [T] vertices per type */
  const int64_t *const *in_indptr; /* [R] -> [num_nodes[rel_dst_type[r]] + 1] */
  const int32_t *const *in_nbr;    /* [R] -> [edge_off[r+1] - edge_off[r]] source vertex ids */
  const int64_t *edge_off;         /* [R+1] */
} hgnn_host_graph;
/* Also registers the graph's edge-type table with the context (as hgnn_set_edge_types would, and like it
 * not while builds are in flight).  A sampler must outlive every graph made from it that is still being
 * built (hgnn_graph_wait has not returned yet). */
hgnn_status hgnn_sampler_create(hgnn_ctx *ctx, const hgnn_host_graph *graph, hgnn_sampler **out);
void hgnn_sampler_destroy(hgnn_ctx *ctx, hgnn_sampler *s);
/* Enqueues ONE task for the context's host threads: layer-wise neighbour sampling of the
 * mini-batch of `targets` (distinct vertices of type target_type; copied), then the index arrays
 * hgnn_build_semantic_csr would make of the sampled lists -- the sampler emits its edges relation
 * by relation with destinations ascending, which IS the merged CSR order, so nothing is looked up
 * or sorted for it; the transpose is built as usual -- then the upload, which also carries the
 * global ids of the first layer's source rows.
 * fanouts[h-1] = neighbours kept per destination vertex and relation in hop h, hop 1 nearest the
 * targets; the block of hop h feeds layer num_layers - h + 1.  transpose_types: NULL, or per
 * layer NULL or [T] as in hgnn_coo_layer.
 * The sample is a pure function of (graph, targets, fanouts, seed):
 *  - a hop's destination vertices are the previous hop's source vertices (hop 1: the targets);
 *    a hop's source list of a type starts with its destination list and grows by each vertex
 *    reached for the first time, in the order reached;
 *  - relations are visited in ascending id, their destination vertices in list order;
 *    destination v (global id) with deg in-neighbours keeps all of them in stored order when
 *    deg <= fanout, else the positions that Floyd's subset algorithm picks: for c = 0..fanout-1,
 *    j = deg - fanout + c, t = floor(mix64(key + c) (j+1) / 2^64), position = j if t was picked before
 *    else t, where key = mix64(mix64(mix64(mix64(seed) ^ hop) ^ r) ^ v) and mix64 is the
 *    SplitMix64 output function; every kept position gives one edge, appended in that order. */
hgnn_status hgnn_sample_and_build(hgnn_ctx *ctx, const hgnn_sampler *s, int32_t target_type,
                                  const int64_t *targets, int64_t num_targets, int32_t num_layers,
                                  const int32_t *fanouts, uint64_t seed,
                                  const int32_t *const *transpose_types, hgnn_graph **out);
/* The sampled mini-batch of a graph made by hgnn_sample_and_build (HGNN_EINVAL for any other).
 * hgnn_graph_ids blocks until the sampling (not the build) has finished: per type the number of
 * first-layer source rows, their global ids on the host and -- valid for device work ordered
 * after hgnn_graph_wait_stream -- on the device (NULL on a host-only context); each output array
 * has T entries and may be NULL.  hgnn_graph_minibatch_view blocks like hgnn_graph_host_view:
 * the layer's row counts and its COO edges as the build consumed them. */
hgnn_status hgnn_graph_ids(hgnn_ctx *ctx, hgnn_graph *g, int64_t *n_rows, const int64_t **host_ids,
                           const int64_t **device_ids);
typedef struct {
  int64_t n_src[HGNN_MAX_TYPES], n_dst[HGNN_MAX_TYPES];
  int64_t num_edges;
  const int64_t *edge_index; /* [2 x num_edges]: local source, local destination */
  const int64_t *edge_id;    /* [num_edges] */
} hgnn_minibatch_view;
hgnn_status hgnn_graph_minibatch_view(hgnn_ctx *ctx, hgnn_graph *g, int32_t layer, hgnn_minibatch_view *view);
/* Makes `stream` wait (on the device; the host does not block once the upload is enqueued) for
 * the graph's upload, so that work enqueued afterwards may read the graph's device arrays --
 * hgnn_layer_fwd/bwd do this themselves; hgnn_merge_features on hgnn_graph_ids' device ids needs it. */
hgnn_status hgnn_graph_wait_stream(hgnn_ctx *ctx, hgnn_graph *g, void *stream);

/* ---- Stages 2-4: projection, aggregation, fusion (Section 2.2; Algorithm 1) ---------------
 * Layer parameters.  All arrays are HOST arrays of DEVICE pointers (dtype elements). */
typedef struct {
  const int32_t *in_dim;       /* host [T] input width per type */
  int32_t out_dim;             /* H */
  int32_t relu;                /* 1: ReLU after fusion + bias */
  const void *const *w_rel;    /* [R] W_r  [in_dim[src(r)] x H]            (mean aggregation) */
  const void *const *w_root;   /* [T] W_0^t [in_dim[t] x H] or NULL entry  (mean aggregation) */
  const void *const *bias;     /* [T] b_t [H] or NULL entry; the array itself may be NULL      */
  const int32_t *input_grad;   /* host [T] or NULL (= all 1): 0 = hgnn_layer_bwd leaves the grad_x_merged rows
                                  of type t unwritten and skips their work (fixed, non-learnable input features) */
  /* attention variant (schema agg = HGNN_AGG_ATTN, fuse = HGNN_FUSE_SEMATTN); unused otherwise */
  const void *const *w_type;   /* [T] W_t [in_dim[t] x H]: per-type projection                              */
  const void *const *a_src;    /* [R] attention vector of the source side      [heads x H/heads]            */
  const void *const *a_dst;    /* [R] attention vector of the destination side [heads x H/heads]            */
  const void *w_sem;           /* semantic attention: W_s [H x 128]                                          */
  const void *b_sem;           /*                     b_s [128]                                              */
  const void *q_sem;           /*                     q   [128]                                              */
} hgnn_layer_params;

/* fp32 gradient buffers mirroring hgnn_layer_params (device, caller-owned, OVERWRITTEN).
 * A NULL entry (or NULL array) skips that gradient. */
typedef struct {
  float *const *dw_rel;  /* [R] */
  float *const *dw_root; /* [T] */
  float *const *dbias;   /* [T] */
  /* attention variant */
  float *const *dw_type; /* [T] */
  float *const *da_src;  /* [R] */
  float *const *da_dst;  /* [R] */
  float *dw_sem, *db_sem, *dq_sem;
} hgnn_layer_grads;

/* Bytes of the two device work areas of one layer on this graph:
 *   saved   written by hgnn_layer_fwd, read by hgnn_layer_bwd (per-relation aggregated features)
 *   scratch temporary for either call (contents undefined afterwards)
 * Both must be 256-byte aligned. */
hgnn_status hgnn_layer_workspace_bytes(hgnn_ctx *ctx, hgnn_graph *g, int32_t layer,
                                       const hgnn_layer_params *p, size_t *saved_bytes,
                                       size_t *scratch_bytes);

/* Forward of one R-GCN style layer (mean aggregation, sum fusion):
 *   h[v] = act( x[v] W_0^{t} + b_t + sum_{r: dst(r)=t} mean_{u in N_r(v)} x[u] W_r ),  t = type(v),
 * an empty neighbourhood contributing zero.  Evaluated as: one relation-segmented gather-mean over
 * the merged CSR (aggregation of the raw features, which commutes with the linear projection),
 * then one grouped GEMM per launch whose K dimension runs over [Z_r1 | Z_r2 | ... | x_dst] so that
 * the semantic fusion is the GEMM's accumulation and bias/activation its epilogue.
 *   x_merged device, type-first [sum_t n_src[t]*in_dim[t]] (layout of hgnn_merge_features)
 *   h_out    device, type-first [sum_t n_dst[t] x H]; type t's block starts at row sum_{t'<t} n_dst[t'].
 *            It is the next layer's x_merged.
 * Waits (on the stream, not the host) for the graph upload; blocks the host only until the host
 * build has been enqueued. */
hgnn_status hgnn_layer_fwd(hgnn_ctx *ctx, void *stream, hgnn_graph *g, int32_t layer,
                           const hgnn_layer_params *p, const void *x_merged, void *h_out,
                           void *saved, size_t saved_bytes, void *scratch, size_t scratch_bytes);

/* hgnn_layer_fwd for callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid allocation) and therefore have no scratch area to pass: the same kernels and the
 * same results, bit for bit, with the forward's work area (transposed weights; in bf16 layers with an activation
 * also the aggregate's low-order plane) in a fixed device array of HGNN_STATIC_SCRATCH_BYTES that the library
 * holds on every GPU it runs on until the process ends.  The call allocates nothing, on the device or the host.
 * Mean-aggregation layers only (HGNN_EUNSUPPORTED otherwise).  A layer that needs more than the fixed array
 * holds is refused with HGNN_EINVAL and a message that states both sizes; nothing is enqueued then.  `saved` is
 * as for hgnn_layer_fwd (size from hgnn_layer_workspace_bytes) and feeds hgnn_layer_bwd unchanged.
 * Every call on a GPU uses that GPU's one array: calls whose device work may overlap (different streams, or
 * several host threads) race; order them on one stream.  The array keeps the last call's contents; each call
 * overwrites every byte it later reads, so nothing needs clearing. */
#define HGNN_STATIC_SCRATCH_BYTES (64u << 20)
hgnn_status hgnn_layer_fwd_static(hgnn_ctx *ctx, void *stream, hgnn_graph *g, int32_t layer,
                                  const hgnn_layer_params *p, const void *x_merged, void *h_out,
                                  void *saved, size_t saved_bytes);

/* The same layer with the aggregation reading its source rows where they live (Section 4.2 merges the semantic
 * graphs' aggregation into one pass over rows picked through index lists; here the list goes all the way back to
 * the per-type feature stores, so that the feature merge of Section 4.1 has to materialise destination rows only):
 * store / ids are the arrays hgnn_merge_features takes (host arrays [T] of device pointers; ids[t] holds the
 * layer's n_src[t] global ids of type t), and x_dst is what hgnn_merge_features writes when it is given
 * n_rows[t] = n_dst[t] -- the first n_dst[t] rows of every type, type-first.  Results are those of hgnn_layer_fwd
 * on the fully merged input, bit for bit.  Mean aggregation with one input width for all types
 * (HGNN_EUNSUPPORTED otherwise); work areas as for hgnn_layer_fwd.  The stores must stay unchanged until the
 * call's device work has finished.  hgnn_layer_bwd_gather is hgnn_layer_bwd for such a layer: its x_dst is that
 * same destination-row buffer; grad_x_merged still covers every source row. */
hgnn_status hgnn_layer_fwd_gather(hgnn_ctx *ctx, void *stream, hgnn_graph *g, int32_t layer,
                                  const hgnn_layer_params *p, const void *const *store,
                                  const int64_t *const *ids, const void *x_dst, void *h_out, void *saved,
                                  size_t saved_bytes, void *scratch, size_t scratch_bytes);
hgnn_status hgnn_layer_bwd_gather(hgnn_ctx *ctx, void *stream, hgnn_graph *g, int32_t layer,
                                  const hgnn_layer_params *p, const void *x_dst, const void *h_out,
                                  const void *saved, const void *grad_h, void *grad_x_merged,
                                  const hgnn_layer_grads *g_out, void *scratch, size_t scratch_bytes);

/* Attention variant (the paper evaluates R-GAT, Section 5.1; semantic fusion, Section 2.2): with a schema
 * created with agg = HGNN_AGG_ATTN and fuse = HGNN_FUSE_SEMATTN, hgnn_layer_fwd / hgnn_layer_bwd evaluate
 *   z_t = x_t W_t                                                     (H = heads * D columns)
 *   e   = LeakyReLU_0.2( a_src[r][k] . z_u^k + a_dst[r][k] . z_v^k )  per relation r, head k, edge u -> v
 *   m_v^r = concat_k sum_u softmax_u(e) z_u^k                         (empty neighbourhood: 0)
 *   w_r = mean_v q . tanh(m_v^r W_s + b_s),  beta = softmax over the relations ending in type(v)
 *   h_v = act( sum_r beta_r m_v^r + b_type(v) )
 * and its gradients.  Everything kept between the stages (z, m, the scores, every gradient between them) is fp32
 * in both storage types: with dtype = HGNN_BF16 the inputs, parameters and incoming gradients are bf16, the
 * projection multiplies them as they are (bf16 MFMA, fp32 result), the small parameters and the incoming gradient
 * are widened (exactly) into the scratch area, h_out is rounded once on the way out, and the projection's backward
 * runs on dZ rounded to bf16 (the gradients of a_src / a_dst are the remainder of a cancellation between a
 * vertex's neighbours, which bf16 intermediates do not carry; the projection's own gradients are plain sums).
 * Requirements: D a multiple of 4 scalars and a power of two times that, H / 4 a power of two <= 64; every
 * in_dim and H a multiple of 16 bytes of dtype; weight pointers 16-byte aligned; the graph built with
 * transpose entries for every type.  hgnn_layer_fwd_naive is not available for this variant. */

/* Backward of the same layer.  grad_h: device [sum_t n_dst[t] x H] (dtype), h_out: the forward's
 * output (needed for the ReLU mask).  Outputs: grad_x_merged (device, layout of x_merged, dtype;
 * NULL skips it) and the fp32 weight/bias gradients in `g_out`.  Gradients of parameters that no
 * edge or row touches are exactly zero. */
hgnn_status hgnn_layer_bwd(hgnn_ctx *ctx, void *stream, hgnn_graph *g, int32_t layer,
                           const hgnn_layer_params *p, const void *x_merged, const void *h_out,
                           const void *saved, const void *grad_h, void *grad_x_merged,
                           const hgnn_layer_grads *g_out, void *scratch, size_t scratch_bytes);

/* Launch-count baseline: the same results as hgnn_layer_fwd / hgnn_layer_bwd, but every stage is
 * launched once per relation / per vertex type (the un-merged structure the paper's Section 3
 * measures).  `launches` (host out, may be NULL) receives the number of kernels enqueued. */
hgnn_status hgnn_layer_fwd_naive(hgnn_ctx *ctx, void *stream, hgnn_graph *g, int32_t layer,
                                 const hgnn_layer_params *p, const void *x_merged, void *h_out,
                                 void *saved, size_t saved_bytes, void *scratch,
                                 size_t scratch_bytes, int32_t *launches);
hgnn_status hgnn_layer_bwd_naive(hgnn_ctx *ctx, void *stream, hgnn_graph *g, int32_t layer,
                                 const hgnn_layer_params *p, const void *x_merged, const void *h_out,
                                 const void *saved, const void *grad_h, void *grad_x_merged,
                                 const hgnn_layer_grads *g_out, void *scratch, size_t scratch_bytes,
                                 int32_t *launches);
/* Materialising baseline: the same layer forward with the aggregation done in the two steps in which
 * Algorithm 1 (Section 4.2) states it -- the source rows of all semantic graphs gathered and concatenated
 * into FeatureCat [num_edges x F] (dtype), then reduced by destination -- instead of the fused gather-mean
 * of hgnn_layer_fwd, which never writes FeatureCat.  Results (h_out, saved) are bit-identical to
 * hgnn_layer_fwd's; hgnn_layer_bwd can follow.  Mean aggregation only, and every vertex type must have
 * the same input width F (else HGNN_EUNSUPPORTED).  feature_cat: device scratch of at least
 * num_edges(layer) * F * sizeof(dtype) bytes, 16-byte aligned (HGNN_EINVAL if smaller); the other
 * arguments as for hgnn_layer_fwd.  `launches` (host out, may be NULL): kernels enqueued. */
hgnn_status hgnn_layer_fwd_two_step(hgnn_ctx *ctx, void *stream, hgnn_graph *g, int32_t layer,
                                    const hgnn_layer_params *p, const void *x_merged, void *h_out,
                                    void *saved, size_t saved_bytes, void *scratch, size_t scratch_bytes,
                                    void *feature_cat, size_t feature_cat_bytes, int32_t *launches);
/* Number of kernels hgnn_layer_fwd / hgnn_layer_bwd enqueue for this layer. */
hgnn_status hgnn_layer_launch_count(hgnn_ctx *ctx, hgnn_graph *g, int32_t layer,
                                    const hgnn_layer_params *p, int32_t *fwd_launches,
                                    int32_t *bwd_launches);

/* ---- Loss of the node-classification configurations (model wrapper, not a paper stage) ----
 * Mean softmax cross-entropy over `rows` rows of `logits` [rows x classes] (dtype) and its gradient
 * w.r.t. the logits (dtype, same shape).  `loss` is a device float, overwritten. */
hgnn_status hgnn_softmax_xent(hgnn_ctx *ctx, void *stream, const void *logits, const int64_t *labels,
                              int64_t rows, int32_t classes, float *loss, void *grad_logits);

/* ---- Parameter update (Section 2.3, step 4; the paper names no optimiser: this library offers
 * Adam, Kingma & Ba 2015, Algorithm 1) -----------------------------------------------------
 * step counts updates from 1.  Per element, in fp32:
 *   m = beta1 m + (1 - beta1) g;  v = beta2 v + (1 - beta2) g^2
 *   theta -= lr (m / (1 - beta1^step)) / (sqrt(v / (1 - beta2^step)) + eps) */
typedef struct {
  float lr, beta1, beta2, eps;
  int64_t step;
} hgnn_adam_params;
/* Updates n tensors in one launch per 48 of them.  Host arrays of device pointers: param[i]
 * (context dtype, numel[i] elements), master[i] (fp32 copy the update is applied to; param[i] is
 * then its rounded copy; the array or an entry may be NULL when the dtype is fp32: the parameter
 * is its own master), grad[i] (fp32, as hgnn_layer_bwd writes them), m[i], v[i] (fp32 moments,
 * zero before the first step). */
hgnn_status hgnn_adam_update(hgnn_ctx *ctx, void *stream, int32_t n, void *const *param, float *const *master,
                             const float *const *grad, float *const *m, float *const *v, const int64_t *numel,
                             const hgnn_adam_params *hp);
/* The same update on the rows ids[0..n_rows) (device, distinct) of an embedding table
 * store [V x feat_dim] (context dtype) with fp32 master / m / v tables of the same shape (master
 * may be NULL for fp32); grad_rows [n_rows x feat_dim] (context dtype) is the gradient of row
 * ids[i] -- the type's block of hgnn_layer_bwd's grad_x_merged of the first layer.  Rows that
 * are not listed keep their values and moments.  feat_dim * sizeof(dtype) must be a multiple of
 * 16 and the tables 16-byte aligned. */
hgnn_status hgnn_adam_update_rows(hgnn_ctx *ctx, void *stream, void *store, float *master, float *m, float *v,
                                  int32_t feat_dim, const int64_t *ids, int64_t n_rows, const void *grad_rows,
                                  const hgnn_adam_params *hp);

/* ---- Measurement aid --------------------------------------------------------------------
 * Attaches a pair of HIP events to every later dispatch of the selected kernels (the events carry the
 * dispatch's own begin and end timestamps) so that a benchmark can report a kernel's average duration
 * without a profiler attached.  A call that launches several kernels (transposed aggregation with
 * long rows) adds their durations up.
 *   hgnn_probe_select(kernel, layer): adds (kernel, layer) to the selection (at most 4 entries);
 *     kernel = hgnn_kernel_id, layer = layer index or < 0 for every layer; kernel < 0 clears the
 *     selection and discards what was collected.
 *   hgnn_probe_read(kernel, layer, ...): waits for the recorded events of that entry and returns their
 *     summed duration in milliseconds and the number of timed calls.
 * HGNN_K_GEMM_DW is the launch that holds the weight-gradient GEMM; in a mean layer's backward it also holds
 * the input-gradient GEMM's tiles when both are computed (HGNN_K_GEMM_DA then times nothing).
 * HGNN_K_RELU_BIAS_BWD is the launch at the start of a mean layer's backward: the ReLU mask / bias pass
 * over grad_h together with the zeroing of the weight gradients (HGNN_K_ZERO_GRADS times only the
 * zeroing of a layer without destination rows). */
typedef enum {
  HGNN_K_MERGE = 0, HGNN_K_TRANSPOSE_W = 1, HGNN_K_SPMM_FWD = 2, HGNN_K_GEMM_FWD = 3, HGNN_K_ZERO_GRADS = 4,
  HGNN_K_RELU_BIAS_BWD = 5, HGNN_K_GEMM_DW = 6, HGNN_K_GEMM_DA = 7, HGNN_K_SPMM_BWD = 8, HGNN_K_XENT = 9
} hgnn_kernel_id;
hgnn_status hgnn_probe_select(hgnn_ctx *ctx, int32_t kernel, int32_t layer);
hgnn_status hgnn_probe_read(hgnn_ctx *ctx, int32_t kernel, int32_t layer, double *total_ms, int64_t *launches);

#ifdef __cplusplus
}
#endif
#endif /* HGNN_H */
