// Internal declarations shared by the host runtime and the kernel launchers.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <atomic>
#include <condition_variable>
#include <cstdint>
#include <cstdio>
#include <deque>
#include <functional>
#include <memory>
#include <mutex>
#include <string>
#include <thread>
#include <vector>

#include "../../include/hgnn.h"

namespace hgnn {

constexpr int kMaxT = HGNN_MAX_TYPES;
constexpr int kMaxR = HGNN_MAX_RELS;
constexpr int kMaxSeg = kMaxR + kMaxT;  // GEMM K-segments: one per relation, one root per type
constexpr int kMaxLayers = 8;

void set_error(const char *fmt, ...);
#define HGNN_FAIL(code, ...)        \
  do {                              \
    ::hgnn::set_error(__VA_ARGS__); \
    return (code);                  \
  } while (0)
#define HGNN_HIP(expr)                                                                  \
  do {                                                                                  \
    hipError_t e_ = (expr);                                                             \
    if (e_ != hipSuccess) HGNN_FAIL(HGNN_EHIP, "%s: %s", #expr, hipGetErrorString(e_)); \
  } while (0)

// Every kernel launch of the library goes through HGNN_LAUNCH.  While a kernel probe is active on the calling
// thread the launch carries its own start/stop events, whose timestamps are those of the dispatch itself (no
// launch gap, no neighbouring work): `probe_take_events` hands out the pair.
bool probe_take_events(hipEvent_t *start, hipEvent_t *stop);
#define HGNN_LAUNCH(kernel, grid, block, shmem, stream, ...)                                          \
  do {                                                                                                \
    hipEvent_t pe0_, pe1_;                                                                            \
    if (::hgnn::probe_take_events(&pe0_, &pe1_))                                                      \
      hipExtLaunchKernelGGL(kernel, grid, block, shmem, stream, pe0_, pe1_, 0, __VA_ARGS__);          \
    else                                                                                              \
      hipLaunchKernelGGL(kernel, grid, block, shmem, stream, __VA_ARGS__);                            \
  } while (0)

// ---------------------------------------------------------------------------------------------
// By-value kernel argument tables.
// ---------------------------------------------------------------------------------------------
struct TypeTab {
  int64_t elem_off[kMaxT + 1];     // scalars of x_merged before type t (source rows)
  int64_t xroot_off[kMaxT + 1];    // scalars before type t's destination rows in the buffer the root term reads
                                   // (= elem_off for x_merged; destination rows back to back for a buffer that holds only those)
  int32_t in_dim[kMaxT];
  int32_t n_dst[kMaxT];
  int32_t row_off[kMaxT + 1];      // source rows before type t
  int32_t out_row_off[kMaxT + 1];  // destination rows before type t
  int32_t num_types;
};
struct RelTab {
  uint32_t z_off4[kMaxR + 1];      // scalars/4 of the per-relation aggregate buffer before relation r
  uint32_t zroot_off4[kMaxT + 1];  // scalars/4 of the root part of the dZ buffer before type t (bwd only)
  uint8_t src[kMaxR], dst[kMaxR];
  int32_t num_rels;
};
struct PtrTab {
  const void *w_rel[kMaxR];
  const void *w_root[kMaxT];
  const void *bias[kMaxT];
};
struct GradPtrTab {
  float *dw_rel[kMaxR];
  float *dw_root[kMaxT];
  float *dbias[kMaxT];
};
// Work list over GEMM segments (relation r -> segment r, root of type t -> segment R + t).
struct SegTab {
  int32_t tile_off[kMaxSeg + 1];
  int32_t num_segs;
};
// Work list of the weight-gradient GEMM: tiles grouped by destination type, inside a type by slice of
// destination rows, so that the tiles that read the same rows of G' (every segment ending in the type, every
// column block) are neighbours and meet in one L2.
struct DwTab {
  int32_t tile_off[kMaxT + 1];   // tiles before destination type d
  uint16_t first[kMaxT + 1];     // entries [first[d], first[d+1]) of seg / u_off belong to type d
  uint16_t u_total[kMaxT];       // 128-row blocks of dW over all segments of type d
  uint16_t u_off[kMaxSeg];       // first block of entry i inside its type
  uint8_t seg[kMaxSeg];          // segment of entry i (relation r -> r, root of type t -> R + t)
};
struct WtTab {                      // where each transposed weight lives in the scratch area
  uint32_t rel4[kMaxR];
  uint32_t root4[kMaxT];
};

// Weight transposes as a job list (Wt[h][f] = W[f][h] per K-segment, in 32x32 tiles), so that the blocks doing them can
// be the first blocks of another launch.
struct TransposeJobs {
  const void *w[kMaxSeg];
  uint32_t off4[kMaxSeg];           // scalars/4 of the transposed copy inside `out`
  int32_t F[kMaxSeg];
  int32_t tile_off[kMaxSeg + 1];    // 32x32 tiles before job i
  int32_t n, H, blocks;             // blocks = blocks that work on the tiles (0: nothing to do)
  void *out;
};

// Device-side index arrays of one layer (all int32, inside the graph's device block).
struct LayerDev {
  const int32_t *rel_row_off, *rel_edge_off, *rowptr, *colidx, *cptr, *crow;
  const int32_t *cperm;                  // CSR position of each transpose entry (uploaded for the attention variant only)
  const int32_t *chunk_row, *chunk_beg;  // transpose rows longer than kLongRow, split in chunks of kChunk edges
  const int32_t *long_row, *long_chunk0; // the long rows and the first chunk of each (n_long + 1 entries)
  int32_t rows, edges, src_rows, n_long, n_chunks;
};

constexpr int kLongRow = 16;  // transpose rows above this length are reduced chunk-wise
constexpr int kChunk = 16;

struct LayerHost {
  int64_t rows = 0, edges = 0, src_rows = 0, tedges = 0;
  int64_t n_src[kMaxT], n_dst[kMaxT];
  // offsets in int32 units into the slab
  size_t o_rel_row_off = 0, o_rel_edge_off = 0, o_rowptr = 0, o_colidx = 0, o_perm = 0, o_cptr = 0,
         o_crow = 0, o_cperm = 0, o_chunk_row = 0, o_chunk_beg = 0, o_long_row = 0, o_long_chunk0 = 0;
  int32_t n_long = 0, n_chunks = 0;
  int32_t max_chunks = 0, max_long = 0;
  uint32_t tmask = ~0u;  // vertex types whose source rows get transpose entries
  hgnn_coo_layer in;  // caller's arrays (valid until the build finishes)
};

struct Slab {  // pinned host block + device block of equal capacity
  int32_t *host = nullptr;
  int32_t *dev = nullptr;
  size_t cap = 0;  // in int32 units
};

class ThreadPool {
 public:
  explicit ThreadPool(int n);
  ~ThreadPool();
  int size() const { return nthreads_; }
  // Runs fn(chunk) for chunk in [0, nchunks) on the workers plus the caller; returns when all are done.
  void parallel_for(int nchunks, const std::function<void(int)> &fn);

 private:
  void worker();
  void drain();
  int nthreads_;
  std::vector<std::thread> th_;
  std::mutex m_;
  std::condition_variable cv_, done_cv_;
  const std::function<void(int)> *fn_ = nullptr;
  int nchunks_ = 0;
  std::atomic<int> next_{0};
  int active_ = 0;
  uint64_t epoch_ = 0;
  bool stop_ = false;
};

// One builder: a host thread that takes whole graphs off the context's queue, its worker pool and its scratch.
// Growable int64 array whose new space stays uninitialised (a std::vector would zero it, and its push_back
// checks the capacity on every element).
struct I64Buf {
  int64_t *p = nullptr;
  size_t n = 0, cap = 0;
  I64Buf() = default;
  I64Buf(const I64Buf &) = delete;
  I64Buf &operator=(const I64Buf &) = delete;
  ~I64Buf() { free(p); }
  bool reserve(size_t c) {
    if (c <= cap) return true;
    c = std::max(c, cap + cap / 2);  // grow in few, large steps: each one is a system call that remaps pages
    void *q = realloc(p, c * sizeof(int64_t));
    if (!q) return false;
    p = (int64_t *)q;
    cap = c;
    return true;
  }
  const int64_t *data() const { return p; }
  size_t size() const { return n; }
};

struct Builder {
  ThreadPool *pool = nullptr;
  std::thread th;
  std::vector<int32_t> key, col, hist, tkey;
  std::vector<std::vector<int32_t>> long_lists;
  std::vector<int32_t> local_of[kMaxT];  // sampler: local row of a global vertex id (-1 = not in the hop), per type
  std::vector<int64_t> hop_ids[2][kMaxT];  // sampler: destination / source lists of the current hop
  I64Buf edge_dst;                         // sampler: local destinations of the hop's edges
};

// A mini-batch to be sampled on a builder's thread before its index arrays are built, and what the sampling
// produced (the arrays hgnn_coo_layer points to).
struct SampleJob {
  const hgnn_sampler *sampler = nullptr;
  int32_t target_type = 0;
  uint64_t seed = 0;
  std::vector<int64_t> targets;
  std::vector<int32_t> fanouts;                 // per hop, nearest the targets first
  std::vector<int32_t> transpose[kMaxLayers];   // per layer: empty (= all types) or [T]
  I64Buf edge_index[kMaxLayers];                // [2 x E]: local source, local destination
  I64Buf edge_id[kMaxLayers];
  int64_t rel_edge_off[kMaxLayers][kMaxR + 1];  // edges of relation r in a layer's lists: [rel_edge_off[r], rel_edge_off[r+1])
  int64_t n_src[kMaxLayers][kMaxT], n_dst[kMaxLayers][kMaxT];
  std::vector<int64_t> ids[kMaxT];              // global ids of the first layer's source rows
};

}  // namespace hgnn

struct hgnn_sampler {
  std::vector<int64_t> num_nodes, edge_off;
  std::vector<const int64_t *> in_indptr;
  std::vector<const int32_t *> in_nbr;
};

struct hgnn_graph {
  int32_t num_layers = 0;
  hgnn::LayerHost L[hgnn::kMaxLayers];
  hgnn::Slab slab;
  size_t used = 0;
  std::mutex m;
  std::condition_variable cv;
  int state = 0;  // 0 building, 1 uploaded (event recorded), 2 failed
  int status = HGNN_OK;
  std::string err;
  hipEvent_t ready = nullptr;
  std::unique_ptr<hgnn::SampleJob> job;  // set for hgnn_sample_and_build
  bool sampled = false;                  // the job's results are complete (guarded by m)
  bool with_perm = true;                 // the build writes perm / cperm (fixed when the build is planned)
  size_t o_ids[hgnn::kMaxT] = {};        // per type: offset of the sampled ids in the block (int32 units)
};

struct hgnn_ctx {
  int device = 0;  // < 0: host-only context (index build and views only)
  int32_t T = 0, R = 0;
  int32_t rel_src[hgnn::kMaxR], rel_dst[hgnn::kMaxR];
  int32_t heads = 1, agg = 0, fuse = 0, dtype = 0;
  bool legacy_gemm = true;  // false with HGNN_DMA_GEMM set in the environment when the context is created: the bf16 forward
                            // GEMM runs on the LDS-DMA core (gemm_dma.h), which measures slower than the register-staged one
  std::vector<hgnn::Builder *> builders;  // each takes whole graphs off the queue and owns a slice of the host threads
  hipStream_t side = nullptr;
  std::mutex qm;
  std::condition_variable qcv;
  std::deque<hgnn_graph *> queue;
  bool stop = false;
  std::mutex pm;  // slab / event pool
  std::vector<hgnn::Slab> free_slabs;
  std::vector<hipEvent_t> free_events;
  bool build_perm = true;            // later builds produce perm / cperm (hgnn_set_build_permutation)
  std::vector<uint8_t> edge_types8;  // compact copy of the registered global edge-type table
  uint64_t types_version = 1;        // bumped whenever that table is replaced
  // device-side index build (hgnn_build_semantic_csr_device): its scratch and its copy of the table above
  void *dev_tmp = nullptr;
  size_t dev_tmp_cap = 0;
  uint8_t *dev_types8 = nullptr;
  uint64_t dev_types8_version = 0;
  // the same table as runs of equal type, kept when there are few of them (edge ids grouped by relation, the usual
  // case): type of id = run_rel[j], j = the run that holds id, found from run_lut[id >> run_shift] (the run in which
  // that block of ids starts) by stepping over at most the few boundaries inside the block; a few hundred cached
  // bytes replace a random read into a table far larger than the caches
  std::vector<int64_t> run_end;
  std::vector<uint8_t> run_rel, run_lut;
  int run_shift = 0;
  std::vector<std::unique_ptr<hgnn::SampleJob>> free_jobs;  // released sampled mini-batches: their buffers are reused (pm)
  // kernel probe (measurement aid)
  int probe_sel[4][2];  // selected (kernel, layer) pairs
  int probe_n = 0;
  std::vector<int> probe_slot;  // selection each recorded event pair belongs to
  std::vector<uint8_t> probe_first;  // 1 for the first launch of a probed call (a call may launch several kernels)
  std::vector<std::pair<hipEvent_t, hipEvent_t>> probe_events;
  size_t probe_used = 0;
};

namespace hgnn {
// log2 of the lanes that share one feature row of `max_dim` scalars: 16 bytes per lane, at most a wavefront
static inline int lanes_log2_for(int max_dim, int esize) {
  int nvec = (max_dim * esize + 15) / 16;
  int l = 0;
  while ((1 << l) < nvec && l < 6) ++l;
  return l;
}

void build_graph_job(hgnn_ctx *ctx, Builder &b, hgnn_graph *g);  // host_build.cpp
hgnn_status plan_graph(hgnn_ctx *ctx, hgnn_graph *g, std::string &msg);  // api.cpp
void index_edge_type_runs(hgnn_ctx *ctx);                                   // api.cpp: fills run_end / run_rel
hgnn_status run_sample_job(hgnn_ctx *ctx, Builder &b, hgnn_graph *g, std::string &msg);  // sampler.cpp

// noalloc.hip: the fixed device work area of hgnn_layer_fwd_static
hgnn_status static_scratch_init(int device);  // with `device` current
void *static_scratch_ptr(int device);
// api.cpp: hgnn_layer_fwd of a mean-aggregation layer with its work area laid out compactly in `area`
hgnn_status layer_fwd_static_area(hgnn_ctx *ctx, void *stream, hgnn_graph *g, int32_t layer, const hgnn_layer_params *p,
                                  const void *x, void *h, void *saved, size_t saved_bytes, void *area, size_t area_bytes);

// ---- kernel launchers (kernels_*.hip); all enqueue on `s` and return ----
// mode 0: rows ids[t][i] of store t -> type-first `out`; mode 1: the same rows -> row pos[t][i] of one interleaved buffer
// `out` (all types one width); mode 2: row pos[t][i] of `interleaved` -> type-first `out`
hgnn_status launch_merge(hipStream_t s, int dtype, int T, const void *const *store, const int32_t *feat_dim,
                         const int64_t *const *ids, const int64_t *n_rows, const int64_t *elem_off, void *out, int mode = 0,
                         const int32_t *const *pos = nullptr, const void *interleaved = nullptr);
// rows [row_begin,row_end) of the merged CSR: z[row] = mean of the x rows in colidx (rounded to the storage type);
// zlo (optional, same layout): what that rounding dropped, rounded in turn
// tj (optional): weight transposes that ride in the same launch as its first blocks (in a launch of their own when
// the aggregation runs on the kernels for ragged widths)
hgnn_status launch_spmm_fwd(hipStream_t s, int dtype, const LayerDev &L, const TypeTab &tt, const RelTab &rt,
                            int max_dim, const void *x, void *z, void *zlo, int row_begin, int row_end,
                            const TransposeJobs *tj = nullptr);
// the same aggregate in the two steps of the paper's Algorithm 1: FeatureCat [edges x F] = gathered source rows,
// then a mean per merged row (all types one width F)
hgnn_status launch_aggregate_literal(hipStream_t s, int dtype, const LayerDev &L, int F, const void *x, void *feature_cat,
                                     void *z, void *zlo);
// dx[c] = sum over transpose row c of dz[crow] (+ root part for destination rows)
hgnn_status launch_spmm_bwd(hipStream_t s, int dtype, const LayerDev &L, const TypeTab &tt, const RelTab &rt,
                            const PtrTab &pt, int max_dim, uint32_t want_types, const void *dz, void *dx, float *partial);
// uniform feature width: return false when the width is outside what they cover (caller falls back)
bool launch_spmm_fwd_uniform(hipStream_t s, int dtype, const LayerDev &L, int F, const void *x, void *z, void *zlo,
                             int row_begin, int row_end, const uint64_t *gaddr = nullptr, const TransposeJobs *tj = nullptr);
void make_transpose_jobs(const TypeTab &tt, const RelTab &rt, const PtrTab &pt, const WtTab &wt, int H, void *wt_buf,
                         TransposeJobs &tj);
hgnn_status launch_transpose_jobs(hipStream_t s, int dtype, const TransposeJobs &tj);
// Aggregation straight from the per-type feature stores: gaddr[e] = address of the row that edge e reads (the row
// ids[t][c - row_off[t]] of store t for the merged source row c = colidx[e]); launch_spmm_fwd_uniform then takes
// gaddr in place of x.
struct GatherSrc {
  const void *store[kMaxT];
  const int64_t *ids[kMaxT];
  int32_t row_off[kMaxT + 1];
  int32_t num_types;
};
hgnn_status launch_gather_addresses(hipStream_t s, const LayerDev &L, const GatherSrc &gs, int row_bytes, uint64_t *gaddr);
bool launch_spmm_bwd_uniform(hipStream_t s, int dtype, const LayerDev &L, const TypeTab &tt, const RelTab &rt, const PtrTab &pt,
                             int F, uint32_t want, const void *dz, void *dx, float *partial);
hgnn_status launch_transpose_weights(hipStream_t s, int dtype, const TypeTab &tt, const RelTab &rt,
                                     const PtrTab &pt, const WtTab &wt, int H, void *wt_buf);
// mode 0: all segments of every type fused (bias/activation epilogue, writes h)
// mode 1: one segment `only_seg`, accumulated into the fp32 buffer acc32 (naive launch structure)
hgnn_status launch_gemm_fwd(hipStream_t s, int dtype, const LayerDev &L, const TypeTab &tt, const RelTab &rt,
                            const PtrTab &pt, const WtTab &wt, const SegTab &tiles, const uint32_t *live_mask, int H,
                            int relu, const void *x, const void *z, const void *zlo, const void *wt_buf, void *h,
                            int only_seg, float *acc32, int tile_mn = 128);
// bf16 forward on the LDS-DMA core; false = shape not covered (nothing was launched), else *st is the launch's status
bool launch_gemm2_fwd(hipStream_t s, const TypeTab &tt, const RelTab &rt, const PtrTab &pt, const WtTab &wt, const uint32_t *live_mask,
                      int H, int relu, const void *x, const void *z, const void *zlo, const void *wt_buf, void *h, hgnn_status *st);
// attention variant
hgnn_status launch_attn_proj(hipStream_t s, int dtype, const TypeTab &tt, const PtrTab &w_type_as_root, const SegTab &tiles, int H,
                             const void *x, void *z, bool z_f32 = false);
hgnn_status launch_attn_agg(hipStream_t s, int dtype, const LayerDev &L, const TypeTab &tt, const RelTab &rt,
                            const void *const *a_src, const void *const *a_dst, int H, int heads, const void *z, void *mout,
                            float *mx, float *ls);
hgnn_status launch_attn_sem(hipStream_t s, int dtype, const LayerDev &L, const TypeTab &tt, const RelTab &rt, int H, const void *mbuf,
                            const void *w_sem, const void *b_sem, const void *q_sem, void *tbuf, float *wsum);
hgnn_status launch_attn_beta(hipStream_t s, const TypeTab &tt, const RelTab &rt, const float *wsum, float *beta, const float *dbeta,
                             float *coef, int mode);
hgnn_status launch_attn_fuse(hipStream_t s, int dtype, const LayerDev &L, const TypeTab &tt, const RelTab &rt, const PtrTab &pt, int H,
                             int relu, const void *mbuf, const float *beta, void *h);
hgnn_status launch_attn_zero(hipStream_t s, float *const *ptrs, const int64_t *counts, int n);
hgnn_status launch_attn_dbeta(hipStream_t s, int dtype, const LayerDev &L, const TypeTab &tt, const RelTab &rt, int H, int ldg,
                              const void *gp, const void *mbuf, float *dbeta);
hgnn_status launch_attn_du(hipStream_t s, int dtype, const LayerDev &L, const RelTab &rt, const void *tbuf, const void *q_sem,
                           const float *coef, void *du, float *dq, float *dbs);
hgnn_status launch_attn_dm(hipStream_t s, int dtype, const LayerDev &L, const TypeTab &tt, const RelTab &rt, int H, int ldg, const void *du,
                           const void *w_sem, const void *gp, const float *beta, void *dm);
hgnn_status launch_attn_dws(hipStream_t s, int dtype, int64_t rows, int H, const void *mbuf, const void *du, float *dws);
hgnn_status launch_attn_agg_bwd(hipStream_t s, int dtype, const LayerDev &L, const TypeTab &tt, const RelTab &rt, const void *const *a_src,
                                const void *const *a_dst, float *const *da_src, float *const *da_dst, int H, int heads, const void *z,
                                const void *mbuf, const void *dm, const float *mx, const float *ls, float *alpha, float *dsb,
                                float *dsum, void *dz, float *partial);
hgnn_status launch_bias_act(hipStream_t s, int dtype, const TypeTab &tt, const PtrTab &pt, int H, int relu,
                            int type, const float *acc32, void *h);
// gp has leading dimension ldg >= H (zero beyond H), and so have the weights in `pt`
hgnn_status launch_gemm_da(hipStream_t s, int dtype, const LayerDev &L, const TypeTab &tt, const RelTab &rt,
                           const PtrTab &pt, const SegTab &tiles, int ldg, bool fast, const void *gp, void *dz);
hgnn_status launch_gemm_bwd(hipStream_t s, int dtype, const LayerDev &L, const TypeTab &tt, const RelTab &rt,
                            const PtrTab &pt, const DwTab &da_tiles, const GradPtrTab &gt, const DwTab &dw_tiles,
                            int split_rows, int H, int ldg, bool fast, const void *x, const void *z, const void *gp, void *dz,
                            const float *bpart, int rpb);  // bpart != NULL: the launch also reduces the partial bias sums
hgnn_status launch_gemm_dw(hipStream_t s, int dtype, const LayerDev &L, const TypeTab &tt, const RelTab &rt,
                           const GradPtrTab &gt, const DwTab &tiles, int split_rows, int H, int ldg, bool fast,
                           const void *x, const void *z, const void *gp);
hgnn_status launch_adam_dense(hipStream_t s, int dtype, int n, void *const *param, float *const *master,
                              const float *const *grad, float *const *m, float *const *v, const int64_t *numel,
                              float lr, float b1, float b2, float eps, double c1, double c2);
hgnn_status launch_adam_rows(hipStream_t s, int dtype, void *store, float *master, float *m, float *v, int F,
                             const int64_t *ids, int64_t n_rows, const void *grad, float lr, float b1, float b2,
                             float eps, double c1, double c2);
// gp (leading dimension ldo >= H, zero beyond H) = grad_h * [h > 0] (or a plain copy without ReLU); dbias = column sums
hgnn_status launch_relu_bias_bwd(hipStream_t s, int dtype, const TypeTab &tt, int H, int ldo, int relu,
                                 const void *grad_h, const void *h, void *gp, const GradPtrTab &gt);
// zero-padded copies [F x Hp] of every weight
hgnn_status launch_pad_weights(hipStream_t s, int dtype, const TypeTab &tt, const RelTab &rt, const PtrTab &pt,
                               const WtTab &wo, int H, int Hp, void *out);
hgnn_status launch_zero_grads(hipStream_t s, const TypeTab &tt, const RelTab &rt, const GradPtrTab &gt, int H);
// ReLU mask / bias column sums (into bpart, rows_per_block rows of G per row of bpart), weight-gradient zeroing and
// padded weight copies (wpad != NULL) in one launch; launch_bias_reduce (or the blocks the merged backward GEMM
// launch sets aside for it) then turns bpart into dbias.
hgnn_status launch_bwd_prep(hipStream_t s, int dtype, const TypeTab &tt, const RelTab &rt, const PtrTab &pt, const WtTab &wo,
                            const GradPtrTab &gt, int H, int ldo, int relu, bool do_rows, bool do_zero, const void *grad_h,
                            const void *h, void *gp, float *bpart, size_t bpart_rows, void *wpad, int *rows_per_block);
hgnn_status launch_bias_reduce(hipStream_t s, const TypeTab &tt, const GradPtrTab &gt, int H, int rpb, const float *bpart);
// blocks of 256 threads that add up the partial bias sums: 32 columns of one type each
inline int bias_reduce_blocks(int num_types, int H) { return num_types * ((H + 31) / 32); }
hgnn_status launch_fill_zero(hipStream_t s, void *p, size_t bytes);
constexpr int kCvtItems = 64;  // tensors per launch of the storage-type conversion
hgnn_status launch_convert(hipStream_t s, bool widen, const void *const *src, void *const *dst, const int64_t *n, int count);
hgnn_status launch_xent(hipStream_t s, int dtype, const void *logits, const int64_t *labels, int64_t rows,
                        int classes, float *loss, void *grad);
}  // namespace hgnn
