// C ABI entry points: argument checks, per-call planning (offset tables), launch sequences.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <unistd.h>

#include "common.h"

namespace hgnn {
const char *get_error();

static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
static inline int esize(int dtype) { return dtype == HGNN_BF16 ? 2 : 4; }

static void builder_main(hgnn_ctx *ctx, Builder *bd) {
  if (ctx->device >= 0) (void)hipSetDevice(ctx->device);
  for (;;) {
    hgnn_graph *g = nullptr;
    {
      std::unique_lock<std::mutex> lk(ctx->qm);
      ctx->qcv.wait(lk, [&] { return ctx->stop || !ctx->queue.empty(); });
      if (ctx->queue.empty()) return;  // stop requested and nothing left
      g = ctx->queue.front();
      ctx->queue.pop_front();
    }
    build_graph_job(ctx, *bd, g);
  }
}

static void free_slab(hgnn_ctx *ctx, Slab &s) {
  if (ctx->device >= 0) {
    if (s.host) (void)hipHostFree(s.host);
    if (s.dev) (void)hipFree(s.dev);
  } else {
    free(s.host);
  }
  s = Slab();
}

static hgnn_status wait_built(hgnn_graph *g) {
  std::unique_lock<std::mutex> lk(g->m);
  g->cv.wait(lk, [&] { return g->state != 0; });
  if (g->state == 2) HGNN_FAIL((hgnn_status)g->status, "graph build failed: %s", g->err.c_str());
  return HGNN_OK;
}

// Everything a layer call derives from (schema, graph, parameters) before launching.
struct Plan {
  TypeTab tt;
  RelTab rt;
  PtrTab pt;
  WtTab wt;
  LayerDev dev;
  int H = 0, max_dim = 0, es = 4;
  int64_t total_dst = 0;
  size_t z_elems = 0, zroot_elems = 0, wt_elems = 0;
  size_t saved_bytes = 0, scratch_bytes = 0;
  size_t off_wt = 0, off_gp = 0, off_dz = 0, off_partial = 0, off_acc32 = 0, off_bpart = 0, bpart_rows = 0, off_zlo = 0, off_gaddr = 0;
};

// The buffer the root term reads holds the destination rows only (n_dst[t] rows per type, back to back).
static void root_rows_only(Plan &pl) {
  int64_t o = 0;
  for (int t = 0; t < pl.tt.num_types; ++t) {
    pl.tt.xroot_off[t] = o;
    o += (int64_t)pl.tt.n_dst[t] * pl.tt.in_dim[t];
  }
  pl.tt.xroot_off[pl.tt.num_types] = o;
}

static hgnn_status layer_dev(hgnn_ctx *ctx, hgnn_graph *g, int32_t layer, LayerDev &D);

static hgnn_status make_plan(hgnn_ctx *ctx, hgnn_graph *g, int32_t layer, const hgnn_layer_params *p, Plan &pl,
                             bool need_built) {
  if (!ctx || !g || !p) HGNN_FAIL(HGNN_EINVAL, "NULL context, graph or parameters");
  if (layer < 0 || layer >= g->num_layers) HGNN_FAIL(HGNN_EINVAL, "layer %d outside [0,%d)", layer, g->num_layers);
  if (ctx->agg != HGNN_AGG_MEAN || ctx->fuse != HGNN_FUSE_SUM)
    HGNN_FAIL(HGNN_EUNSUPPORTED, "only mean aggregation with sum fusion is implemented");
  if (!p->in_dim || !p->w_rel || !p->w_root || p->out_dim <= 0) HGNN_FAIL(HGNN_EINVAL, "incomplete layer parameters");
  const int T = ctx->T, R = ctx->R;
  const LayerHost &L = g->L[layer];
  pl.es = esize(ctx->dtype);
  const int vec = 16 / pl.es;
  pl.H = p->out_dim;
  std::memset(&pl.tt, 0, sizeof(pl.tt));
  std::memset(&pl.rt, 0, sizeof(pl.rt));
  std::memset(&pl.pt, 0, sizeof(pl.pt));
  std::memset(&pl.wt, 0, sizeof(pl.wt));
  pl.tt.num_types = T;
  pl.rt.num_rels = R;
  int64_t eo = 0;
  for (int t = 0; t < T; ++t) {
    if (p->in_dim[t] <= 0 || p->in_dim[t] % vec != 0)
      HGNN_FAIL(HGNN_EUNSUPPORTED, "in_dim[%d]=%d is not a positive multiple of %d", t, p->in_dim[t], vec);
    pl.tt.in_dim[t] = p->in_dim[t];
    pl.tt.n_dst[t] = (int32_t)L.n_dst[t];
    pl.tt.elem_off[t] = eo;
    pl.tt.xroot_off[t] = eo;
    eo += L.n_src[t] * (int64_t)p->in_dim[t];
    pl.tt.row_off[t + 1] = pl.tt.row_off[t] + (int32_t)L.n_src[t];
    pl.tt.out_row_off[t + 1] = pl.tt.out_row_off[t] + (int32_t)L.n_dst[t];
    if (L.n_src[t] > 0) pl.max_dim = std::max(pl.max_dim, p->in_dim[t]);
    pl.pt.w_root[t] = p->w_root[t];
    pl.pt.bias[t] = p->bias ? p->bias[t] : nullptr;
  }
  pl.tt.elem_off[T] = eo;
  pl.tt.xroot_off[T] = eo;
  pl.total_dst = pl.tt.out_row_off[T];
  if ((int64_t)pl.total_dst * pl.H >= (int64_t)1 << 40) HGNN_FAIL(HGNN_EOVERFLOW, "output too large");
  size_t z = 0, w = 0;
  for (int r = 0; r < R; ++r) {
    const int s = ctx->rel_src[r], d = ctx->rel_dst[r];
    if (!p->w_rel[r]) HGNN_FAIL(HGNN_EINVAL, "w_rel[%d] is NULL", r);
    pl.rt.src[r] = (uint8_t)s;
    pl.rt.dst[r] = (uint8_t)d;
    pl.rt.z_off4[r] = (uint32_t)(z / 4);
    z += (size_t)L.n_dst[d] * p->in_dim[s];
    pl.pt.w_rel[r] = p->w_rel[r];
    pl.wt.rel4[r] = (uint32_t)(w / 4);
    w += (size_t)p->in_dim[s] * pl.H;
  }
  pl.rt.z_off4[R] = (uint32_t)(z / 4);
  pl.z_elems = z;
  size_t zr = z;
  for (int t = 0; t < T; ++t) {
    pl.rt.zroot_off4[t] = (uint32_t)(zr / 4);
    if (p->w_root[t]) zr += (size_t)L.n_dst[t] * p->in_dim[t];
    pl.wt.root4[t] = (uint32_t)(w / 4);
    if (p->w_root[t]) w += (size_t)p->in_dim[t] * pl.H;
  }
  pl.rt.zroot_off4[T] = (uint32_t)(zr / 4);
  pl.zroot_elems = zr - z;
  pl.wt_elems = w;
  if (zr / 4 >= ((size_t)1 << 32) || w / 4 >= ((size_t)1 << 32)) HGNN_FAIL(HGNN_EOVERFLOW, "work area too large");
  pl.saved_bytes = align_up(std::max<size_t>(z, 1) * pl.es, 256);
  size_t o = 0;
  const size_t Hpad = ((size_t)pl.H + vec - 1) / vec * vec;  // the backward pads H to whole 16-byte pieces when needed
  pl.off_wt = o;      o += align_up(std::max<size_t>(w / pl.H * Hpad, 1) * pl.es, 256);
  pl.off_gp = o;      o += align_up(std::max<size_t>((size_t)pl.total_dst * Hpad, 1) * pl.es, 256);
  pl.off_dz = o;      o += align_up(std::max<size_t>(zr, 1) * pl.es, 256);
  pl.off_partial = o; o += align_up(std::max<size_t>((size_t)L.max_chunks * std::max(pl.max_dim, 1), 1) * 4, 256);
  pl.off_acc32 = o;   o += align_up(std::max<size_t>((size_t)pl.total_dst * pl.H, 1) * 4, 256);
  // partial bias-gradient sums: one row of H floats per block of destination rows of a type (64 rows per block
  // when the row pass runs in its 16-bytes-per-lane form, which the width decides; 8 otherwise)
  const bool row_pass_vec = pl.H % vec == 0 && pl.H / vec <= 256;
  pl.bpart_rows = (size_t)pl.total_dst / (row_pass_vec ? 64 : 8) + T;
  pl.off_bpart = o;   o += align_up(pl.bpart_rows * pl.H * 4, 256);
  pl.off_zlo = o;     o += (pl.es == 2 && p->relu) ? align_up(std::max<size_t>(z, 1) * pl.es, 256) : 0;
  pl.off_gaddr = o;   o += align_up(std::max<size_t>((size_t)L.edges, 1) * 8, 256);  // per-edge row addresses (gather from the stores)
  pl.scratch_bytes = o;
  if (need_built) {
    hgnn_status st = layer_dev(ctx, g, layer, pl.dev);
    if (st != HGNN_OK) return st;
  }
  return HGNN_OK;
}

// Waits for the host build and fills the device-side view of one layer's index arrays.
static hgnn_status layer_dev(hgnn_ctx *ctx, hgnn_graph *g, int32_t layer, LayerDev &D) {
  const LayerHost &L = g->L[layer];
  {
    hgnn_status st = wait_built(g);
    if (st != HGNN_OK) return st;
    if (ctx->device < 0) HGNN_FAIL(HGNN_EUNSUPPORTED, "host-only context cannot run device work");
    const int32_t *b = g->slab.dev;
    D.rel_row_off = b + L.o_rel_row_off; D.rel_edge_off = b + L.o_rel_edge_off;
    D.rowptr = b + L.o_rowptr; D.colidx = b + L.o_colidx; D.cptr = b + L.o_cptr; D.crow = b + L.o_crow;
    D.cperm = b + L.o_cperm;
    D.chunk_row = b + L.o_chunk_row; D.chunk_beg = b + L.o_chunk_beg;
    D.long_row = b + L.o_long_row; D.long_chunk0 = b + L.o_long_chunk0;
    D.rows = (int32_t)L.rows; D.edges = (int32_t)L.edges; D.src_rows = (int32_t)L.src_rows;
    D.n_long = L.n_long; D.n_chunks = L.n_chunks;
  }
  return HGNN_OK;
}

// While alive, the launches made on this thread are timed if the probe selects (kernel, layer).
static thread_local hgnn_ctx *tl_probe_ctx = nullptr;
static thread_local int tl_probe_slot = -1;
static thread_local bool tl_probe_first = false;

struct Probe {
  bool active = false;
  Probe(hgnn_ctx *c, hipStream_t, int kernel, int layer, bool enabled = true) {
    int slot = -1;
    if (!enabled) return;
    for (int i = 0; i < c->probe_n; ++i)
      if (c->probe_sel[i][0] == kernel && (c->probe_sel[i][1] < 0 || c->probe_sel[i][1] == layer)) slot = i;
    if (slot < 0) return;
    tl_probe_ctx = c;
    tl_probe_slot = slot;
    tl_probe_first = true;
    active = true;
  }
  ~Probe() {
    if (active) tl_probe_ctx = nullptr;
  }
};

bool probe_take_events(hipEvent_t *start, hipEvent_t *stop) {
  hgnn_ctx *c = tl_probe_ctx;
  if (!c) return false;
  if (c->probe_used == c->probe_events.size()) {
    hipEvent_t a, b;
    if (hipEventCreate(&a) != hipSuccess) return false;
    if (hipEventCreate(&b) != hipSuccess) { (void)hipEventDestroy(a); return false; }
    c->probe_events.emplace_back(a, b);
  }
  c->probe_slot.resize(c->probe_events.size());
  c->probe_first.resize(c->probe_events.size());
  c->probe_slot[c->probe_used] = tl_probe_slot;
  c->probe_first[c->probe_used] = tl_probe_first ? 1 : 0;
  tl_probe_first = false;
  auto &pr = c->probe_events[c->probe_used++];
  *start = pr.first;
  *stop = pr.second;
  return true;
}

// ---------------------------------------------------------------------------------------------
// Attention variant: plan (tables, work-area layout) shared by forward and backward.
// ---------------------------------------------------------------------------------------------
struct AttnPlan {
  TypeTab tt;
  RelTab rt;
  PtrTab pt;      // w_root := w_type (per-type projection), bias
  LayerDev dev;
  int H = 0, heads = 1, es = 4;
  int64_t src_rows = 0, rows = 0, edges = 0, total_dst = 0;
  // saved (forward -> backward)
  size_t s_z = 0, s_m = 0, s_t = 0, s_mx = 0, s_ls = 0, s_beta = 0, s_wsum = 0, saved_bytes = 0;
  // scratch (backward)
  size_t c_gp = 0, c_small = 0, c_du = 0, c_dm = 0, c_alpha = 0, c_ds = 0, c_dsum = 0, c_dz = 0, c_partial = 0, scratch_bytes = 0;
  // fp32 copies of what the boundary holds in bf16 (scratch; bf16 storage only)
  bool widen = false;
  size_t c_w32 = 0, c_h32 = 0, c_g32 = 0, c_dz16 = 0;
};
constexpr int kSemDimHost = 128;

static hgnn_status make_attn_plan(hgnn_ctx *ctx, hgnn_graph *g, int32_t layer, const hgnn_layer_params *p, AttnPlan &pl,
                                  bool need_built) {
  if (!ctx || !g || !p) HGNN_FAIL(HGNN_EINVAL, "NULL context, graph or parameters");
  if (layer < 0 || layer >= g->num_layers) HGNN_FAIL(HGNN_EINVAL, "layer %d outside [0,%d)", layer, g->num_layers);
  if (ctx->fuse != HGNN_FUSE_SEMATTN) HGNN_FAIL(HGNN_EUNSUPPORTED, "attention aggregation is implemented with semantic-attention fusion only");
  if (!p->in_dim || !p->w_type || !p->a_src || !p->a_dst || !p->w_sem || !p->b_sem || !p->q_sem || p->out_dim <= 0)
    HGNN_FAIL(HGNN_EINVAL, "incomplete attention layer parameters");
  const int T = ctx->T, R = ctx->R;
  const LayerHost &L = g->L[layer];
  // The attention variant computes and keeps its intermediates (projected features, aggregates, scores, every
  // gradient between the stages) in fp32 whatever the storage type: the gradients of the attention vectors are what
  // is left of a cancellation between the neighbours of a vertex (the softmax gradient sums to zero over them), and
  // the ReLU decisions sit on sums without head-room, so both need more than bf16 intermediates carry.  In bf16
  // storage the inputs, parameters and incoming gradients are widened into scratch (exact) and the layer output and
  // the input gradient are rounded once on the way out.
  pl.es = 4;
  pl.widen = ctx->dtype == HGNN_BF16;
  const int vec = 4, vec_io = 16 / esize(ctx->dtype);
  pl.H = p->out_dim;
  pl.heads = ctx->heads;
  if (pl.H % pl.heads) HGNN_FAIL(HGNN_EINVAL, "out_dim %d is not a multiple of heads %d", pl.H, pl.heads);
  const int D = pl.H / pl.heads;
  auto pow2 = [](int n) { return n > 0 && (n & (n - 1)) == 0; };
  if (D % vec || !pow2(D / vec) || !pow2(pl.H / vec) || pl.H / vec > 64)
    HGNN_FAIL(HGNN_EUNSUPPORTED, "attention needs out_dim/heads = %d scalars x a power of two and out_dim/%d a power of two <= 64", vec, vec);
  if (L.tmask != ~0u) HGNN_FAIL(HGNN_EINVAL, "the attention variant needs the transpose entries of every vertex type");
  std::memset(&pl.tt, 0, sizeof(pl.tt));
  std::memset(&pl.rt, 0, sizeof(pl.rt));
  std::memset(&pl.pt, 0, sizeof(pl.pt));
  pl.tt.num_types = T;
  pl.rt.num_rels = R;
  int64_t eo = 0;
  for (int t = 0; t < T; ++t) {
    if (p->in_dim[t] <= 0 || p->in_dim[t] % vec_io != 0)
      HGNN_FAIL(HGNN_EUNSUPPORTED, "in_dim[%d]=%d is not a positive multiple of %d", t, p->in_dim[t], vec_io);
    if (!p->w_type[t] || ((uintptr_t)p->w_type[t] & 15)) HGNN_FAIL(HGNN_EINVAL, "w_type[%d] is NULL or not 16-byte aligned", t);
    pl.tt.in_dim[t] = p->in_dim[t];
    pl.tt.n_dst[t] = (int32_t)L.n_dst[t];
    pl.tt.elem_off[t] = eo;
    pl.tt.xroot_off[t] = eo;
    eo += L.n_src[t] * (int64_t)p->in_dim[t];
    pl.tt.row_off[t + 1] = pl.tt.row_off[t] + (int32_t)L.n_src[t];
    pl.tt.out_row_off[t + 1] = pl.tt.out_row_off[t] + (int32_t)L.n_dst[t];
    pl.pt.w_root[t] = p->w_type[t];
    pl.pt.bias[t] = p->bias ? p->bias[t] : nullptr;
  }
  pl.tt.elem_off[T] = eo;
  for (int r = 0; r < R; ++r) {
    if (!p->a_src[r] || !p->a_dst[r] || (((uintptr_t)p->a_src[r] | (uintptr_t)p->a_dst[r]) & 15))
      HGNN_FAIL(HGNN_EINVAL, "a_src[%d] / a_dst[%d] is NULL or not 16-byte aligned", r, r);
    pl.rt.src[r] = (uint8_t)ctx->rel_src[r];
    pl.rt.dst[r] = (uint8_t)ctx->rel_dst[r];
  }
  if (((uintptr_t)p->w_sem | (uintptr_t)p->b_sem | (uintptr_t)p->q_sem) & 15) HGNN_FAIL(HGNN_EINVAL, "semantic attention parameters must be 16-byte aligned");
  pl.src_rows = L.src_rows; pl.rows = L.rows; pl.edges = L.edges; pl.total_dst = pl.tt.out_row_off[T];
  const size_t H = (size_t)pl.H, es = (size_t)pl.es, hd = (size_t)pl.heads;
  auto take = [](size_t &o, size_t bytes) { const size_t at = o; o += align_up(std::max<size_t>(bytes, 1), 256); return at; };
  size_t o = 0;
  pl.s_z = take(o, (size_t)pl.src_rows * H * es);
  pl.s_m = take(o, (size_t)pl.rows * H * es);
  pl.s_t = take(o, (size_t)pl.rows * kSemDimHost * es);
  pl.s_mx = take(o, (size_t)pl.rows * hd * 4);
  pl.s_ls = take(o, (size_t)pl.rows * hd * 4);
  pl.s_beta = take(o, (size_t)kMaxR * 4);
  pl.s_wsum = take(o, (size_t)kMaxR * 4);
  pl.saved_bytes = o;
  o = 0;
  pl.c_gp = take(o, (size_t)pl.total_dst * H * es);
  pl.c_small = take(o, (size_t)4 * kMaxR * 4);                 // dbeta, coef
  pl.c_du = take(o, (size_t)pl.rows * kSemDimHost * es);
  pl.c_dm = take(o, (size_t)pl.rows * H * es);
  pl.c_alpha = take(o, (size_t)pl.edges * hd * 4);
  pl.c_ds = take(o, (size_t)pl.edges * hd * 4);
  pl.c_dsum = take(o, (size_t)pl.rows * hd * 4);
  pl.c_dz = take(o, (size_t)pl.src_rows * H * es);
  pl.c_partial = take(o, (size_t)L.max_chunks * H * 4);
  if (pl.widen) {
    if (pl.H % vec_io) HGNN_FAIL(HGNN_EUNSUPPORTED, "out_dim %d is not a multiple of %d", pl.H, vec_io);
    size_t wf = (size_t)2 * R * H + H * kSemDimHost + 2 * kSemDimHost + (size_t)T * H;
    pl.c_w32 = take(o, wf * 4);
    pl.c_h32 = take(o, (size_t)pl.total_dst * H * 4);
    pl.c_g32 = take(o, (size_t)pl.total_dst * H * 4);
    pl.c_dz16 = take(o, (size_t)pl.src_rows * H * 2);   // the projected features' gradient rounded for the projection's backward
  }
  pl.scratch_bytes = o;
  if (need_built) return layer_dev(ctx, g, layer, pl.dev);
  return HGNN_OK;
}

// fp32 stand-ins (in the scratch area) of the parameters of a bf16 layer that its fp32 kernels read: attention vectors,
// semantic-attention parameters, biases.  `q` then takes the place of the caller's parameter block for those kernels.
// The per-type projection weights and the input stay bf16: the projection and its backward run on the bf16 MFMA kernels
// (a product of two bf16 numbers is exact in fp32).  Not copyable: q points into the arrays beside it.
struct AttnWide {
  hgnn_layer_params q;
  const void *bias[kMaxT], *a_src[kMaxR], *a_dst[kMaxR];
  AttnWide() = default;
  AttnWide(const AttnWide &) = delete;
};
static hgnn_status attn_widen(hgnn_ctx *ctx, hipStream_t s, AttnPlan &pl, const hgnn_layer_params *p, char *sc, AttnWide &w) {
  const int T = ctx->T, R = ctx->R;
  const int64_t H = pl.H;
  std::vector<const void *> src;
  std::vector<void *> dst;
  std::vector<int64_t> cnt;
  float *at = (float *)(sc + pl.c_w32);
  auto put = [&](const void *from, int64_t n) -> const void * {
    if (!from) return nullptr;
    float *to = at;
    at += n;
    src.push_back(from); dst.push_back(to); cnt.push_back(n);
    return to;
  };
  w.q = *p;
  for (int t = 0; t < T; ++t) {
    w.bias[t] = put(p->bias ? p->bias[t] : nullptr, H);
    pl.pt.bias[t] = w.bias[t];
  }
  for (int r = 0; r < R; ++r) {
    w.a_src[r] = put(p->a_src[r], H);
    w.a_dst[r] = put(p->a_dst[r], H);
  }
  w.q.bias = p->bias ? w.bias : nullptr;
  w.q.a_src = w.a_src;
  w.q.a_dst = w.a_dst;
  w.q.w_sem = put(p->w_sem, H * kSemDimHost);
  w.q.b_sem = put(p->b_sem, kSemDimHost);
  w.q.q_sem = put(p->q_sem, kSemDimHost);
  return launch_convert(s, true, src.data(), dst.data(), cnt.data(), (int)src.size());
}

static hgnn_status attn_fwd(hgnn_ctx *ctx, void *stream, hgnn_graph *g, int32_t layer, const hgnn_layer_params *p, const void *x,
                            void *h, void *saved, size_t saved_bytes, void *scratch, size_t scratch_bytes) {
  AttnPlan pl;
  hgnn_status st = make_attn_plan(ctx, g, layer, p, pl, true);
  if (st != HGNN_OK) return st;
  if (pl.src_rows > 0 && !x) HGNN_FAIL(HGNN_EINVAL, "x_merged is NULL");
  if (pl.total_dst > 0 && !h) HGNN_FAIL(HGNN_EINVAL, "h_out is NULL");
  if (!saved || !scratch) HGNN_FAIL(HGNN_EINVAL, "NULL work area");
  if (saved_bytes < pl.saved_bytes || scratch_bytes < pl.scratch_bytes)
    HGNN_FAIL(HGNN_EINVAL, "work areas too small: need %zu saved, %zu scratch bytes", pl.saved_bytes, pl.scratch_bytes);
  if (((uintptr_t)saved | (uintptr_t)scratch | (uintptr_t)x | (uintptr_t)h) & 15)
    HGNN_FAIL(HGNN_EINVAL, "device buffers must be 16-byte aligned");
  hipStream_t s = (hipStream_t)stream;
  HGNN_HIP(hipStreamWaitEvent(s, g->ready, 0));
  char *sv = (char *)saved;
  const int T = ctx->T;
  AttnWide wide;
  void *h_io = h;
  if (pl.widen) {
    if ((st = attn_widen(ctx, s, pl, p, (char *)scratch, wide)) != HGNN_OK) return st;
    p = &wide.q;
    h = (char *)scratch + pl.c_h32;
  }
  SegTab tl;   // projection tiles: every source row of every type
  std::memset(&tl, 0, sizeof(tl));
  tl.num_segs = T;
  const int tn = (pl.H + 127) / 128;
  for (int t = 0; t < T; ++t) tl.tile_off[t + 1] = tl.tile_off[t] + (int)((g->L[layer].n_src[t] + 127) / 128) * tn;
  {
    Probe pb(ctx, s, HGNN_K_GEMM_FWD, layer);
    // bf16 storage: bf16 operands straight from the caller's buffers, fp32 result
    if ((st = launch_attn_proj(s, ctx->dtype, pl.tt, pl.pt, tl, pl.H, x, sv + pl.s_z, pl.widen)) != HGNN_OK) return st;
  }
  {
    Probe pb(ctx, s, HGNN_K_SPMM_FWD, layer);
    if ((st = launch_attn_agg(s, HGNN_F32, pl.dev, pl.tt, pl.rt, p->a_src, p->a_dst, pl.H, pl.heads, sv + pl.s_z, sv + pl.s_m,
                              (float *)(sv + pl.s_mx), (float *)(sv + pl.s_ls))) != HGNN_OK) return st;
  }
  float *wsum = (float *)(sv + pl.s_wsum), *beta = (float *)(sv + pl.s_beta);
  if ((st = launch_fill_zero(s, wsum, (size_t)kMaxR * 4)) != HGNN_OK) return st;
  if ((st = launch_attn_sem(s, HGNN_F32, pl.dev, pl.tt, pl.rt, pl.H, sv + pl.s_m, p->w_sem, p->b_sem, p->q_sem, sv + pl.s_t, wsum)) != HGNN_OK) return st;
  if ((st = launch_attn_beta(s, pl.tt, pl.rt, wsum, beta, nullptr, nullptr, 0)) != HGNN_OK) return st;
  if ((st = launch_attn_fuse(s, HGNN_F32, pl.dev, pl.tt, pl.rt, pl.pt, pl.H, p->relu, sv + pl.s_m, beta, h)) != HGNN_OK) return st;
  if (pl.widen && pl.total_dst > 0) {
    const void *src = h;
    const int64_t n = pl.total_dst * (int64_t)pl.H;
    return launch_convert(s, false, &src, &h_io, &n, 1);
  }
  return HGNN_OK;
}

static hgnn_status attn_bwd(hgnn_ctx *ctx, void *stream, hgnn_graph *g, int32_t layer, const hgnn_layer_params *p, const void *x,
                            const void *h_out, const void *saved, const void *grad_h, void *grad_x, const hgnn_layer_grads *go,
                            void *scratch, size_t scratch_bytes) {
  AttnPlan pl;
  hgnn_status st = make_attn_plan(ctx, g, layer, p, pl, true);
  if (st != HGNN_OK) return st;
  if (!saved || !scratch || !go) HGNN_FAIL(HGNN_EINVAL, "NULL work area or gradient table");
  if (!go->dw_type || !go->da_src || !go->da_dst || !go->dw_sem || !go->db_sem || !go->dq_sem)
    HGNN_FAIL(HGNN_EINVAL, "the attention backward needs every gradient buffer of the attention parameters");
  if (pl.total_dst > 0 && (!x || !grad_h || (p->relu && !h_out))) HGNN_FAIL(HGNN_EINVAL, "NULL input");
  if (scratch_bytes < pl.scratch_bytes) HGNN_FAIL(HGNN_EINVAL, "scratch too small: need %zu bytes", pl.scratch_bytes);
  if (((uintptr_t)saved | (uintptr_t)scratch | (uintptr_t)x | (uintptr_t)grad_h | (uintptr_t)grad_x) & 15)
    HGNN_FAIL(HGNN_EINVAL, "device buffers must be 16-byte aligned");
  const int R = ctx->R, T = ctx->T, H = pl.H;
  hipStream_t s = (hipStream_t)stream;
  HGNN_HIP(hipStreamWaitEvent(s, g->ready, 0));
  const char *sv = (const char *)saved;
  char *sc = (char *)scratch;
  const LayerHost &L = g->L[layer];
  AttnWide wide;
  if (pl.widen) {
    if ((st = attn_widen(ctx, s, pl, p, sc, wide)) != HGNN_OK) return st;
    p = &wide.q;
    // incoming gradient and (for the ReLU decisions, a sign test that the rounding of the output keeps) the output
    const void *src[2] = {grad_h, p->relu ? h_out : nullptr};
    void *dst[2] = {sc + pl.c_g32, sc + pl.c_h32};
    const int64_t n[2] = {pl.total_dst * (int64_t)H, p->relu ? pl.total_dst * (int64_t)H : 0};
    if ((st = launch_convert(s, true, src, dst, n, 2)) != HGNN_OK) return st;
    grad_h = dst[0];
    h_out = dst[1];
  }
  float *dbeta = (float *)(sc + pl.c_small), *coef = dbeta + kMaxR;
  const float *beta = (const float *)(sv + pl.s_beta);
  // zero everything that is accumulated into
  GradPtrTab gt;
  std::memset(&gt, 0, sizeof(gt));
  bool any_db = false;
  {
    std::vector<float *> zp;
    std::vector<int64_t> zn;
    for (int t = 0; t < T; ++t) {
      if (!go->dw_type[t]) HGNN_FAIL(HGNN_EINVAL, "dw_type[%d] is NULL", t);
      gt.dw_root[t] = go->dw_type[t];
      gt.dbias[t] = (go->dbias && p->bias && p->bias[t]) ? go->dbias[t] : nullptr;
      any_db |= gt.dbias[t] != nullptr;
      zp.push_back(go->dw_type[t]); zn.push_back((int64_t)p->in_dim[t] * H);
      if (gt.dbias[t]) { zp.push_back(gt.dbias[t]); zn.push_back(H); }
    }
    for (int r = 0; r < R; ++r) {
      if (!go->da_src[r] || !go->da_dst[r]) HGNN_FAIL(HGNN_EINVAL, "da_src[%d] / da_dst[%d] is NULL", r, r);
      zp.push_back(go->da_src[r]); zn.push_back(H);
      zp.push_back(go->da_dst[r]); zn.push_back(H);
    }
    zp.push_back(go->dw_sem); zn.push_back((int64_t)H * kSemDimHost);
    zp.push_back(go->db_sem); zn.push_back(kSemDimHost);
    zp.push_back(go->dq_sem); zn.push_back(kSemDimHost);
    zp.push_back(dbeta); zn.push_back(2 * kMaxR);
    Probe pb(ctx, s, HGNN_K_ZERO_GRADS, layer);
    if ((st = launch_attn_zero(s, zp.data(), zn.data(), (int)zp.size())) != HGNN_OK) return st;
  }
  // activation / bias backward
  const void *gp = grad_h;
  if (pl.total_dst > 0 && (p->relu || any_db)) {
    Probe pb(ctx, s, HGNN_K_RELU_BIAS_BWD, layer);
    if ((st = launch_relu_bias_bwd(s, HGNN_F32, pl.tt, H, H, p->relu, grad_h, h_out, sc + pl.c_gp, gt)) != HGNN_OK) return st;
    if (p->relu) gp = sc + pl.c_gp;   // without an activation the pass only sums the bias gradient
  }
  // semantic-attention fusion backward
  if ((st = launch_attn_dbeta(s, HGNN_F32, pl.dev, pl.tt, pl.rt, H, H, gp, sv + pl.s_m, dbeta)) != HGNN_OK) return st;
  if ((st = launch_attn_beta(s, pl.tt, pl.rt, nullptr, const_cast<float *>(beta), dbeta, coef, 1)) != HGNN_OK) return st;
  if ((st = launch_attn_du(s, HGNN_F32, pl.dev, pl.rt, sv + pl.s_t, p->q_sem, coef, sc + pl.c_du, go->dq_sem, go->db_sem)) != HGNN_OK) return st;
  {
    Probe pb(ctx, s, HGNN_K_GEMM_DW, layer);
    if ((st = launch_attn_dws(s, HGNN_F32, pl.rows, H, sv + pl.s_m, sc + pl.c_du, go->dw_sem)) != HGNN_OK) return st;
  }
  {
    Probe pb(ctx, s, HGNN_K_GEMM_DA, layer);
    if ((st = launch_attn_dm(s, HGNN_F32, pl.dev, pl.tt, pl.rt, H, H, sc + pl.c_du, p->w_sem, gp, beta, sc + pl.c_dm)) != HGNN_OK) return st;
  }
  // aggregation backward
  {
    Probe pb(ctx, s, HGNN_K_SPMM_BWD, layer);
    if ((st = launch_attn_agg_bwd(s, HGNN_F32, pl.dev, pl.tt, pl.rt, p->a_src, p->a_dst, go->da_src, go->da_dst, H, pl.heads, sv + pl.s_z,
                                  sv + pl.s_m, sc + pl.c_dm, (const float *)(sv + pl.s_mx), (const float *)(sv + pl.s_ls),
                                  (float *)(sc + pl.c_alpha), (float *)(sc + pl.c_ds), (float *)(sc + pl.c_dsum), sc + pl.c_dz,
                                  (float *)(sc + pl.c_partial))) != HGNN_OK) return st;
  }
  // projection backward on the layer GEMMs: every type is a "root" segment over ALL its source rows
  TypeTab tt2 = pl.tt;
  RelTab rt2 = pl.rt;
  for (int t = 0; t < T; ++t) {
    tt2.n_dst[t] = (int32_t)L.n_src[t];
    tt2.out_row_off[t + 1] = pl.tt.row_off[t + 1];
    rt2.zroot_off4[t] = (uint32_t)(pl.tt.elem_off[t] / 4);
  }
  tt2.out_row_off[0] = 0;
  if (pl.src_rows > 0) {
    DwTab dt;
    std::memset(&dt, 0, sizeof(dt));
    int ne = 0;
    for (int t = 0; t < T; ++t) {
      dt.first[t] = (uint16_t)ne;
      int u = 0;
      if (L.n_src[t] > 0) {
        dt.seg[ne] = (uint8_t)(R + t);
        dt.u_off[ne] = 0;
        u = (p->in_dim[t] + 127) / 128;
        ++ne;
      }
      dt.u_total[t] = (uint16_t)u;
    }
    dt.first[T] = (uint16_t)ne;
    const int tiles_h = (H + 127) / 128;
    int split_rows = 4096;
    for (;;) {
      int64_t tiles = 0;
      for (int t = 0; t < T; ++t) tiles += (int64_t)dt.u_total[t] * tiles_h * ((L.n_src[t] + split_rows - 1) / split_rows);
      if (tiles >= 320 || split_rows <= 1024) break;
      split_rows /= 2;
    }
    for (int t = 0; t < T; ++t)
      dt.tile_off[t + 1] = dt.tile_off[t] + dt.u_total[t] * tiles_h * (int)((L.n_src[t] + split_rows - 1) / split_rows);
    // bf16 storage: both GEMMs run on the bf16 MFMA kernels, on the caller's own x and weights and on dZ rounded to
    // bf16 (a relative 2^-9 per element of a gradient that is summed over the rows; no decision hangs on it), and the
    // input gradient leaves in the storage type directly
    const void *dzp = sc + pl.c_dz;
    const int gdt = pl.widen ? HGNN_BF16 : HGNN_F32;
    if (pl.widen) {
      const void *src = dzp;
      void *dst = sc + pl.c_dz16;
      const int64_t n = pl.src_rows * (int64_t)H;
      if ((st = launch_convert(s, false, &src, &dst, &n, 1)) != HGNN_OK) return st;
      dzp = dst;
    }
    if ((st = launch_gemm_dw(s, gdt, pl.dev, tt2, rt2, gt, dt, split_rows, H, H, true, x, nullptr, dzp)) != HGNN_OK) return st;
    if (grad_x) {
      SegTab tl;
      std::memset(&tl, 0, sizeof(tl));
      tl.num_segs = R + T;
      for (int sgi = 0; sgi < R + T; ++sgi) {
        int cnt = 0;
        if (sgi >= R) {
          const int t = sgi - R;
          const bool want = !p->input_grad || p->input_grad[t];
          if (want && L.n_src[t] > 0) cnt = (int)((L.n_src[t] + 127) / 128) * ((p->in_dim[t] + 127) / 128);
        }
        tl.tile_off[sgi + 1] = tl.tile_off[sgi] + cnt;
      }
      if ((st = launch_gemm_da(s, gdt, pl.dev, tt2, rt2, pl.pt, tl, H, true, dzp, grad_x)) != HGNN_OK) return st;
    }
  }
  return HGNN_OK;
}

// A forward launch of fewer 128x128 tiles than this leaves compute units without a block (two fit on each of
// the 256): it uses 64x64 tiles instead -- four times as many, four resident per compute unit.  (Measured on
// the headline's second layer, 96 tiles of 40 K-steps: 42 -> 33 us.  The backward GEMMs have short reductions
// and gain nothing from smaller tiles.)
constexpr int kSmallTileLimit = 512;

// Tile table of the forward GEMM; returns the tile edge (128 or 64).
static int fwd_tiles(const Plan &pl, SegTab &tl, bool allow_small) {
  const int T = pl.tt.num_types;
  for (int mn = 128;; mn = 64) {
    std::memset(&tl, 0, sizeof(tl));
    const int tn = (pl.H + mn - 1) / mn;
    for (int t = 0; t < T; ++t) tl.tile_off[t + 1] = tl.tile_off[t] + ((pl.tt.n_dst[t] + mn - 1) / mn) * tn;
    tl.num_segs = T;
    if (mn == 64 || !allow_small || tl.tile_off[T] >= kSmallTileLimit) return mn;
  }
}

}  // namespace hgnn

using namespace hgnn;

extern "C" {

const char *hgnn_last_error(void) { return hgnn::get_error(); }

hgnn_status hgnn_create(hgnn_ctx **out, const hgnn_schema *s, int device, int host_threads, int concurrent_builds) {
  if (!out || !s || !s->rel_src_type || !s->rel_dst_type) HGNN_FAIL(HGNN_EINVAL, "NULL argument");
  *out = nullptr;
  if (s->num_types < 1 || s->num_types > kMaxT) HGNN_FAIL(HGNN_EINVAL, "num_types %d outside [1,%d]", s->num_types, kMaxT);
  if (s->num_rels < 1 || s->num_rels > kMaxR) HGNN_FAIL(HGNN_EINVAL, "num_rels %d outside [1,%d]", s->num_rels, kMaxR);
  if (s->dtype != HGNN_F32 && s->dtype != HGNN_BF16) HGNN_FAIL(HGNN_EINVAL, "unknown dtype %d", s->dtype);
  for (int r = 0; r < s->num_rels; ++r)
    if (s->rel_src_type[r] < 0 || s->rel_src_type[r] >= s->num_types || s->rel_dst_type[r] < 0 ||
        s->rel_dst_type[r] >= s->num_types)
      HGNN_FAIL(HGNN_EINVAL, "relation %d has a vertex type outside [0,%d)", r, s->num_types);
  hgnn_ctx *c = new (std::nothrow) hgnn_ctx();
  if (!c) HGNN_FAIL(HGNN_ENOMEM, "out of host memory");
  c->device = device;
  c->T = s->num_types;
  c->R = s->num_rels;
  for (int r = 0; r < c->R; ++r) {
    c->rel_src[r] = s->rel_src_type[r];
    c->rel_dst[r] = s->rel_dst_type[r];
  }
  c->heads = s->heads < 1 ? 1 : s->heads;
  c->agg = s->agg;
  c->fuse = s->fuse;
  c->dtype = s->dtype;
  c->legacy_gemm = getenv("HGNN_DMA_GEMM") == nullptr;
  if (device >= 0) {
    hipError_t e = hipSetDevice(device);
    if (e == hipSuccess) e = hipStreamCreateWithFlags(&c->side, hipStreamNonBlocking);
    if (e != hipSuccess) {
      delete c;
      HGNN_FAIL(HGNN_EHIP, "device %d: %s", device, hipGetErrorString(e));
    }
    const hgnn_status sst = static_scratch_init(device);  // where this device keeps hgnn_layer_fwd_static's work area
    if (sst != HGNN_OK) {
      (void)hipStreamDestroy(c->side);
      delete c;
      return sst;
    }
  }
  int n = host_threads;
  if (n <= 0) {
    long on = sysconf(_SC_NPROCESSORS_ONLN);
    n = (int)std::min<long>(16, std::max<long>(1, on));
  }
  // Graphs are independent, so several are built at once, each by a builder with its own share
  // of the host threads.  Few builders with several threads each finish one build soonest; one
  // single-threaded builder per host thread gives the most builds per second (no barriers between
  // the phases of a build), which is what a caller that queues many mini-batches ahead wants.
  int nb = concurrent_builds > 0 ? std::min(n, concurrent_builds) : std::max(1, std::min(4, n / 4));
  for (int i = 0; i < nb; ++i) {
    Builder *b = new Builder();
    b->pool = new ThreadPool(n / nb + (i < n % nb ? 1 : 0));
    c->builders.push_back(b);
  }
  for (Builder *b : c->builders) b->th = std::thread(builder_main, c, b);
  *out = c;
  return HGNN_OK;
}

void hgnn_destroy(hgnn_ctx *c) {
  if (!c) return;
  {
    std::lock_guard<std::mutex> lk(c->qm);
    c->stop = true;
  }
  c->qcv.notify_all();
  for (Builder *b : c->builders) {
    if (b->th.joinable()) b->th.join();
    delete b->pool;
    delete b;
  }
  if (c->device >= 0) {
    (void)hipSetDevice(c->device);
    (void)hipStreamSynchronize(c->side);
  }
  for (auto &s : c->free_slabs) free_slab(c, s);
  for (auto e : c->free_events) (void)hipEventDestroy(e);
  for (auto &pr : c->probe_events) {
    (void)hipEventDestroy(pr.first);
    (void)hipEventDestroy(pr.second);
  }
  if (c->side) (void)hipStreamDestroy(c->side);
  if (c->dev_tmp) (void)hipFree(c->dev_tmp);
  if (c->dev_types8) (void)hipFree(c->dev_types8);
  delete c;
}

hgnn_status hgnn_merge_features(hgnn_ctx *ctx, void *stream, const void *const *store, const int32_t *feat_dim,
                                const int64_t *const *ids, const int64_t *n_rows, void *x_merged, int32_t *row_off,
                                int64_t *elem_off) {
  if (!ctx || !store || !feat_dim || !ids || !n_rows || !row_off || !elem_off) HGNN_FAIL(HGNN_EINVAL, "NULL argument");
  const int T = ctx->T, vec = 16 / esize(ctx->dtype);
  int64_t ro = 0, eo = 0;
  int64_t tmp_eo[kMaxT + 1];
  int32_t tmp_ro[kMaxT + 1];
  for (int t = 0; t < T; ++t) {
    if (n_rows[t] < 0) HGNN_FAIL(HGNN_EINVAL, "n_rows[%d] is negative", t);
    if (feat_dim[t] <= 0 || feat_dim[t] % vec != 0)
      HGNN_FAIL(HGNN_EINVAL, "feat_dim[%d]=%d is not a positive multiple of %d", t, feat_dim[t], vec);
    if (n_rows[t] > 0 && (!store[t] || !ids[t])) HGNN_FAIL(HGNN_EINVAL, "type %d has rows but a NULL store or id list", t);
    tmp_ro[t] = (int32_t)ro;
    tmp_eo[t] = eo;
    ro += n_rows[t];
    eo += n_rows[t] * (int64_t)feat_dim[t];
    if (ro > INT32_MAX) HGNN_FAIL(HGNN_EOVERFLOW, "more than 2^31-1 merged rows");
  }
  tmp_ro[T] = (int32_t)ro;
  tmp_eo[T] = eo;
  if (ro > 0 && !x_merged) HGNN_FAIL(HGNN_EINVAL, "x_merged is NULL");
  if (ctx->device < 0) HGNN_FAIL(HGNN_EUNSUPPORTED, "host-only context cannot run device work");
  hgnn_status st;
  {
    Probe pb(ctx, (hipStream_t)stream, HGNN_K_MERGE, -1);
    st = launch_merge((hipStream_t)stream, ctx->dtype, T, store, feat_dim, ids, n_rows, tmp_eo, x_merged);
  }
  if (st != HGNN_OK) return st;
  std::memcpy(row_off, tmp_ro, sizeof(int32_t) * (T + 1));
  std::memcpy(elem_off, tmp_eo, sizeof(int64_t) * (T + 1));
  return HGNN_OK;
}

// The two halves of the index-first baseline: offsets as hgnn_merge_features computes them, one width for all types.
static hgnn_status index_first_common(hgnn_ctx *ctx, const int32_t *feat_dim, const int64_t *n_rows, const int32_t *const *pos,
                                      int64_t *tmp_eo, int32_t *tmp_ro) {
  const int T = ctx->T, vec = 16 / esize(ctx->dtype);
  int64_t ro = 0, eo = 0;
  for (int t = 0; t < T; ++t) {
    if (n_rows[t] < 0) HGNN_FAIL(HGNN_EINVAL, "n_rows[%d] is negative", t);
    if (feat_dim[t] <= 0 || feat_dim[t] % vec != 0)
      HGNN_FAIL(HGNN_EINVAL, "feat_dim[%d]=%d is not a positive multiple of %d", t, feat_dim[t], vec);
    if (feat_dim[t] != feat_dim[0]) HGNN_FAIL(HGNN_EUNSUPPORTED, "an interleaved buffer needs one width for all types");
    if (n_rows[t] > 0 && !pos[t]) HGNN_FAIL(HGNN_EINVAL, "type %d has rows but a NULL position list", t);
    tmp_ro[t] = (int32_t)ro;
    tmp_eo[t] = eo;
    ro += n_rows[t];
    eo += n_rows[t] * (int64_t)feat_dim[t];
    if (ro > INT32_MAX) HGNN_FAIL(HGNN_EOVERFLOW, "more than 2^31-1 merged rows");
  }
  tmp_ro[T] = (int32_t)ro;
  tmp_eo[T] = eo;
  if (ctx->device < 0) HGNN_FAIL(HGNN_EUNSUPPORTED, "host-only context cannot run device work");
  return HGNN_OK;
}

hgnn_status hgnn_merge_features_index_first(hgnn_ctx *ctx, void *stream, const void *const *store, const int32_t *feat_dim,
                                            const int64_t *const *ids, const int64_t *n_rows, const int32_t *const *pos,
                                            void *x_interleaved) {
  if (!ctx || !store || !feat_dim || !ids || !n_rows || !pos) HGNN_FAIL(HGNN_EINVAL, "NULL argument");
  int64_t tmp_eo[kMaxT + 1];
  int32_t tmp_ro[kMaxT + 1];
  hgnn_status st = index_first_common(ctx, feat_dim, n_rows, pos, tmp_eo, tmp_ro);
  if (st != HGNN_OK) return st;
  for (int t = 0; t < ctx->T; ++t)
    if (n_rows[t] > 0 && (!store[t] || !ids[t])) HGNN_FAIL(HGNN_EINVAL, "type %d has rows but a NULL store or id list", t);
  if (tmp_ro[ctx->T] > 0 && !x_interleaved) HGNN_FAIL(HGNN_EINVAL, "x_interleaved is NULL");
  Probe pb(ctx, (hipStream_t)stream, HGNN_K_MERGE, -1);
  return launch_merge((hipStream_t)stream, ctx->dtype, ctx->T, store, feat_dim, ids, n_rows, tmp_eo, x_interleaved, 1, pos, nullptr);
}

hgnn_status hgnn_select_type_first(hgnn_ctx *ctx, void *stream, const void *x_interleaved, const int32_t *feat_dim,
                                   const int32_t *const *pos, const int64_t *n_rows, void *x_merged, int32_t *row_off,
                                   int64_t *elem_off) {
  if (!ctx || !feat_dim || !pos || !n_rows || !row_off || !elem_off) HGNN_FAIL(HGNN_EINVAL, "NULL argument");
  int64_t tmp_eo[kMaxT + 1];
  int32_t tmp_ro[kMaxT + 1];
  hgnn_status st = index_first_common(ctx, feat_dim, n_rows, pos, tmp_eo, tmp_ro);
  if (st != HGNN_OK) return st;
  if (tmp_ro[ctx->T] > 0 && (!x_interleaved || !x_merged)) HGNN_FAIL(HGNN_EINVAL, "NULL buffer");
  {
    Probe pb(ctx, (hipStream_t)stream, HGNN_K_MERGE, -1);
    st = launch_merge((hipStream_t)stream, ctx->dtype, ctx->T, nullptr, feat_dim, nullptr, n_rows, tmp_eo, x_merged, 2, pos, x_interleaved);
  }
  if (st != HGNN_OK) return st;
  std::memcpy(row_off, tmp_ro, sizeof(int32_t) * (ctx->T + 1));
  std::memcpy(elem_off, tmp_eo, sizeof(int64_t) * (ctx->T + 1));
  return HGNN_OK;
}

extern "C++" {
namespace hgnn {
constexpr size_t kMaxTypeRuns = 32;
void index_edge_type_runs(hgnn_ctx *ctx) {
  ctx->run_end.clear();
  ctx->run_rel.clear();
  const std::vector<uint8_t> &t = ctx->edge_types8;
  for (size_t i = 0; i < t.size(); ++i)
    if (i + 1 == t.size() || t[i + 1] != t[i]) {
      ctx->run_end.push_back((int64_t)i + 1);
      ctx->run_rel.push_back(t[i]);
      if (ctx->run_end.size() > kMaxTypeRuns) {  // not grouped by relation: the byte table it is
        ctx->run_end.clear();
        ctx->run_rel.clear();
        return;
      }
    }
  ctx->run_shift = 0;
  while ((t.size() >> ctx->run_shift) > 1024) ++ctx->run_shift;
  ctx->run_lut.assign((t.size() >> ctx->run_shift) + 1, 0);
  for (size_t b = 0, j = 0; b < ctx->run_lut.size(); ++b) {
    while (j + 1 < ctx->run_end.size() && (int64_t)(b << ctx->run_shift) >= ctx->run_end[j]) ++j;
    ctx->run_lut[b] = (uint8_t)j;
  }
}

// Validates the layers' inputs (g->L[l].in), lays the index arrays out in one block and takes a pinned/device
// block and an event from the context's pool (or allocates them).  Runs on the caller's thread for
// hgnn_build_semantic_csr and on a builder's thread for sampled mini-batches, hence the message by reference.
hgnn_status plan_graph(hgnn_ctx *ctx, hgnn_graph *g, std::string &msg) {
  const int T = ctx->T, R = ctx->R, num_layers = g->num_layers;
  g->with_perm = ctx->build_perm || ctx->agg == HGNN_AGG_ATTN;  // the attention backward walks cperm
  char buf[256];
  auto fail = [&](hgnn_status st, const char *fmt, auto... a) {
    std::snprintf(buf, sizeof(buf), fmt, a...);
    msg = buf;
    return st;
  };
  size_t o = 0;
  auto take = [&](size_t n) {
    size_t at = o;
    o += (n + 63) / 64 * 64;  // keep every array 256-byte aligned
    return at;
  };
  for (int l = 0; l < num_layers; ++l) {
    LayerHost &L = g->L[l];
    const hgnn_coo_layer &in = L.in;
    if (in.num_edges < 0 || !in.n_src || !in.n_dst) return fail(HGNN_EINVAL, "layer %d: bad edge count or NULL n_src/n_dst", l);
    if (in.num_edges > 0 && !in.edge_type && in.edge_id && !in.global_edge_type && ctx->edge_types8.empty())
      return fail(HGNN_EINVAL, "layer %d: edge_id without a global edge-type table (none given, none registered)", l);
    if (in.num_edges > 0 && (!in.edge_index || (!in.edge_type && !in.edge_id))) return fail(HGNN_EINVAL, "layer %d: NULL edge arrays", l);
    if (in.num_edges > INT32_MAX) return fail(HGNN_EOVERFLOW, "layer %d: more than 2^31-1 edges", l);
    L.edges = in.num_edges;
    int64_t src_rows = 0, rows = 0;
    for (int t = 0; t < T; ++t) {
      if (in.n_src[t] < 0 || in.n_dst[t] < 0 || in.n_dst[t] > in.n_src[t])
        return fail(HGNN_EINVAL, "layer %d: type %d has n_dst=%lld, n_src=%lld (need 0 <= n_dst <= n_src)", l, t,
                    (long long)in.n_dst[t], (long long)in.n_src[t]);
      L.n_src[t] = in.n_src[t];
      L.n_dst[t] = in.n_dst[t];
      if (in.transpose_types && !in.transpose_types[t]) L.tmask &= ~(1u << t);
      src_rows += in.n_src[t];
    }
    for (int r = 0; r < R; ++r) rows += in.n_dst[ctx->rel_dst[r]];
    if (src_rows > INT32_MAX - 1 || rows > INT32_MAX - 1) return fail(HGNN_EOVERFLOW, "layer %d: more than 2^31-2 rows", l);
    L.rows = rows;
    L.src_rows = src_rows;
    L.max_long = (int32_t)(L.edges / kLongRow + 1);
    L.max_chunks = (int32_t)(L.edges / kChunk + L.max_long + 1);
    L.o_rel_row_off = take(R + 1);
    L.o_rel_edge_off = take(R + 1);
    L.o_rowptr = take(rows + 1);
    L.o_colidx = take(L.edges);
    L.o_cptr = take(src_rows + 1);
    L.o_crow = take(L.edges);
    L.o_chunk_row = take(L.max_chunks);
    L.o_chunk_beg = take(L.max_chunks);
    L.o_long_row = take(L.max_long);
    L.o_long_chunk0 = take(L.max_long + 1);
  }
  const bool cperm_on_device = ctx->agg == HGNN_AGG_ATTN;   // the attention backward walks edges by CSR position
  if (cperm_on_device)
    for (int l = 0; l < num_layers; ++l) g->L[l].o_cperm = take(g->L[l].edges);
  if (g->job)  // a sampled mini-batch carries the global ids of its first layer's source rows (int64)
    for (int t = 0; t < T; ++t) g->o_ids[t] = take(2 * g->job->ids[t].size());
  const size_t dev_used = o;  // arrays below stay on the host (views only)
  for (int l = 0; l < num_layers; ++l) {
    g->L[l].o_perm = take(g->L[l].edges);
    if (!cperm_on_device) g->L[l].o_cperm = take(g->L[l].edges);
  }
  g->used = dev_used;
  const size_t need = std::max<size_t>(o, 64);
  // a pooled slab (with its two events) or a new one
  {
    std::lock_guard<std::mutex> lk(ctx->pm);
    for (size_t i = 0; i < ctx->free_slabs.size(); ++i)
      if (ctx->free_slabs[i].cap >= need) {
        g->slab = ctx->free_slabs[i];
        ctx->free_slabs.erase(ctx->free_slabs.begin() + i);
        break;
      }
    if (!g->slab.host && !ctx->free_slabs.empty()) {  // too small: drop one so the pool does not grow forever
      free_slab(ctx, ctx->free_slabs.back());
      ctx->free_slabs.pop_back();
    }
    if (!ctx->free_events.empty()) {
      g->ready = ctx->free_events.back();
      ctx->free_events.pop_back();
    }
  }
  if (!g->slab.host) {
    const size_t cap = need + need / 4;
    if (ctx->device >= 0) {
      (void)hipSetDevice(ctx->device);
      hipError_t e = hipHostMalloc((void **)&g->slab.host, cap * sizeof(int32_t), hipHostMallocDefault);
      if (e == hipSuccess) e = hipMalloc((void **)&g->slab.dev, cap * sizeof(int32_t));
      if (e != hipSuccess) {
        free_slab(ctx, g->slab);
        g->slab = Slab();
        return fail(HGNN_ENOMEM, "graph buffers (%zu bytes): %s", cap * sizeof(int32_t), hipGetErrorString(e));
      }
    } else {
      g->slab.host = (int32_t *)malloc(cap * sizeof(int32_t));
      if (!g->slab.host) return fail(HGNN_ENOMEM, "out of host memory (%zu bytes)", cap * sizeof(int32_t));
    }
    g->slab.cap = cap;
  }
  if (ctx->device >= 0 && !g->ready) {
    hipError_t e = hipEventCreateWithFlags(&g->ready, hipEventDisableTiming);
    if (e != hipSuccess) return fail(HGNN_EHIP, "hipEventCreate: %s", hipGetErrorString(e));
  }
  return HGNN_OK;
}
}  // namespace hgnn
}  // extern "C++"

// Hands a planned (or to-be-sampled) graph to the builders.
static void enqueue_graph(hgnn_ctx *ctx, hgnn_graph *g) {
  {
    std::lock_guard<std::mutex> lk(ctx->qm);
    ctx->queue.push_back(g);
  }
  ctx->qcv.notify_one();
}

// Gives back whatever plan_graph took and deletes the graph (error paths before the graph reaches a builder).
static void drop_graph(hgnn_ctx *ctx, hgnn_graph *g) {
  {
    std::lock_guard<std::mutex> lk(ctx->pm);
    if (g->slab.host) ctx->free_slabs.push_back(g->slab);
    if (g->ready) ctx->free_events.push_back(g->ready);
  }
  delete g;
}

hgnn_status hgnn_build_semantic_csr(hgnn_ctx *ctx, int32_t num_layers, const hgnn_coo_layer *layers, hgnn_graph **out) {
  if (!ctx || !layers || !out) HGNN_FAIL(HGNN_EINVAL, "NULL argument");
  *out = nullptr;
  if (num_layers < 1 || num_layers > kMaxLayers) HGNN_FAIL(HGNN_EINVAL, "num_layers %d outside [1,%d]", num_layers, kMaxLayers);
  hgnn_graph *g = new (std::nothrow) hgnn_graph();
  if (!g) HGNN_FAIL(HGNN_ENOMEM, "out of host memory");
  g->num_layers = num_layers;
  for (int l = 0; l < num_layers; ++l) g->L[l].in = layers[l];
  std::string msg;
  const hgnn_status st = plan_graph(ctx, g, msg);
  if (st != HGNN_OK) {
    drop_graph(ctx, g);
    HGNN_FAIL(st, "%s", msg.c_str());
  }
  enqueue_graph(ctx, g);
  *out = g;
  return HGNN_OK;
}

hgnn_status hgnn_sample_and_build(hgnn_ctx *ctx, const hgnn_sampler *sm, int32_t target_type, const int64_t *targets,
                                  int64_t num_targets, int32_t num_layers, const int32_t *fanouts, uint64_t seed,
                                  const int32_t *const *transpose_types, hgnn_graph **out) {
  if (!ctx || !sm || !fanouts || !out || num_targets < 0 || (num_targets > 0 && !targets)) HGNN_FAIL(HGNN_EINVAL, "NULL argument");
  *out = nullptr;
  if (num_layers < 1 || num_layers > kMaxLayers) HGNN_FAIL(HGNN_EINVAL, "num_layers %d outside [1,%d]", num_layers, kMaxLayers);
  if (target_type < 0 || target_type >= ctx->T) HGNN_FAIL(HGNN_EINVAL, "target_type %d outside [0,%d)", target_type, ctx->T);
  for (int h = 0; h < num_layers; ++h)
    if (fanouts[h] < 1 || fanouts[h] > 64) HGNN_FAIL(HGNN_EINVAL, "fanouts[%d]=%d outside [1,64]", h, fanouts[h]);
  for (int64_t i = 0; i < num_targets; ++i)
    if (targets[i] < 0 || targets[i] >= sm->num_nodes[target_type])
      HGNN_FAIL(HGNN_EINVAL, "targets[%lld]=%lld is not a vertex of type %d", (long long)i, (long long)targets[i], target_type);
  hgnn_graph *g = new (std::nothrow) hgnn_graph();
  if (!g) HGNN_FAIL(HGNN_ENOMEM, "out of host memory");
  g->num_layers = num_layers;
  {
    std::lock_guard<std::mutex> lk(ctx->pm);
    if (!ctx->free_jobs.empty()) {
      g->job = std::move(ctx->free_jobs.back());
      ctx->free_jobs.pop_back();
    }
  }
  if (!g->job) g->job.reset(new SampleJob());
  SampleJob &job = *g->job;
  for (int l = 0; l < kMaxLayers; ++l) job.transpose[l].clear();
  job.sampler = sm;
  job.target_type = target_type;
  job.seed = seed;
  job.targets.assign(targets, targets + num_targets);
  job.fanouts.assign(fanouts, fanouts + num_layers);
  if (transpose_types)
    for (int l = 0; l < num_layers; ++l)
      if (transpose_types[l]) job.transpose[l].assign(transpose_types[l], transpose_types[l] + ctx->T);
  enqueue_graph(ctx, g);
  *out = g;
  return HGNN_OK;
}

hgnn_status hgnn_graph_ids(hgnn_ctx *ctx, hgnn_graph *g, int64_t *n_rows, const int64_t **host_ids, const int64_t **device_ids) {
  if (!ctx || !g) HGNN_FAIL(HGNN_EINVAL, "NULL argument");
  if (!g->job) HGNN_FAIL(HGNN_EINVAL, "the graph was not made by hgnn_sample_and_build");
  {
    std::unique_lock<std::mutex> lk(g->m);
    g->cv.wait(lk, [&] { return g->sampled || g->state != 0; });
    if (!g->sampled) HGNN_FAIL((hgnn_status)g->status, "%s", g->err.c_str());
  }
  if (device_ids) {  // their place in the block is fixed by the plan that follows the sampling
    std::unique_lock<std::mutex> lk(g->m);
    g->cv.wait(lk, [&] { return g->state != 0; });
    if (g->state != 1) HGNN_FAIL((hgnn_status)g->status, "%s", g->err.c_str());
  }
  for (int t = 0; t < ctx->T; ++t) {
    const size_t n = g->job->ids[t].size();
    if (n_rows) n_rows[t] = (int64_t)n;
    if (host_ids) host_ids[t] = n ? g->job->ids[t].data() : nullptr;
    if (device_ids) device_ids[t] = (n && g->slab.dev) ? reinterpret_cast<const int64_t *>(g->slab.dev + g->o_ids[t]) : nullptr;
  }
  return HGNN_OK;
}

hgnn_status hgnn_graph_minibatch_view(hgnn_ctx *ctx, hgnn_graph *g, int32_t layer, hgnn_minibatch_view *view) {
  if (!ctx || !g || !view) HGNN_FAIL(HGNN_EINVAL, "NULL argument");
  if (!g->job) HGNN_FAIL(HGNN_EINVAL, "the graph was not made by hgnn_sample_and_build");
  if (layer < 0 || layer >= g->num_layers) HGNN_FAIL(HGNN_EINVAL, "layer %d outside [0,%d)", layer, g->num_layers);
  const hgnn_status st = hgnn_graph_wait(ctx, g);
  if (st != HGNN_OK) return st;
  std::memset(view, 0, sizeof(*view));
  for (int t = 0; t < ctx->T; ++t) {
    view->n_src[t] = g->job->n_src[layer][t];
    view->n_dst[t] = g->job->n_dst[layer][t];
  }
  view->num_edges = (int64_t)g->job->edge_id[layer].size();
  view->edge_index = g->job->edge_index[layer].data();
  view->edge_id = g->job->edge_id[layer].data();
  return HGNN_OK;
}

hgnn_status hgnn_graph_wait_stream(hgnn_ctx *ctx, hgnn_graph *g, void *stream) {
  if (!ctx || !g) HGNN_FAIL(HGNN_EINVAL, "NULL argument");
  if (ctx->device < 0) HGNN_FAIL(HGNN_EUNSUPPORTED, "host-only context cannot run device work");
  {
    std::unique_lock<std::mutex> lk(g->m);
    g->cv.wait(lk, [&] { return g->state != 0; });
    if (g->state != 1) HGNN_FAIL((hgnn_status)g->status, "%s", g->err.c_str());
  }
  HGNN_HIP(hipStreamWaitEvent((hipStream_t)stream, g->ready, 0));
  return HGNN_OK;
}

hgnn_status hgnn_set_edge_types(hgnn_ctx *ctx, const int32_t *global_edge_type, int64_t num_global_edges) {
  if (!ctx || num_global_edges < 0 || (num_global_edges > 0 && !global_edge_type)) HGNN_FAIL(HGNN_EINVAL, "NULL argument");
  std::vector<uint8_t> t((size_t)num_global_edges);
  for (int64_t i = 0; i < num_global_edges; ++i) {
    const int32_t r = global_edge_type[i];
    if (r < 0 || r >= ctx->R) HGNN_FAIL(HGNN_EINVAL, "global_edge_type[%lld]=%d outside [0,%d)", (long long)i, r, ctx->R);
    t[(size_t)i] = (uint8_t)r;
  }
  ctx->edge_types8.swap(t);
  ++ctx->types_version;
  index_edge_type_runs(ctx);
  return HGNN_OK;
}

hgnn_status hgnn_set_build_permutation(hgnn_ctx *ctx, int32_t enabled) {
  if (!ctx) HGNN_FAIL(HGNN_EINVAL, "NULL context");
  ctx->build_perm = enabled != 0;
  return HGNN_OK;
}

hgnn_status hgnn_graph_wait(hgnn_ctx *ctx, hgnn_graph *g) {
  if (!ctx || !g) HGNN_FAIL(HGNN_EINVAL, "NULL argument");
  hgnn_status st = wait_built(g);
  if (st != HGNN_OK) return st;
  if (ctx->device >= 0) HGNN_HIP(hipEventSynchronize(g->ready));
  return HGNN_OK;
}

hgnn_status hgnn_graph_host_view(hgnn_ctx *ctx, hgnn_graph *g, int32_t layer, hgnn_csr_view *v) {
  if (!ctx || !g || !v) HGNN_FAIL(HGNN_EINVAL, "NULL argument");
  if (layer < 0 || layer >= g->num_layers) HGNN_FAIL(HGNN_EINVAL, "layer %d outside [0,%d)", layer, g->num_layers);
  hgnn_status st = wait_built(g);
  if (st != HGNN_OK) return st;
  const LayerHost &L = g->L[layer];
  const int32_t *b = g->slab.host;
  v->rows = L.rows; v->edges = L.edges; v->src_rows = L.src_rows; v->transpose_edges = L.tedges;
  v->rel_row_off = b + L.o_rel_row_off; v->rel_edge_off = b + L.o_rel_edge_off;
  v->rowptr = b + L.o_rowptr; v->colidx = b + L.o_colidx; v->perm = g->with_perm ? b + L.o_perm : nullptr;
  v->cptr = b + L.o_cptr; v->crow = b + L.o_crow; v->cperm = g->with_perm ? b + L.o_cperm : nullptr;
  return HGNN_OK;
}

void hgnn_graph_release(hgnn_ctx *ctx, hgnn_graph *g) {
  if (!ctx || !g) return;
  {
    std::unique_lock<std::mutex> lk(g->m);
    g->cv.wait(lk, [&] { return g->state != 0; });
  }
  // the pinned block is rewritten by the next build: its upload must have left it
  if (ctx->device >= 0 && g->state == 1) (void)hipEventSynchronize(g->ready);
  {
    std::lock_guard<std::mutex> lk(ctx->pm);
    if (g->slab.host) ctx->free_slabs.push_back(g->slab);
    if (g->ready) ctx->free_events.push_back(g->ready);
    if (g->job && ctx->free_jobs.size() < 64) ctx->free_jobs.push_back(std::move(g->job));
  }
  delete g;
}

hgnn_status hgnn_layer_workspace_bytes(hgnn_ctx *ctx, hgnn_graph *g, int32_t layer, const hgnn_layer_params *p,
                                       size_t *saved_bytes, size_t *scratch_bytes) {
  if (ctx && ctx->agg == HGNN_AGG_ATTN) {
    AttnPlan ap;
    hgnn_status sa = make_attn_plan(ctx, g, layer, p, ap, false);
    if (sa != HGNN_OK) return sa;
    if (saved_bytes) *saved_bytes = ap.saved_bytes;
    if (scratch_bytes) *scratch_bytes = ap.scratch_bytes;
    return HGNN_OK;
  }
  Plan pl;
  hgnn_status st = make_plan(ctx, g, layer, p, pl, false);
  if (st != HGNN_OK) return st;
  if (saved_bytes) *saved_bytes = pl.saved_bytes;
  if (scratch_bytes) *scratch_bytes = pl.scratch_bytes;
  return HGNN_OK;
}

// Whether the layer's aggregation is one launch of the gather-mean kernel for a single input width (which can carry the
// weight transposes): rows to aggregate, all types one width, a row of at most 256 16-byte pieces.
static bool transposes_ride(const Plan &pl) {
  if (pl.dev.rows <= 0) return false;
  for (int t = 0; t < pl.tt.num_types; ++t)
    if (pl.tt.in_dim[t] != pl.tt.in_dim[0]) return false;
  return (int64_t)pl.tt.in_dim[0] * pl.es <= 256 * 16;
}

static hgnn_status fwd_common(hgnn_ctx *ctx, void *stream, hgnn_graph *g, int32_t layer, const hgnn_layer_params *p,
                              const void *x, void *h, void *saved, size_t saved_bytes, void *scratch, size_t scratch_bytes,
                              bool naive, int32_t *launches, void *feature_cat = nullptr, size_t feature_cat_bytes = 0,
                              bool static_area = false, const void *const *gather_store = nullptr,
                              const int64_t *const *gather_ids = nullptr) {
  Plan pl;
  hgnn_status st = make_plan(ctx, g, layer, p, pl, true);
  if (st != HGNN_OK) return st;
  if (pl.total_dst > 0 && (!x || !h)) HGNN_FAIL(HGNN_EINVAL, "x_merged or h_out is NULL");
  GatherSrc gs;
  if (gather_store) {
    // source rows are read where they live: x holds the destination rows only
    std::memset(&gs, 0, sizeof(gs));
    gs.num_types = ctx->T;
    for (int t = 0; t < ctx->T; ++t) {
      if (p->in_dim[t] != p->in_dim[0]) HGNN_FAIL(HGNN_EUNSUPPORTED, "gathering from the stores needs one input width for all types");
      gs.row_off[t + 1] = pl.tt.row_off[t + 1];
      if (g->L[layer].n_src[t] > 0 && (!gather_store[t] || !gather_ids || !gather_ids[t]))
        HGNN_FAIL(HGNN_EINVAL, "type %d has source rows but a NULL store or id list", t);
      if ((uintptr_t)gather_store[t] & 15) HGNN_FAIL(HGNN_EINVAL, "feature stores must be 16-byte aligned");
      gs.store[t] = gather_store[t];
      gs.ids[t] = gather_ids[t];
    }
    root_rows_only(pl);
  }
  if (!saved || !scratch) HGNN_FAIL(HGNN_EINVAL, "NULL work area");
  if (static_area) {
    // the forward's own part of the work area, laid out back to back: transposed weights, low-order plane
    const size_t wt_bytes = pl.off_gp - pl.off_wt, zlo_bytes = pl.scratch_bytes - pl.off_zlo;
    if (wt_bytes + zlo_bytes > scratch_bytes)
      HGNN_FAIL(HGNN_EINVAL, "layer needs %zu bytes of work area, the static one holds %zu: use hgnn_layer_fwd with a caller-provided area",
                wt_bytes + zlo_bytes, scratch_bytes);
    pl.off_wt = 0;
    pl.off_zlo = wt_bytes;
    pl.scratch_bytes = wt_bytes + zlo_bytes;
  }
  if (saved_bytes < pl.saved_bytes || scratch_bytes < pl.scratch_bytes)
    HGNN_FAIL(HGNN_EINVAL, "work areas too small: need %zu saved, %zu scratch bytes", pl.saved_bytes, pl.scratch_bytes);
  if (((uintptr_t)saved | (uintptr_t)scratch | (uintptr_t)x | (uintptr_t)h) & 15)
    HGNN_FAIL(HGNN_EINVAL, "device buffers must be 16-byte aligned");
  hipStream_t s = (hipStream_t)stream;
  HGNN_HIP(hipStreamWaitEvent(s, g->ready, 0));
  char *sc = (char *)scratch;
  void *wtb = sc + pl.off_wt;
  // bf16 storage, layer with an activation: the aggregate is kept as a pair (rounded value, remainder), so that the
  // pre-activation -- and with it the decision of every unit, which the backward pass depends on discontinuously --
  // does not carry the rounding of the aggregate to 8 significant bits
  void *zlo = (ctx->dtype == HGNN_BF16 && p->relu) ? sc + pl.off_zlo : nullptr;
  int n = 0;
  SegTab tl;
  const int tile_mn = fwd_tiles(pl, tl, !naive);
  const int R = ctx->R, T = ctx->T;
  uint32_t live[kMaxR / 32] = {0};
  {
    const int32_t *reo = g->slab.host + g->L[layer].o_rel_edge_off;
    for (int r = 0; r < R; ++r)
      if (reo[r + 1] > reo[r]) live[r >> 5] |= 1u << (r & 31);
  }
  // The weight transposes ride in the aggregation launch (as its first blocks) where that launch is the gather-mean
  // kernel for one input width; otherwise they are a launch of their own.
  TransposeJobs tj;
  make_transpose_jobs(pl.tt, pl.rt, pl.pt, pl.wt, pl.H, wtb, tj);
  const bool rides = !naive && !feature_cat && transposes_ride(pl);
  if (!rides) {
    Probe pb(ctx, s, HGNN_K_TRANSPOSE_W, layer, !static_area);
    if ((st = launch_transpose_jobs(s, ctx->dtype, tj)) != HGNN_OK) return st;
    ++n;
  }
  if (!naive) {
    if (feature_cat) {
      // Algorithm 1 in two steps (gather into FeatureCat, then reduce by destination) instead of the fused kernel
      for (int t = 0; t < T; ++t)
        if (p->in_dim[t] != p->in_dim[0]) HGNN_FAIL(HGNN_EUNSUPPORTED, "the two-step aggregation needs one input width for all types");
      const size_t need = (size_t)pl.dev.edges * p->in_dim[0] * pl.es;
      if (feature_cat_bytes < need) HGNN_FAIL(HGNN_EINVAL, "feature_cat too small: need %zu bytes", need);
      if ((uintptr_t)feature_cat & 15) HGNN_FAIL(HGNN_EINVAL, "device buffers must be 16-byte aligned");
      Probe pb(ctx, s, HGNN_K_SPMM_FWD, layer, !static_area);
      if ((st = launch_aggregate_literal(s, ctx->dtype, pl.dev, p->in_dim[0], x, feature_cat, saved, zlo)) != HGNN_OK) return st;
      n += (pl.dev.edges > 0) + (pl.dev.rows > 0);
    } else {
      if (gather_store) {
        uint64_t *gaddr = (uint64_t *)(sc + pl.off_gaddr);
        if ((st = launch_gather_addresses(s, pl.dev, gs, p->in_dim[0] * pl.es, gaddr)) != HGNN_OK) return st;
        if (pl.dev.edges > 0) ++n;
        Probe pb(ctx, s, HGNN_K_SPMM_FWD, layer);
        if (pl.dev.rows > 0) {
          if (!launch_spmm_fwd_uniform(s, ctx->dtype, pl.dev, p->in_dim[0], nullptr, saved, zlo, 0, pl.dev.rows, gaddr, rides ? &tj : nullptr))
            HGNN_FAIL(HGNN_EUNSUPPORTED, "input width %d is outside what the gather kernels cover", p->in_dim[0]);
          HGNN_HIP(hipGetLastError());
          ++n;
        }
      } else {
        Probe pb(ctx, s, HGNN_K_SPMM_FWD, layer, !static_area);
        if ((st = launch_spmm_fwd(s, ctx->dtype, pl.dev, pl.tt, pl.rt, pl.max_dim, x, saved, zlo, 0, pl.dev.rows, rides ? &tj : nullptr)) != HGNN_OK) return st;
        if (pl.dev.rows > 0) ++n;
      }
    }
    {
      Probe pb(ctx, s, HGNN_K_GEMM_FWD, layer, !static_area);
      bool done = false;
      if (ctx->dtype == HGNN_BF16 && !ctx->legacy_gemm) {
        done = launch_gemm2_fwd(s, pl.tt, pl.rt, pl.pt, pl.wt, live, pl.H, p->relu, x, saved, zlo, wtb, h, &st);
        if (done && st != HGNN_OK) return st;
      }
      if (!done && (st = launch_gemm_fwd(s, ctx->dtype, pl.dev, pl.tt, pl.rt, pl.pt, pl.wt, tl, live, pl.H, p->relu, x, saved, zlo, wtb, h, -1, nullptr, tile_mn)) != HGNN_OK) return st;
    }
    if (tl.tile_off[T] > 0) ++n;
  } else {
    // the un-merged launch structure: one aggregation and one projection launch per relation, one root
    // projection and one bias/activation launch per vertex type
    float *acc32 = (float *)(sc + pl.off_acc32);
    if ((st = launch_fill_zero(s, acc32, (size_t)pl.total_dst * pl.H * 4)) != HGNN_OK) return st;
    ++n;
    const LayerHost &L = g->L[layer];
    const int32_t *rro = g->slab.host + L.o_rel_row_off;
    for (int r = 0; r < R; ++r) {
      if (rro[r + 1] == rro[r]) continue;
      if ((st = launch_spmm_fwd(s, ctx->dtype, pl.dev, pl.tt, pl.rt, pl.max_dim, x, saved, zlo, rro[r], rro[r + 1])) != HGNN_OK) return st;
      ++n;
      SegTab one;
      std::memset(&one, 0, sizeof(one));
      one.num_segs = T;
      const int d = ctx->rel_dst[r];
      for (int t = 0; t < T; ++t)
        one.tile_off[t + 1] = one.tile_off[t] + (t == d ? tl.tile_off[t + 1] - tl.tile_off[t] : 0);
      if ((st = launch_gemm_fwd(s, ctx->dtype, pl.dev, pl.tt, pl.rt, pl.pt, pl.wt, one, live, pl.H, 0, x, saved, zlo, wtb, h, r, acc32)) != HGNN_OK) return st;
      ++n;
    }
    for (int t = 0; t < T; ++t) {
      if (pl.tt.n_dst[t] == 0) continue;
      if (p->w_root[t]) {
        SegTab one;
        std::memset(&one, 0, sizeof(one));
        one.num_segs = T;
        for (int u = 0; u < T; ++u)
          one.tile_off[u + 1] = one.tile_off[u] + (u == t ? tl.tile_off[u + 1] - tl.tile_off[u] : 0);
        if ((st = launch_gemm_fwd(s, ctx->dtype, pl.dev, pl.tt, pl.rt, pl.pt, pl.wt, one, live, pl.H, 0, x, saved, zlo, wtb, h, R + t, acc32)) != HGNN_OK) return st;
        ++n;
      }
      if ((st = launch_bias_act(s, ctx->dtype, pl.tt, pl.pt, pl.H, p->relu, t, acc32, h)) != HGNN_OK) return st;
      ++n;
    }
  }
  if (launches) *launches = n;
  return HGNN_OK;
}

extern "C++" {
namespace hgnn {
hgnn_status layer_fwd_static_area(hgnn_ctx *ctx, void *stream, hgnn_graph *g, int32_t layer, const hgnn_layer_params *p,
                                  const void *x, void *h, void *saved, size_t saved_bytes, void *area, size_t area_bytes) {
  if (ctx->agg == HGNN_AGG_ATTN) HGNN_FAIL(HGNN_EUNSUPPORTED, "hgnn_layer_fwd_static covers the mean-aggregation layer only");
  return fwd_common(ctx, stream, g, layer, p, x, h, saved, saved_bytes, area, area_bytes, false, nullptr, nullptr, 0, true);
}
}  // namespace hgnn
}  // extern "C++"

hgnn_status hgnn_layer_fwd(hgnn_ctx *ctx, void *stream, hgnn_graph *g, int32_t layer, const hgnn_layer_params *p,
                           const void *x_merged, void *h_out, void *saved, size_t saved_bytes, void *scratch,
                           size_t scratch_bytes) {
  if (ctx && ctx->agg == HGNN_AGG_ATTN)
    return attn_fwd(ctx, stream, g, layer, p, x_merged, h_out, saved, saved_bytes, scratch, scratch_bytes);
  return fwd_common(ctx, stream, g, layer, p, x_merged, h_out, saved, saved_bytes, scratch, scratch_bytes, false, nullptr);
}

hgnn_status hgnn_layer_fwd_gather(hgnn_ctx *ctx, void *stream, hgnn_graph *g, int32_t layer, const hgnn_layer_params *p,
                                  const void *const *store, const int64_t *const *ids, const void *x_dst, void *h_out,
                                  void *saved, size_t saved_bytes, void *scratch, size_t scratch_bytes) {
  if (!ctx || !store || !ids) HGNN_FAIL(HGNN_EINVAL, "NULL argument");
  if (ctx->agg == HGNN_AGG_ATTN) HGNN_FAIL(HGNN_EUNSUPPORTED, "hgnn_layer_fwd_gather covers the mean-aggregation layer only");
  return fwd_common(ctx, stream, g, layer, p, x_dst, h_out, saved, saved_bytes, scratch, scratch_bytes, false, nullptr, nullptr, 0,
                    false, store, ids);
}

hgnn_status hgnn_layer_fwd_naive(hgnn_ctx *ctx, void *stream, hgnn_graph *g, int32_t layer, const hgnn_layer_params *p,
                                 const void *x_merged, void *h_out, void *saved, size_t saved_bytes, void *scratch,
                                 size_t scratch_bytes, int32_t *launches) {
  return fwd_common(ctx, stream, g, layer, p, x_merged, h_out, saved, saved_bytes, scratch, scratch_bytes, true, launches);
}

hgnn_status hgnn_layer_fwd_two_step(hgnn_ctx *ctx, void *stream, hgnn_graph *g, int32_t layer, const hgnn_layer_params *p,
                                    const void *x_merged, void *h_out, void *saved, size_t saved_bytes, void *scratch,
                                    size_t scratch_bytes, void *feature_cat, size_t feature_cat_bytes, int32_t *launches) {
  if (!feature_cat) HGNN_FAIL(HGNN_EINVAL, "feature_cat is NULL");
  return fwd_common(ctx, stream, g, layer, p, x_merged, h_out, saved, saved_bytes, scratch, scratch_bytes, false, launches,
                    feature_cat, feature_cat_bytes);
}

static void seg_tiles_da(hgnn_ctx *ctx, const Plan &pl, const hgnn_layer_params *p, const int32_t *rel_edge_off, SegTab &tl) {
  const int R = ctx->R, T = ctx->T;
  std::memset(&tl, 0, sizeof(tl));
  tl.num_segs = R + T;
  for (int sgi = 0; sgi < R + T; ++sgi) {
    int cnt = 0;
    const bool is_rel = sgi < R;
    const int d = is_rel ? ctx->rel_dst[sgi] : sgi - R;
    const int F = pl.tt.in_dim[is_rel ? ctx->rel_src[sgi] : d];
    bool live = is_rel ? rel_edge_off[sgi + 1] > rel_edge_off[sgi] : p->w_root[d] != nullptr;
    if (p->input_grad && !p->input_grad[is_rel ? ctx->rel_src[sgi] : d]) live = false;  // nobody reads this dZ
    if (live && pl.tt.n_dst[d] > 0) cnt = ((pl.tt.n_dst[d] + 127) / 128) * ((F + 127) / 128);
    tl.tile_off[sgi + 1] = tl.tile_off[sgi] + cnt;
  }
}

// The same tiles grouped for the merged backward launch: per destination type, per 128-row block, the column blocks
// of every live segment whose input gradient is wanted.
static void grouped_tiles_da(hgnn_ctx *ctx, const Plan &pl, const SegTab &by_seg, DwTab &tl) {
  const int R = ctx->R, T = ctx->T;
  std::memset(&tl, 0, sizeof(tl));
  int ne = 0;
  for (int d = 0; d < T; ++d) {
    tl.first[d] = (uint16_t)ne;
    int u = 0;
    for (int sgi = 0; sgi < R + T; ++sgi) {
      const bool is_rel = sgi < R;
      if ((is_rel ? ctx->rel_dst[sgi] : sgi - R) != d || by_seg.tile_off[sgi + 1] == by_seg.tile_off[sgi]) continue;
      tl.seg[ne] = (uint8_t)sgi;
      tl.u_off[ne] = (uint16_t)u;
      u += (pl.tt.in_dim[is_rel ? ctx->rel_src[sgi] : d] + 127) / 128;
      ++ne;
    }
    tl.u_total[d] = (uint16_t)u;
    tl.tile_off[d + 1] = tl.tile_off[d] + u * ((pl.tt.n_dst[d] + 127) / 128);
  }
  tl.first[T] = (uint16_t)ne;
}

static hgnn_status bwd_common(hgnn_ctx *ctx, void *stream, hgnn_graph *g, int32_t layer, const hgnn_layer_params *p,
                              const void *x_merged, const void *h_out, const void *saved, const void *grad_h,
                              void *grad_x_merged, const hgnn_layer_grads *go, void *scratch, size_t scratch_bytes, bool naive,
                              int32_t *launches, bool x_dst_only = false) {
  if (launches) *launches = 0;
  if (ctx && ctx->agg == HGNN_AGG_ATTN) {
    if (naive) HGNN_FAIL(HGNN_EUNSUPPORTED, "the per-relation launch loop exists for the mean-aggregation layer only");
    return attn_bwd(ctx, stream, g, layer, p, x_merged, h_out, saved, grad_h, grad_x_merged, go, scratch, scratch_bytes);
  }
  Plan pl;
  hgnn_status st = make_plan(ctx, g, layer, p, pl, true);
  if (st != HGNN_OK) return st;
  if (x_dst_only) root_rows_only(pl);
  if (!saved || !scratch || !go) HGNN_FAIL(HGNN_EINVAL, "NULL work area or gradient table");
  if (pl.total_dst > 0 && (!x_merged || !grad_h || (p->relu && !h_out))) HGNN_FAIL(HGNN_EINVAL, "NULL input");
  if (scratch_bytes < pl.scratch_bytes) HGNN_FAIL(HGNN_EINVAL, "scratch too small: need %zu bytes", pl.scratch_bytes);
  if (((uintptr_t)saved | (uintptr_t)scratch | (uintptr_t)x_merged | (uintptr_t)grad_h | (uintptr_t)grad_x_merged |
       (uintptr_t)h_out) & 15)
    HGNN_FAIL(HGNN_EINVAL, "device buffers must be 16-byte aligned");
  const int R = ctx->R, T = ctx->T;
  GradPtrTab gt;
  std::memset(&gt, 0, sizeof(gt));
  bool any_dw = false, any_db = false;
  for (int r = 0; r < R; ++r) {
    gt.dw_rel[r] = go->dw_rel ? go->dw_rel[r] : nullptr;
    any_dw |= gt.dw_rel[r] != nullptr;
  }
  for (int t = 0; t < T; ++t) {
    gt.dw_root[t] = (go->dw_root && p->w_root[t]) ? go->dw_root[t] : nullptr;
    gt.dbias[t] = (go->dbias && p->bias && p->bias[t]) ? go->dbias[t] : nullptr;
    any_dw |= gt.dw_root[t] != nullptr;
    any_db |= gt.dbias[t] != nullptr;
  }
  hipStream_t s = (hipStream_t)stream;
  HGNN_HIP(hipStreamWaitEvent(s, g->ready, 0));
  char *sc = (char *)scratch;
  const LayerHost &L = g->L[layer];
  const int32_t *reo = g->slab.host + L.o_rel_edge_off;
  if ((any_dw || any_db) && pl.total_dst == 0) {  // nothing flows back: the gradients are zero
    Probe pb(ctx, s, HGNN_K_ZERO_GRADS, layer);
    return launch_zero_grads(s, pl.tt, pl.rt, gt, pl.H);
  }
  // The GEMMs want 16-byte aligned rows.  When H is not a multiple of 16 bytes (or a weight pointer is not
  // aligned) they run on zero-padded copies: G' gets leading dimension Hp in the scratch area (written by the
  // ReLU/bias pass, which then always runs) and so do the weights.
  const int vec = 16 / pl.es;
  const int Hp = (pl.H + vec - 1) / vec * vec;
  bool pad = Hp != pl.H;
  for (int r = 0; r < R; ++r) pad |= ((uintptr_t)p->w_rel[r] & 15) != 0;
  for (int t = 0; t < T; ++t) pad |= p->w_root[t] && ((uintptr_t)p->w_root[t] & 15) != 0;
  int ldg = pl.H;
  PtrTab wpt = pl.pt;
  WtTab wo;
  std::memset(&wo, 0, sizeof(wo));
  void *wpad = nullptr;
  if (pad && pl.total_dst > 0) {
    ldg = Hp;
    size_t w = 0;
    char *wp = sc + pl.off_wt;
    for (int r = 0; r < R; ++r) {
      wo.rel4[r] = (uint32_t)(w / 4);
      wpt.w_rel[r] = wp + w * pl.es;
      w += (size_t)p->in_dim[ctx->rel_src[r]] * Hp;
    }
    for (int t = 0; t < T; ++t) {
      wo.root4[t] = (uint32_t)(w / 4);
      if (p->w_root[t]) {
        wpt.w_root[t] = wp + w * pl.es;
        w += (size_t)p->in_dim[t] * Hp;
      }
    }
    if (grad_x_merged) wpad = wp;
  }
  if (naive) {
    // The un-merged launch structure: the same kernels, launched once per vertex type (ReLU mask / bias gradient,
    // transposed aggregation) and once per relation or root term (weight gradient, input gradient), after one
    // launch that zeroes the gradients (and one that pads the weights where the width asks for it).
    int n = 0;
    void *gpw = sc + pl.off_gp;
    const void *gpn = grad_h;
    if (wpad) {
      if ((st = launch_pad_weights(s, ctx->dtype, pl.tt, pl.rt, pl.pt, wo, pl.H, ldg, wpad)) != HGNN_OK) return st;
      ++n;
    }
    if (any_dw || any_db) {
      if ((st = launch_zero_grads(s, pl.tt, pl.rt, gt, pl.H)) != HGNN_OK) return st;
      ++n;
    }
    if (pl.total_dst > 0 && (p->relu || any_db || ldg != pl.H)) {
      for (int t = 0; t < T; ++t) {
        if (pl.tt.n_dst[t] == 0) continue;
        TypeTab one = pl.tt;
        for (int u = 0; u < T; ++u)
          if (u != t) one.n_dst[u] = 0;
        if ((st = launch_relu_bias_bwd(s, ctx->dtype, one, pl.H, ldg, p->relu, grad_h, h_out, gpw, gt)) != HGNN_OK) return st;
        ++n;
      }
      if (p->relu || ldg != pl.H) gpn = gpw;
    }
    const bool fastn = (ldg % (16 / pl.es)) == 0;
    const bool want_dxn = grad_x_merged && pl.dev.src_rows > 0;
    if (want_dxn)
      for (int t = 0; t < T; ++t)
        if ((!p->input_grad || p->input_grad[t]) && !((L.tmask >> t) & 1u) && L.n_src[t] > 0)
          HGNN_FAIL(HGNN_EINVAL, "input gradient of type %d asked for, but the graph was built without its transpose entries", t);
    void *dzn = sc + pl.off_dz;
    const int tiles_hn = (pl.H + 127) / 128;
    for (int sgi = 0; sgi < R + T && pl.total_dst > 0; ++sgi) {
      const bool is_rel = sgi < R;
      const int d = is_rel ? ctx->rel_dst[sgi] : sgi - R;
      const int F = pl.tt.in_dim[is_rel ? ctx->rel_src[sgi] : d];
      if (pl.tt.n_dst[d] == 0) continue;
      const bool live = is_rel ? reo[sgi + 1] > reo[sgi] : p->w_root[d] != nullptr;
      if (!live) continue;
      if (is_rel ? gt.dw_rel[sgi] != nullptr : gt.dw_root[d] != nullptr) {  // weight gradient of this segment
        DwTab one;
        std::memset(&one, 0, sizeof(one));
        for (int u = 0; u <= T; ++u) one.first[u] = (uint16_t)(u > d ? 1 : 0);
        one.seg[0] = (uint8_t)sgi;
        one.u_off[0] = 0;
        one.u_total[d] = (uint16_t)((F + 127) / 128);
        const int split_rows = 2048;
        const int cnt = one.u_total[d] * tiles_hn * ((pl.tt.n_dst[d] + split_rows - 1) / split_rows);
        for (int u = d; u < T; ++u) one.tile_off[u + 1] = cnt;
        if ((st = launch_gemm_dw(s, ctx->dtype, pl.dev, pl.tt, pl.rt, gt, one, split_rows, pl.H, ldg, fastn, x_merged, saved, gpn)) != HGNN_OK) return st;
        ++n;
      }
      if (want_dxn && (!p->input_grad || p->input_grad[is_rel ? ctx->rel_src[sgi] : d])) {  // input gradient of this segment
        SegTab one;
        std::memset(&one, 0, sizeof(one));
        one.num_segs = R + T;
        const int cnt = ((pl.tt.n_dst[d] + 127) / 128) * ((F + 127) / 128);
        for (int u = sgi; u < R + T; ++u) one.tile_off[u + 1] = cnt;
        if ((st = launch_gemm_da(s, ctx->dtype, pl.dev, pl.tt, pl.rt, wpt, one, ldg, fastn, gpn, dzn)) != HGNN_OK) return st;
        ++n;
      }
    }
    if (want_dxn) {
      for (int t = 0; t < T; ++t) {
        if ((p->input_grad && !p->input_grad[t]) || L.n_src[t] == 0) continue;
        if ((st = launch_spmm_bwd(s, ctx->dtype, pl.dev, pl.tt, pl.rt, pl.pt, pl.max_dim, 1u << t, dzn, grad_x_merged, (float *)(sc + pl.off_partial))) != HGNN_OK) return st;
        n += 1 + (pl.dev.n_long > 0);
      }
    }
    if (launches) *launches = n;
    return HGNN_OK;
  }
  // One launch: the row pass over G (ReLU mask, padded copy, column sums for the bias gradient as partial sums
  // per block), zeroing of the weight gradients, the padded weights.  The partial sums are added up by a few
  // blocks of the backward GEMM launch below, or by a launch of their own when that one does not run.
  const void *gp = grad_h;
  const bool row_pass = pl.total_dst > 0 && (p->relu || any_db || ldg != pl.H);
  float *bpart = any_db ? (float *)(sc + pl.off_bpart) : nullptr;
  int rpb = 0;  // rows of G per row of bpart: set by the launcher
  if (pl.total_dst > 0) {
    void *gpw = sc + pl.off_gp;
    Probe pb(ctx, s, HGNN_K_RELU_BIAS_BWD, layer);
    if ((st = launch_bwd_prep(s, ctx->dtype, pl.tt, pl.rt, pl.pt, wo, gt, pl.H, ldg, p->relu, row_pass, any_dw, grad_h, h_out, gpw,
                              bpart, pl.bpart_rows, wpad, &rpb)) != HGNN_OK) return st;
    if (p->relu || ldg != pl.H) gp = gpw;
  }
  const bool fast = (ldg % vec) == 0;
  const bool want_dx = grad_x_merged && pl.dev.src_rows > 0;
  if (want_dx)
    for (int t = 0; t < T; ++t)
      if ((!p->input_grad || p->input_grad[t]) && !((L.tmask >> t) & 1u) && L.n_src[t] > 0)
        HGNN_FAIL(HGNN_EINVAL, "input gradient of type %d asked for, but the graph was built without its transpose entries", t);
  SegTab da_tl;
  if (want_dx) seg_tiles_da(ctx, pl, p, reo, da_tl);
  void *dz = sc + pl.off_dz;
  bool da_done = false;
  if (any_dw && pl.total_dst > 0) {
    // Work list: per destination type its live segments (relations with edges, then the root) and the 128-row
    // blocks of their weight gradients.  The reduction is split over destination rows so that the launch has
    // about two blocks per CU, but not into slices under 2048 rows: every extra split costs a tile's worth of
    // atomic adds, which outweigh the shorter reduction below that (in the merged launch, whose input-gradient
    // tiles fill the chip anyway: 2048 beat 1024, 1536, 3072 and 4096 by 5 to 20 us per step on the headline).
    DwTab tl;
    std::memset(&tl, 0, sizeof(tl));
    int ne = 0;
    for (int d = 0; d < T; ++d) {
      tl.first[d] = (uint16_t)ne;
      int u = 0;
      if (pl.tt.n_dst[d] > 0)
        for (int sgi = 0; sgi < R + T; ++sgi) {
          const bool is_rel = sgi < R;
          if (is_rel ? (ctx->rel_dst[sgi] != d || reo[sgi + 1] == reo[sgi] || !gt.dw_rel[sgi]) : (sgi - R != d || !gt.dw_root[d])) continue;
          tl.seg[ne] = (uint8_t)sgi;
          tl.u_off[ne] = (uint16_t)u;
          u += (pl.tt.in_dim[is_rel ? ctx->rel_src[sgi] : d] + 127) / 128;
          ++ne;
        }
      tl.u_total[d] = (uint16_t)u;
    }
    tl.first[T] = (uint16_t)ne;
    const int tiles_h = (pl.H + 127) / 128;
    int split_rows = 4096;
    for (;;) {
      int64_t tiles = 0;
      for (int d = 0; d < T; ++d) tiles += (int64_t)tl.u_total[d] * tiles_h * ((pl.tt.n_dst[d] + split_rows - 1) / split_rows);
      if (tiles >= 320 || split_rows <= 2048) break;
      split_rows /= 2;
    }
    for (int d = 0; d < T; ++d)
      tl.tile_off[d + 1] = tl.tile_off[d] + tl.u_total[d] * tiles_h * ((pl.tt.n_dst[d] + split_rows - 1) / split_rows);
    Probe pb(ctx, s, HGNN_K_GEMM_DW, layer);
    if (want_dx && da_tl.tile_off[da_tl.num_segs] > 0 && tl.tile_off[T] > 0) {
      // both backward GEMMs read G' and are independent of each other: one launch
      DwTab da_grouped;
      grouped_tiles_da(ctx, pl, da_tl, da_grouped);
      if ((st = launch_gemm_bwd(s, ctx->dtype, pl.dev, pl.tt, pl.rt, wpt, da_grouped, gt, tl, split_rows, pl.H, ldg, fast, x_merged,
                                saved, gp, dz, bpart, rpb)) != HGNN_OK) return st;
      da_done = true;
      bpart = nullptr;
    } else if ((st = launch_gemm_dw(s, ctx->dtype, pl.dev, pl.tt, pl.rt, gt, tl, split_rows, pl.H, ldg, fast, x_merged, saved, gp)) != HGNN_OK) {
      return st;
    }
  }
  if (bpart && (st = launch_bias_reduce(s, pl.tt, gt, pl.H, rpb, bpart)) != HGNN_OK) return st;
  if (want_dx) {
    if (!da_done) {
      Probe pb(ctx, s, HGNN_K_GEMM_DA, layer);
      if ((st = launch_gemm_da(s, ctx->dtype, pl.dev, pl.tt, pl.rt, wpt, da_tl, ldg, fast, gp, dz)) != HGNN_OK) return st;
    }
    Probe pb(ctx, s, HGNN_K_SPMM_BWD, layer);
    uint32_t want = 0;
    for (int t = 0; t < T; ++t)
      if (!p->input_grad || p->input_grad[t]) want |= 1u << t;
    if ((st = launch_spmm_bwd(s, ctx->dtype, pl.dev, pl.tt, pl.rt, pl.pt, pl.max_dim, want, dz, grad_x_merged, (float *)(sc + pl.off_partial))) != HGNN_OK) return st;
  }
  return HGNN_OK;
}

hgnn_status hgnn_layer_bwd(hgnn_ctx *ctx, void *stream, hgnn_graph *g, int32_t layer, const hgnn_layer_params *p,
                           const void *x_merged, const void *h_out, const void *saved, const void *grad_h,
                           void *grad_x_merged, const hgnn_layer_grads *go, void *scratch, size_t scratch_bytes) {
  return bwd_common(ctx, stream, g, layer, p, x_merged, h_out, saved, grad_h, grad_x_merged, go, scratch, scratch_bytes, false, nullptr);
}

hgnn_status hgnn_layer_bwd_gather(hgnn_ctx *ctx, void *stream, hgnn_graph *g, int32_t layer, const hgnn_layer_params *p,
                                  const void *x_dst, const void *h_out, const void *saved, const void *grad_h,
                                  void *grad_x_merged, const hgnn_layer_grads *go, void *scratch, size_t scratch_bytes) {
  if (ctx && ctx->agg == HGNN_AGG_ATTN) HGNN_FAIL(HGNN_EUNSUPPORTED, "hgnn_layer_bwd_gather covers the mean-aggregation layer only");
  return bwd_common(ctx, stream, g, layer, p, x_dst, h_out, saved, grad_h, grad_x_merged, go, scratch, scratch_bytes, false, nullptr, true);
}

hgnn_status hgnn_layer_bwd_naive(hgnn_ctx *ctx, void *stream, hgnn_graph *g, int32_t layer, const hgnn_layer_params *p,
                                 const void *x_merged, const void *h_out, const void *saved, const void *grad_h,
                                 void *grad_x_merged, const hgnn_layer_grads *go, void *scratch, size_t scratch_bytes,
                                 int32_t *launches) {
  return bwd_common(ctx, stream, g, layer, p, x_merged, h_out, saved, grad_h, grad_x_merged, go, scratch, scratch_bytes, true, launches);
}

hgnn_status hgnn_layer_launch_count(hgnn_ctx *ctx, hgnn_graph *g, int32_t layer, const hgnn_layer_params *p,
                                    int32_t *fwd_launches, int32_t *bwd_launches) {
  if (ctx && ctx->agg == HGNN_AGG_ATTN) {
    AttnPlan ap;
    hgnn_status sa = make_attn_plan(ctx, g, layer, p, ap, true);
    if (sa != HGNN_OK) return sa;
    // forward: projection, aggregation, zero scores, semantic scores, relation softmax, fusion
    if (fwd_launches) *fwd_launches = 6;
    // backward: zero, (activation/bias), relation dots, relation softmax, du, dW_s, dm, row pass, transpose pass, dW_t, dX
    if (bwd_launches) *bwd_launches = 10 + ((p->relu || p->bias) ? 1 : 0);
    return HGNN_OK;
  }
  Plan pl;
  hgnn_status st = make_plan(ctx, g, layer, p, pl, true);
  if (st != HGNN_OK) return st;
  if (fwd_launches) *fwd_launches = (transposes_ride(pl) ? 0 : 1) + (pl.dev.rows > 0) + (pl.total_dst > 0);
  if (bwd_launches) {
    // zero grads + ReLU mask + bias partial sums (one launch), dW and dA GEMMs + bias sums (one launch), transposed
    // aggregation (+ long-row pass); without destination rows only the zeroing
    *bwd_launches = pl.total_dst > 0 ? 2 + (pl.dev.src_rows > 0 ? 1 + (pl.dev.n_long > 0) : 0) : 1;
  }
  return HGNN_OK;
}

hgnn_status hgnn_softmax_xent(hgnn_ctx *ctx, void *stream, const void *logits, const int64_t *labels, int64_t rows,
                              int32_t classes, float *loss, void *grad_logits) {
  if (!ctx || !loss) HGNN_FAIL(HGNN_EINVAL, "NULL argument");
  if (rows < 0 || classes < 1) HGNN_FAIL(HGNN_EINVAL, "bad shape %lld x %d", (long long)rows, classes);
  if (rows > 0 && (!logits || !labels || !grad_logits)) HGNN_FAIL(HGNN_EINVAL, "NULL argument");
  if (ctx->device < 0) HGNN_FAIL(HGNN_EUNSUPPORTED, "host-only context cannot run device work");
  Probe pb(ctx, (hipStream_t)stream, HGNN_K_XENT, -1);
  return launch_xent((hipStream_t)stream, ctx->dtype, logits, labels, rows, classes, loss, grad_logits);
}

static hgnn_status check_adam(const hgnn_adam_params *hp, double &c1, double &c2) {
  if (!hp) HGNN_FAIL(HGNN_EINVAL, "NULL argument");
  if (hp->step < 1 || !(hp->beta1 >= 0.f && hp->beta1 < 1.f) || !(hp->beta2 >= 0.f && hp->beta2 < 1.f) || !(hp->eps >= 0.f))
    HGNN_FAIL(HGNN_EINVAL, "Adam needs step >= 1, beta1 and beta2 in [0,1), eps >= 0");
  c1 = 1.0 / (1.0 - std::pow((double)hp->beta1, (double)hp->step));
  c2 = 1.0 / (1.0 - std::pow((double)hp->beta2, (double)hp->step));
  return HGNN_OK;
}

hgnn_status hgnn_adam_update(hgnn_ctx *ctx, void *stream, int32_t n, void *const *param, float *const *master,
                             const float *const *grad, float *const *m, float *const *v, const int64_t *numel,
                             const hgnn_adam_params *hp) {
  if (!ctx || n < 0 || (n > 0 && (!param || !grad || !m || !v || !numel))) HGNN_FAIL(HGNN_EINVAL, "NULL argument");
  double c1, c2;
  hgnn_status st = check_adam(hp, c1, c2);
  if (st != HGNN_OK) return st;
  for (int i = 0; i < n; ++i) {
    if (numel[i] < 0 || numel[i] > (int64_t)INT32_MAX * 1024) HGNN_FAIL(HGNN_EINVAL, "numel[%d]=%lld out of range", i, (long long)numel[i]);
    if (numel[i] > 0 && (!param[i] || !grad[i] || !m[i] || !v[i])) HGNN_FAIL(HGNN_EINVAL, "tensor %d: NULL pointer", i);
    if (numel[i] > 0 && ctx->dtype != HGNN_F32 && (!master || !master[i]))
      HGNN_FAIL(HGNN_EINVAL, "tensor %d: a bf16 parameter needs an fp32 master copy", i);
  }
  if (ctx->device < 0) HGNN_FAIL(HGNN_EUNSUPPORTED, "host-only context cannot run device work");
  return launch_adam_dense((hipStream_t)stream, ctx->dtype, n, param, master, grad, m, v, numel, hp->lr, hp->beta1, hp->beta2,
                           hp->eps, c1, c2);
}

hgnn_status hgnn_adam_update_rows(hgnn_ctx *ctx, void *stream, void *store, float *master, float *m, float *v,
                                  int32_t feat_dim, const int64_t *ids, int64_t n_rows, const void *grad_rows,
                                  const hgnn_adam_params *hp) {
  if (!ctx || n_rows < 0) HGNN_FAIL(HGNN_EINVAL, "NULL argument");
  double c1, c2;
  hgnn_status st = check_adam(hp, c1, c2);
  if (st != HGNN_OK) return st;
  const int vec = 16 / esize(ctx->dtype);
  if (feat_dim <= 0 || feat_dim % vec != 0) HGNN_FAIL(HGNN_EINVAL, "feat_dim=%d is not a positive multiple of %d", feat_dim, vec);
  if (n_rows > 0 && (!store || !m || !v || !ids || !grad_rows)) HGNN_FAIL(HGNN_EINVAL, "NULL argument");
  if (n_rows > 0 && ctx->dtype != HGNN_F32 && !master) HGNN_FAIL(HGNN_EINVAL, "a bf16 table needs an fp32 master copy");
  for (const void *p : {(const void *)store, (const void *)master, (const void *)m, (const void *)v, grad_rows})
    if (reinterpret_cast<uintptr_t>(p) & 15) HGNN_FAIL(HGNN_EINVAL, "tables and gradient rows must be 16-byte aligned");
  if (ctx->device < 0) HGNN_FAIL(HGNN_EUNSUPPORTED, "host-only context cannot run device work");
  return launch_adam_rows((hipStream_t)stream, ctx->dtype, store, master, m, v, feat_dim, ids, n_rows, grad_rows, hp->lr,
                          hp->beta1, hp->beta2, hp->eps, c1, c2);
}

hgnn_status hgnn_probe_select(hgnn_ctx *ctx, int32_t kernel, int32_t layer) {
  if (!ctx) HGNN_FAIL(HGNN_EINVAL, "NULL context");
  if (kernel > HGNN_K_XENT) HGNN_FAIL(HGNN_EINVAL, "unknown kernel id %d", kernel);
  if (kernel < 0) {
    ctx->probe_n = 0;
    ctx->probe_used = 0;
    return HGNN_OK;
  }
  if (ctx->probe_n >= 4) HGNN_FAIL(HGNN_EINVAL, "at most 4 kernels can be selected at a time");
  ctx->probe_sel[ctx->probe_n][0] = kernel;
  ctx->probe_sel[ctx->probe_n][1] = layer;
  ++ctx->probe_n;
  return HGNN_OK;
}

hgnn_status hgnn_probe_read(hgnn_ctx *ctx, int32_t kernel, int32_t layer, double *total_ms, int64_t *launches) {
  if (!ctx || !total_ms || !launches) HGNN_FAIL(HGNN_EINVAL, "NULL argument");
  double sum = 0;
  int64_t n = 0;
  for (size_t i = 0; i < ctx->probe_used; ++i) {
    const int sl = ctx->probe_slot[i];
    if (ctx->probe_sel[sl][0] != kernel || ctx->probe_sel[sl][1] != layer) continue;
    float ms = 0;
    HGNN_HIP(hipEventSynchronize(ctx->probe_events[i].second));
    HGNN_HIP(hipEventElapsedTime(&ms, ctx->probe_events[i].first, ctx->probe_events[i].second));
    sum += ms;
    n += ctx->probe_first[i];
  }
  *total_ms = sum;
  *launches = n;
  return HGNN_OK;
}

}  // extern "C"
