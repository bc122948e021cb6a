// Host side of the semantic graph build (paper Section 4.3): edge-type matching and selection
// (Algorithm 2) fused with a stable parallel counting sort into one merged, relation-segmented
// CSR per layer, plus its transpose for the backward pass.  Integer work only.  The paper runs
// the selection with one OpenMP thread per relation; here the threads split the edge list
// instead (relations are very uneven in size), which yields the same arrays.
#include <algorithm>
#include <cstdarg>
#include <cstring>

#include "common.h"

namespace hgnn {

static thread_local char g_err[512] = "";
void set_error(const char *fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}
const char *get_error() { return g_err; }

// ------------------------------------------------------------------------------------------
ThreadPool::ThreadPool(int n) : nthreads_(n < 1 ? 1 : n) {
  for (int i = 0; i < nthreads_ - 1; ++i) th_.emplace_back([this] { worker(); });
}
ThreadPool::~ThreadPool() {
  {
    std::lock_guard<std::mutex> lk(m_);
    stop_ = true;
  }
  cv_.notify_all();
  for (auto &t : th_) t.join();
}
void ThreadPool::drain() {
  for (;;) {
    int i = next_.fetch_add(1, std::memory_order_relaxed);
    if (i >= nchunks_) break;
    (*fn_)(i);
  }
}
void ThreadPool::worker() {
  uint64_t seen = 0;
  for (;;) {
    {
      std::unique_lock<std::mutex> lk(m_);
      cv_.wait(lk, [&] { return stop_ || epoch_ != seen; });
      if (stop_) return;
      seen = epoch_;
    }
    drain();
    {
      std::lock_guard<std::mutex> lk(m_);
      if (--active_ == 0) done_cv_.notify_all();
    }
  }
}
void ThreadPool::parallel_for(int nchunks, const std::function<void(int)> &fn) {
  if (nchunks <= 0) return;
  if (th_.empty() || nchunks == 1) {
    for (int i = 0; i < nchunks; ++i) fn(i);
    return;
  }
  {
    std::lock_guard<std::mutex> lk(m_);
    fn_ = &fn;
    nchunks_ = nchunks;
    next_.store(0);
    active_ = (int)th_.size();
    ++epoch_;
  }
  cv_.notify_all();
  drain();
  std::unique_lock<std::mutex> lk(m_);
  done_cv_.wait(lk, [&] { return active_ == 0; });
  fn_ = nullptr;
}

// ------------------------------------------------------------------------------------------
namespace {

struct BuildError {
  std::mutex m;
  int status = HGNN_OK;
  std::string msg;
  std::atomic<bool> failed{false};
  void set(int st, const std::string &s) {
    std::lock_guard<std::mutex> lk(m);
    if (status == HGNN_OK) {
      status = st;
      msg = s;
      failed.store(true);
    }
  }
};

// Stable counting sort of items 0..n-1 by key[i] in [0,nkeys): pos[i] receives the output slot.
// ptr (nkeys+1) receives the exclusive prefix of the key counts.  `hist` is P*nkeys scratch.
template <class Emit>
void counting_sort_positions(ThreadPool &pool, int P, int64_t n, const int32_t *key, int64_t nkeys,
                             int32_t *ptr, std::vector<int32_t> &hist, Emit emit) {
  hist.resize((size_t)P * (size_t)nkeys);
  const int64_t slice = (n + P - 1) / P;
  pool.parallel_for(P, [&](int p) {
    int32_t *h = hist.data() + (size_t)p * nkeys;
    std::memset(h, 0, sizeof(int32_t) * (size_t)nkeys);
    const int64_t a = std::min<int64_t>(n, p * slice), b = std::min<int64_t>(n, a + slice);
    for (int64_t i = a; i < b; ++i) ++h[key[i]];
  });
  const int KC = std::max(1, P * 4);
  const int64_t kslice = (nkeys + KC - 1) / KC;
  pool.parallel_for(KC, [&](int c) {
    const int64_t a = std::min<int64_t>(nkeys, c * kslice), b = std::min<int64_t>(nkeys, a + kslice);
    for (int64_t k = a; k < b; ++k) {
      int32_t run = 0;
      for (int p = 0; p < P; ++p) {
        int32_t *h = hist.data() + (size_t)p * nkeys + k;
        const int32_t t = *h;
        *h = run;
        run += t;
      }
      ptr[k + 1] = run;
    }
  });
  ptr[0] = 0;
  for (int64_t k = 0; k < nkeys; ++k) ptr[k + 1] += ptr[k];
  pool.parallel_for(P, [&](int p) {
    int32_t *h = hist.data() + (size_t)p * nkeys;
    const int64_t a = std::min<int64_t>(n, p * slice), b = std::min<int64_t>(n, a + slice);
    for (int64_t i = a; i < b; ++i) {
      const int32_t k = key[i];
      emit(i, ptr[k] + h[k]++);
    }
  });
}

}  // namespace

static bool build_layer(hgnn_ctx *ctx, hgnn_graph *g, int l, BuildError &err) {
  LayerHost &L = g->L[l];
  const hgnn_coo_layer &in = L.in;
  const int T = ctx->T, R = ctx->R;
  int32_t *base = g->slab.host;
  int32_t *rel_row_off = base + L.o_rel_row_off, *rel_edge_off = base + L.o_rel_edge_off;
  int32_t *rowptr = base + L.o_rowptr, *colidx = base + L.o_colidx, *perm = base + L.o_perm;
  int32_t *cptr = base + L.o_cptr, *crow = base + L.o_crow, *cperm = base + L.o_cperm;
  int32_t row_off[kMaxT + 1];
  row_off[0] = 0;
  for (int t = 0; t < T; ++t) row_off[t + 1] = row_off[t] + (int32_t)L.n_src[t];
  rel_row_off[0] = 0;
  for (int r = 0; r < R; ++r) rel_row_off[r + 1] = rel_row_off[r] + (int32_t)L.n_dst[ctx->rel_dst[r]];
  const int64_t E = L.edges, rows = L.rows, src_rows = L.src_rows;
  ThreadPool &pool = *ctx->pool;
  const int P = (int)std::max<int64_t>(1, std::min<int64_t>(pool.size(), (E + 8191) / 8192));
  ctx->key.resize((size_t)E);
  ctx->col.resize((size_t)E);
  ctx->rowid.resize((size_t)E);
  int32_t *key = ctx->key.data(), *col = ctx->col.data(), *rowid = ctx->rowid.data();

  // Algorithm 2, line "EdgeTypeLayer <- IndexSelect(EdgeType, EdgeID[i])" and the per-relation
  // compare, done for all relations in one pass: each edge gets its merged row and source row.
  const int64_t slice = (E + P - 1) / P;
  pool.parallel_for(P, [&](int p) {
    const int64_t a = std::min<int64_t>(E, p * slice), b = std::min<int64_t>(E, a + slice);
    const int64_t *ei64 = in.index_is_i64 ? (const int64_t *)in.edge_index : nullptr;
    const int32_t *ei32 = in.index_is_i64 ? nullptr : (const int32_t *)in.edge_index;
    for (int64_t e = a; e < b; ++e) {
      int64_t r;
      if (in.edge_type) {
        r = in.edge_type[e];
      } else {
        const int64_t id = in.edge_id[e];
        if (id < 0 || id >= in.num_global_edges) {
          err.set(HGNN_EINVAL, "layer " + std::to_string(l) + ": edge_id[" + std::to_string(e) + "]=" +
                                   std::to_string(id) + " outside the global edge-type table");
          return;
        }
        r = in.global_edge_type[id];
      }
      if (r < 0 || r >= R) {
        err.set(HGNN_EINVAL, "layer " + std::to_string(l) + ": edge " + std::to_string(e) + " has type " +
                                 std::to_string(r) + " outside [0," + std::to_string(R) + ")");
        return;
      }
      const int64_t s = ei64 ? ei64[e] : (int64_t)ei32[e];
      const int64_t d = ei64 ? ei64[E + e] : (int64_t)ei32[E + e];
      const int ts = ctx->rel_src[r], td = ctx->rel_dst[r];
      if (s < 0 || s >= L.n_src[ts] || d < 0 || d >= L.n_dst[td]) {
        err.set(HGNN_EINVAL, "layer " + std::to_string(l) + ": edge " + std::to_string(e) + " (" +
                                 std::to_string(s) + "->" + std::to_string(d) + ", relation " +
                                 std::to_string(r) + ") outside its source/destination row range");
        return;
      }
      key[e] = rel_row_off[r] + (int32_t)d;
      col[e] = row_off[ts] + (int32_t)s;
    }
  });
  if (err.failed.load()) return false;

  // merged CSR: stable by (relation, destination)
  counting_sort_positions(pool, P, E, key, rows, rowptr, ctx->hist, [&](int64_t e, int32_t pos) {
    colidx[pos] = col[e];
    perm[pos] = (int32_t)e;
    rowid[pos] = key[e];
  });
  for (int r = 0; r <= R; ++r) rel_edge_off[r] = rowptr[rel_row_off[r]];

  // transpose: CSR positions grouped by source row, ascending position inside a group
  counting_sort_positions(pool, P, E, colidx, src_rows, cptr, ctx->hist, [&](int64_t k, int32_t pos) {
    crow[pos] = rowid[k];
    cperm[pos] = (int32_t)k;
  });

  // long transpose rows are cut into chunks so that no single wave walks thousands of edges
  int32_t *chunk_row = base + L.o_chunk_row, *chunk_beg = base + L.o_chunk_beg;
  int32_t *long_row = base + L.o_long_row, *long_chunk0 = base + L.o_long_chunk0;
  int32_t nl = 0, nc = 0;
  for (int64_t c = 0; c < src_rows; ++c) {
    const int32_t len = cptr[c + 1] - cptr[c];
    if (len > kLongRow) {
      long_row[nl] = (int32_t)c;
      long_chunk0[nl] = nc;
      ++nl;
      for (int32_t b = cptr[c]; b < cptr[c + 1]; b += kChunk) {
        chunk_row[nc] = (int32_t)c;
        chunk_beg[nc] = b;
        ++nc;
      }
    }
  }
  long_chunk0[nl] = nc;
  L.n_long = nl;
  L.n_chunks = nc;
  return true;
}

void build_graph_job(hgnn_ctx *ctx, hgnn_graph *g) {
  BuildError err;
  bool ok = true;
  for (int l = 0; l < g->num_layers && ok; ++l) ok = build_layer(ctx, g, l, err);
  int status = ok ? HGNN_OK : err.status;
  std::string msg = err.msg;
  if (ok && ctx->device >= 0) {
    hipError_t e = hipMemcpyAsync(g->slab.dev, g->slab.host, g->used * sizeof(int32_t), hipMemcpyHostToDevice, ctx->side);
    if (e == hipSuccess) e = hipEventRecord(g->ready, ctx->side);
    if (e != hipSuccess) {
      status = HGNN_EHIP;
      msg = std::string("graph upload: ") + hipGetErrorString(e);
    }
  }
  {
    std::lock_guard<std::mutex> lk(g->m);
    g->status = status;
    g->err = msg;
    g->state = (status == HGNN_OK) ? 1 : 2;
  }
  g->cv.notify_all();
}

}  // namespace hgnn
