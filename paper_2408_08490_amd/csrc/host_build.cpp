// Host side of the semantic graph build (paper Section 4.3): edge-type matching and selection
// (Algorithm 2) fused with a stable parallel counting sort into one merged, relation-segmented
// CSR per layer, plus its transpose for the backward pass.  Integer work only.  The paper runs
// the selection with one OpenMP thread per relation; here the threads split the edge list
// instead (relations are very uneven in size), which yields the same arrays.
#include <algorithm>
#include <chrono>
#include <cstdlib>
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

constexpr int kBucketShift = 12;  // 4096 consecutive keys form one bucket (its counters stay in L1)

}  // namespace

// Two-level stable counting sort, used twice per layer (edges by merged row; CSR positions by source
// row).  Level 1 splits the items into key-range buckets (threads own contiguous item slices, so the
// order inside a bucket is the input order); level 2 sorts every bucket on its own with a local
// histogram and writes the final arrays and the bucket's part of the row pointer.
// A level-1 record carries (key, item, payload).  Wide: three ints.  Packed: two ints -- only the key's offset
// inside its bucket is needed once the record lies in the bucket, and it fits above the payload when the
// payload stays below 2^(32 - kBucketShift): a third less to write, to fetch for ownership and to read back.
struct WideRec {
  static constexpr int W = 3;
  static void put(int32_t *r, int32_t key, int32_t item, int32_t payload) { r[0] = key; r[1] = item; r[2] = payload; }
  static int32_t key_low(const int32_t *r, int32_t k0) { return r[0] - k0; }
  static int32_t item(const int32_t *r) { return r[1]; }
  static int32_t payload(const int32_t *r) { return r[2]; }
};
struct PackedRec {
  static constexpr int W = 2, kPayloadBits = 32 - kBucketShift;
  static void put(int32_t *r, int32_t key, int32_t item, int32_t payload) {
    r[0] = item;
    r[1] = (int32_t)(((uint32_t)key << kPayloadBits) | (uint32_t)payload);  // the shift drops the bucket's bits
  }
  static int32_t key_low(const int32_t *r, int32_t) { return (int32_t)((uint32_t)r[1] >> kPayloadBits); }
  static int32_t item(const int32_t *r) { return r[0]; }
  static int32_t payload(const int32_t *r) { return (int32_t)((uint32_t)r[1] & ((1u << kPayloadBits) - 1u)); }
};

// One int: for builds that leave the permutation out, the item is not carried at all.
struct SlimRec {
  static constexpr int W = 1, kPayloadBits = 32 - kBucketShift;
  static void put(int32_t *r, int32_t key, int32_t, int32_t payload) {
    r[0] = (int32_t)(((uint32_t)key << kPayloadBits) | (uint32_t)payload);
  }
  static int32_t key_low(const int32_t *r, int32_t) { return (int32_t)((uint32_t)r[0] >> kPayloadBits); }
  static int32_t item(const int32_t *) { return 0; }
  static int32_t payload(const int32_t *r) { return (int32_t)((uint32_t)r[0] & ((1u << kPayloadBits) - 1u)); }
};

struct PhaseTimer {
  bool on;
  std::chrono::steady_clock::time_point t0;
  PhaseTimer() : on(getenv("HGNN_BUILD_TIMING") != nullptr), t0(std::chrono::steady_clock::now()) {}
  void lap(const char *what) {
    if (!on) return;
    auto t1 = std::chrono::steady_clock::now();
    fprintf(stderr, "  [build] %-28s %8.3f ms\n", what, std::chrono::duration<double, std::milli>(t1 - t0).count());
    t0 = t1;
  }
};

static bool build_layer(hgnn_ctx *ctx, Builder &bd, hgnn_graph *g, int l, BuildError &err) {
  PhaseTimer tm;
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
  ThreadPool &pool = *bd.pool;
  const int P = (int)std::max<int64_t>(1, std::min<int64_t>(pool.size(), (E + 16383) / 16384));
  const int B1 = (int)((rows + (1 << kBucketShift) - 1) >> kBucketShift);
  const int B2 = (int)((src_rows + (1 << kBucketShift) - 1) >> kBucketShift);
  auto grow = [](std::vector<int32_t> &v, size_t n) {
    if (v.size() < n) v.resize(n + n / 4);
  };
  grow(bd.key, (size_t)E);
  grow(bd.col, (size_t)E);
  grow(bd.tkey, (size_t)E * 3);  // level-1 records: (key, item, payload)
  // counter rows are padded to whole 128-byte lines: neighbouring threads must not share a line
  const size_t S1 = ((size_t)B1 + 63) / 32 * 32, S2 = ((size_t)B2 + 63) / 32 * 32;
  grow(bd.hist, (size_t)P * S1 + (size_t)std::max(B1, 1) * S2 + B1 + B2 + 2 + 64);
  int32_t *key = bd.key.data(), *col = bd.col.data();
  int32_t *trec = bd.tkey.data();
  int32_t *cnt1 = reinterpret_cast<int32_t *>((reinterpret_cast<uintptr_t>(bd.hist.data()) + 127) & ~(uintptr_t)127);  // [P][S1]
  int32_t *cnt2 = cnt1 + (size_t)P * S1;                     // [B1][S2]
  int32_t *base1 = cnt2 + (size_t)std::max(B1, 1) * S2;      // [B1+1]
  int32_t *base2 = base1 + B1 + 1;                           // [B2+1]
  std::memset(cnt1, 0, sizeof(int32_t) * (size_t)P * S1);
  std::memset(cnt2, 0, sizeof(int32_t) * (size_t)std::max(B1, 1) * S2);
  tm.lap("setup");

  // A mini-batch drawn by the library's own sampler arrives relation by relation, destinations ascending, and
  // its edges were read off the graph: there is nothing to look up, check or sort -- the merged CSR is the input
  // order itself.
  // (a test can ask for the three-int records where the two-int ones would do)
  static const bool wide_records = getenv("HGNN_WIDE_RECORDS") != nullptr;
  const bool csc_packed = rows <= (int64_t)1 << PackedRec::kPayloadBits && !wide_records;
  const bool presorted = g->job != nullptr;
  const bool with_perm = g->with_perm;
  if (presorted) {
    const SampleJob &job = *g->job;
    const int64_t *es = job.edge_index[l].data(), *ed = es + E;
    const int64_t *reo = job.rel_edge_off[l];
    for (int r = 0; r < R; ++r) {
      const int32_t row0 = rel_row_off[r], col0 = row_off[ctx->rel_src[r]];
      const int32_t nd = rel_row_off[r + 1] - row0;
      const bool want = (L.tmask >> ctx->rel_src[r]) & 1u;
      int64_t e = reo[r];
      const int64_t e_end = reo[r + 1];
      for (int32_t i = 0; i < nd; ++i) {
        rowptr[row0 + i] = (int32_t)e;
        int32_t *c2 = cnt2 + (size_t)((row0 + i) >> kBucketShift) * S2;
        for (; e < e_end && ed[e] == i; ++e) {
          const int32_t c = col0 + (int32_t)es[e];
          colidx[e] = c;
          if (with_perm) perm[e] = (int32_t)e;
          if (want) ++c2[c >> kBucketShift];
        }
      }
    }
    for (int b = 0; b <= B1; ++b) base1[b] = b < B1 ? rowptr[(size_t)b << kBucketShift] : (int32_t)E;
    tm.lap("csr from sampler order");
  } else {
  // Algorithm 2: the layer's edge types are looked up through the edge ids (or taken as given) and matched
  // against the relations -- for all relations in one pass: each edge gets its merged row and source row.
  const int64_t slice = (E + P - 1) / P;
  pool.parallel_for(P, [&](int p) {
    const int64_t a = std::min<int64_t>(E, p * slice), b = std::min<int64_t>(E, a + slice);
    const int64_t *ei64 = in.index_is_i64 ? (const int64_t *)in.edge_index : nullptr;
    const int32_t *ei32 = in.index_is_i64 ? nullptr : (const int32_t *)in.edge_index;
    int32_t *cnt = cnt1 + (size_t)p * S1;
    const uint8_t *types8 = ctx->edge_types8.data();
    const int64_t n_types8 = (int64_t)ctx->edge_types8.size();
    const int nruns = (int)ctx->run_end.size();
    const int64_t *run_end = ctx->run_end.data();
    const uint8_t *run_rel = ctx->run_rel.data(), *run_lut = ctx->run_lut.data();
    const int run_shift = ctx->run_shift;
    for (int64_t e = a; e < b; ++e) {
      int64_t r;
      if (in.edge_type) {
        r = in.edge_type[e];
      } else if (!in.global_edge_type && nruns > 0) {   // the registered table, as runs of equal type
        const int64_t id = in.edge_id[e];
        if (id < 0 || id >= n_types8) {
          err.set(HGNN_EINVAL, "layer " + std::to_string(l) + ": edge_id[" + std::to_string(e) + "]=" +
                                   std::to_string(id) + " outside the registered edge-type table");
          return;
        }
        int j = run_lut[id >> run_shift];
        while (id >= run_end[j]) ++j;  // ends: id < n_types8 = the last run's end
        r = run_rel[j];
      } else if (!in.global_edge_type) {   // the registered compact table
        if (e + 48 < b) {
          const int64_t nid = in.edge_id[e + 48];
          if (nid >= 0 && nid < n_types8) __builtin_prefetch(types8 + nid);
        }
        const int64_t id = in.edge_id[e];
        if (id < 0 || id >= n_types8) {
          err.set(HGNN_EINVAL, "layer " + std::to_string(l) + ": edge_id[" + std::to_string(e) + "]=" +
                                   std::to_string(id) + " outside the registered edge-type table");
          return;
        }
        r = types8[id];
      } else {
        if (e + 48 < b) {
          const int64_t nid = in.edge_id[e + 48];
          if (nid >= 0 && nid < in.num_global_edges) __builtin_prefetch(in.global_edge_type + nid);
        }
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
      const int32_t k = rel_row_off[r] + (int32_t)d;
      key[e] = k;
      col[e] = row_off[ts] + (int32_t)s;
      ++cnt[k >> kBucketShift];
    }
  });
  if (err.failed.load()) return false;
  tm.lap("select (Alg.2) + count");

  // ---- merged CSR: stable by (relation, destination) ----
  {
    int32_t run = 0;
    for (int b = 0; b < B1; ++b) {
      base1[b] = run;
      for (int p = 0; p < P; ++p) {
        const int32_t t = cnt1[(size_t)p * S1 + b];
        cnt1[(size_t)p * S1 + b] = run;
        run += t;
      }
    }
    base1[B1] = run;
  }
  auto csr_sort = [&](auto rec_format, auto perm_flag) {
    using Rec = decltype(rec_format);
    constexpr bool kPerm = decltype(perm_flag)::value;
    pool.parallel_for(P, [&](int p) {
      const int64_t a = std::min<int64_t>(E, p * slice), b = std::min<int64_t>(E, a + slice);
      int32_t *off = cnt1 + (size_t)p * S1;
      for (int64_t e = a; e < b; ++e) {
        const int32_t q = off[key[e] >> kBucketShift]++;
        Rec::put(trec + (size_t)q * Rec::W, key[e], (int32_t)e, col[e]);
      }
    });
    tm.lap("csr level-1 scatter");
    pool.parallel_for(B1, [&](int b) {
      int32_t h[(1 << kBucketShift) + 1];
      const int32_t k0 = b << kBucketShift;
      const int32_t nk = (int32_t)std::min<int64_t>(1 << kBucketShift, rows - k0);
      std::memset(h, 0, sizeof(int32_t) * (nk + 1));
      const int32_t ja = base1[b], jb = base1[b + 1];
      for (int32_t j = ja; j < jb; ++j) ++h[Rec::key_low(trec + (size_t)j * Rec::W, k0)];
      int32_t run = ja;
      for (int32_t i = 0; i < nk; ++i) {
        const int32_t t = h[i];
        h[i] = run;
        rowptr[k0 + i] = run;
        run += t;
      }
      for (int32_t j = ja; j < jb; ++j) {
        const int32_t *rec = trec + (size_t)j * Rec::W;
        const int32_t pos = h[Rec::key_low(rec, k0)]++;
        colidx[pos] = Rec::payload(rec);
        if constexpr (kPerm) perm[pos] = Rec::item(rec);
      }
    });
    tm.lap("csr level-2 buckets");
  };
  const bool fits = src_rows <= (int64_t)1 << PackedRec::kPayloadBits && !wide_records;
  if (with_perm) {
    if (fits) csr_sort(PackedRec(), std::true_type());
    else csr_sort(WideRec(), std::true_type());
  } else {
    if (fits) csr_sort(SlimRec(), std::false_type());
    else csr_sort(WideRec(), std::false_type());
  }
  }
  rowptr[rows] = (int32_t)E;
  for (int r = 0; r <= R; ++r) rel_edge_off[r] = rowptr[rel_row_off[r]];

  // All sources of a relation have one type, and the CSR is ordered by relation: the positions whose source row
  // is wanted are whole relation ranges, so the others are skipped without being read.
  int n_pr = 0;
  int32_t pr_lo[kMaxR], pr_hi[kMaxR];
  for (int r = 0; r < R; ++r) {
    if (!((L.tmask >> ctx->rel_src[r]) & 1u) || rel_edge_off[r + 1] == rel_edge_off[r]) continue;
    if (n_pr > 0 && pr_hi[n_pr - 1] == rel_edge_off[r]) pr_hi[n_pr - 1] = rel_edge_off[r + 1];
    else { pr_lo[n_pr] = rel_edge_off[r]; pr_hi[n_pr] = rel_edge_off[r + 1]; ++n_pr; }
  }
  // level-1 counts of the transpose: per CSR bucket, how many of its wanted positions fall into each bucket of
  // source rows (a sweep of its own over the wanted ranges: inside the scatter loop above the test "is this
  // source row wanted" is a coin flip for the branch predictor and cost more than the whole sweep)
  if (!presorted)
    pool.parallel_for(B1, [&](int b1) {
      int32_t *c2 = cnt2 + (size_t)b1 * S2;
      for (int i = 0; i < n_pr; ++i) {
        const int32_t ka = std::max(base1[b1], pr_lo[i]), kb = std::min(base1[b1 + 1], pr_hi[i]);
        for (int32_t k = ka; k < kb; ++k) ++c2[colidx[k] >> kBucketShift];
      }
    });
  // ---- transpose: CSR positions grouped by source row, ascending position inside a group ----
  // the level-1 slices are the CSR position ranges of the buckets above (already in CSR order)
  {
    int32_t run = 0;
    for (int b2 = 0; b2 < B2; ++b2) {
      base2[b2] = run;
      for (int b1 = 0; b1 < B1; ++b1) {
        const int32_t t = cnt2[(size_t)b1 * S2 + b2];
        cnt2[(size_t)b1 * S2 + b2] = run;
        run += t;
      }
    }
    base2[B2] = run;
  }
  pool.parallel_for(B1, [&](int b1) {
    int32_t *off = cnt2 + (size_t)b1 * S2;
    for (int i = 0; i < n_pr; ++i) {
      const int32_t ka = std::max(base1[b1], pr_lo[i]), kb = std::min(base1[b1 + 1], pr_hi[i]);
      if (ka >= kb) continue;
      // the merged row of CSR position k: positions are walked in order, so the row pointer is walked along
      int32_t row = b1 << kBucketShift;
      {  // first row of the bucket that ends after ka
        int32_t hi = (int32_t)std::min<int64_t>(rows, (int64_t)(b1 + 1) << kBucketShift);
        while (row + 1 < hi) {
          const int32_t mid = row + (hi - row) / 2;
          if (rowptr[mid] <= ka) row = mid; else hi = mid;
        }
      }
      for (int32_t k = ka; k < kb; ++k) {
        while (rowptr[row + 1] <= k) ++row;
        const int32_t c = colidx[k];
        const int32_t q = off[c >> kBucketShift]++;
        if (!csc_packed) WideRec::put(trec + (size_t)q * WideRec::W, c, k, row);
        else if (with_perm) PackedRec::put(trec + (size_t)q * PackedRec::W, c, k, row);
        else SlimRec::put(trec + q, c, k, row);
      }
    }
  });
  tm.lap("csc level-1 scatter");
  std::vector<std::vector<int32_t>> &longs = bd.long_lists;
  if ((int)longs.size() < B2) longs.resize(B2);
  auto csc_level2 = [&](auto rec_format, auto perm_flag) {
    using Rec = decltype(rec_format);
    constexpr bool kPerm = decltype(perm_flag)::value;
    pool.parallel_for(B2, [&](int b) {
      int32_t h[(1 << kBucketShift) + 1];
      const int32_t k0 = b << kBucketShift;
      const int32_t nk = (int32_t)std::min<int64_t>(1 << kBucketShift, src_rows - k0);
      std::memset(h, 0, sizeof(int32_t) * (nk + 1));
      const int32_t ja = base2[b], jb = base2[b + 1];
      for (int32_t j = ja; j < jb; ++j) ++h[Rec::key_low(trec + (size_t)j * Rec::W, k0)];
      int32_t run = ja;
      longs[b].clear();
      for (int32_t i = 0; i < nk; ++i) {
        const int32_t t = h[i];
        if (t > kLongRow) longs[b].push_back(k0 + i);
        h[i] = run;
        cptr[k0 + i] = run;
        run += t;
      }
      for (int32_t j = ja; j < jb; ++j) {
        const int32_t *rec = trec + (size_t)j * Rec::W;
        const int32_t pos = h[Rec::key_low(rec, k0)]++;
        crow[pos] = Rec::payload(rec);
        if constexpr (kPerm) cperm[pos] = Rec::item(rec);
      }
    });
  };
  if (with_perm) {
    if (csc_packed) csc_level2(PackedRec(), std::true_type());
    else csc_level2(WideRec(), std::true_type());
  } else {
    if (csc_packed) csc_level2(SlimRec(), std::false_type());
    else csc_level2(WideRec(), std::false_type());
  }
  cptr[src_rows] = base2[B2];
  L.tedges = base2[B2];
  tm.lap("csc level-2 buckets");

  // long transpose rows are cut into chunks so that no single wave walks thousands of edges
  int32_t *chunk_row = base + L.o_chunk_row, *chunk_beg = base + L.o_chunk_beg;
  int32_t *long_row = base + L.o_long_row, *long_chunk0 = base + L.o_long_chunk0;
  int32_t nl = 0, nc = 0;
  for (int b = 0; b < B2; ++b)
    for (int32_t c : longs[b]) {
      long_row[nl] = c;
      long_chunk0[nl] = nc;
      ++nl;
      for (int32_t q = cptr[c]; q < cptr[c + 1]; q += kChunk) {
        chunk_row[nc] = c;
        chunk_beg[nc] = q;
        ++nc;
      }
    }
  long_chunk0[nl] = nc;
  L.n_long = nl;
  L.n_chunks = nc;
  tm.lap("long-row chunks");
  return true;
}

void build_graph_job(hgnn_ctx *ctx, Builder &bd, hgnn_graph *g) {
  BuildError err;
  bool ok = true;
  if (g->job) {  // sample first; only then are the sizes known that the block is laid out for
    std::string m;
    hgnn_status st = run_sample_job(ctx, bd, g, m);
    if (st == HGNN_OK) {
      {
        std::lock_guard<std::mutex> lk(g->m);
        g->sampled = true;
      }
      g->cv.notify_all();
      st = plan_graph(ctx, g, m);
    }
    if (st != HGNN_OK) {
      err.set(st, m);
      ok = false;
    } else {
      for (int t = 0; t < ctx->T; ++t)
        if (!g->job->ids[t].empty())
          std::memcpy(g->slab.host + g->o_ids[t], g->job->ids[t].data(), g->job->ids[t].size() * sizeof(int64_t));
    }
  }
  for (int l = 0; l < g->num_layers && ok; ++l) ok = build_layer(ctx, bd, g, l, err);
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
    // notified under the lock: a waiter may release (delete) the graph as soon as it sees the new state, so the
    // unlock must be this thread's last touch of it
    std::lock_guard<std::mutex> lk(g->m);
    g->status = status;
    g->err = msg;
    g->state = (status == HGNN_OK) ? 1 : 2;
    g->cv.notify_all();
  }
}

}  // namespace hgnn
