// The semantic-graph build of Algorithm 2 done on the GPU instead of on host threads: the baseline that the paper's
// Section 4.3 argues against (edge-type matching and selection as device kernels in front of the layer's compute).
// It produces the same index arrays, bit for bit, in the same block layout as the host build, so every layer entry
// point runs on its graphs unchanged; bench.py times it against the host build.
//
//   keys      key[e] = rel_row_off[type(e)] + dst(e)  (the merged CSR row), value e; source row of x_merged per edge
//   sort 1    stable radix sort by key  -> perm, rowptr (lower bound of every row in the sorted keys), colidx
//   sort 2    stable radix sort of the CSR positions by source row -> cperm, cptr, crow (the transpose)
//   chunks    transpose rows longer than kLongRow cut into chunks of kChunk entries (two prefix sums)
// The call is synchronous: it returns after the arrays have been copied back into the graph's host block (the views
// and the host-side tables of the layer calls read them there) and the counts that size later launches are known.
#include <hipcub/hipcub.hpp>

#include <cstring>
#include <new>
#include <string>

#include "common.h"

namespace hgnn {

struct DevSchema {
  int32_t rel_row_off[kMaxR + 1];
  int32_t row_off[kMaxT + 1];
  int32_t n_src[kMaxT], n_dst[kMaxT];
  uint8_t rel_src[kMaxR], rel_dst[kMaxR];
  uint32_t tmask;
  int32_t R, T, rows, src_rows;
};

// error flag bits
constexpr int kBadType = 1, kBadSrc = 2, kBadDst = 4;

template <typename I>
__global__ void __launch_bounds__(256) dev_keys_kernel(const I *__restrict__ ei, int E, const int32_t *__restrict__ etype,
                                                        const int64_t *__restrict__ eid, const uint8_t *__restrict__ types8,
                                                        int64_t n_types8, DevSchema sc, int32_t *__restrict__ key,
                                                        int32_t *__restrict__ val, int32_t *__restrict__ colsrc,
                                                        int32_t *__restrict__ flag) {
  const int e = blockIdx.x * 256 + threadIdx.x;
  if (e >= E) return;
  int r = -1;
  if (etype) {
    r = etype[e];
  } else {
    const int64_t id = eid[e];
    if (id >= 0 && id < n_types8) r = types8[id];
  }
  int bad = 0;
  int32_t k = sc.rows, cs = 0;  // an invalid edge sorts behind every row
  if (r < 0 || r >= sc.R) {
    bad = kBadType;
  } else {
    const int64_t s = (int64_t)ei[e], d = (int64_t)ei[(int64_t)E + e];
    const int st = sc.rel_src[r], dt = sc.rel_dst[r];
    if (s < 0 || s >= sc.n_src[st]) bad |= kBadSrc;
    if (d < 0 || d >= sc.n_dst[dt]) bad |= kBadDst;
    if (!bad) {
      k = sc.rel_row_off[r] + (int32_t)d;
      cs = sc.row_off[st] + (int32_t)s;
    }
  }
  if (bad) atomicOr(flag, bad);
  key[e] = k;
  val[e] = e;
  colsrc[e] = cs;
}

// colidx[k] = source row of the edge at CSR position k; key2[k] = that row when its vertex type gets transpose
// entries, else a key behind every row; val2[k] = k
__global__ void __launch_bounds__(256) dev_csr_fill_kernel(int E, const int32_t *__restrict__ perm, const int32_t *__restrict__ colsrc,
                                                            DevSchema sc, int32_t *__restrict__ colidx, int32_t *__restrict__ key2,
                                                            int32_t *__restrict__ val2) {
  const int k = blockIdx.x * 256 + threadIdx.x;
  if (k >= E) return;
  const int32_t c = colsrc[perm[k]];
  colidx[k] = c;
  int t = 0;
  while (t + 1 < sc.T && c >= sc.row_off[t + 1]) ++t;
  key2[k] = ((sc.tmask >> t) & 1u) ? c : sc.src_rows;
  val2[k] = k;
}

// ptr[row] = first position of the sorted keys that is >= row, for row = 0..nrows
__global__ void __launch_bounds__(256) dev_lower_bound_kernel(const int32_t *__restrict__ keys, int E, int nrows, int32_t *__restrict__ ptr) {
  const int row = blockIdx.x * 256 + threadIdx.x;
  if (row > nrows) return;
  int lo = 0, hi = E;
  while (lo < hi) {
    const int mid = lo + (hi - lo) / 2;
    if (keys[mid] < row) lo = mid + 1; else hi = mid;
  }
  ptr[row] = lo;
}

__global__ void dev_rel_tables_kernel(DevSchema sc, const int32_t *__restrict__ rowptr, int32_t *__restrict__ rel_row_off,
                                      int32_t *__restrict__ rel_edge_off) {
  const int r = blockIdx.x * blockDim.x + threadIdx.x;
  if (r > sc.R) return;
  rel_row_off[r] = sc.rel_row_off[r];
  rel_edge_off[r] = rowptr[sc.rel_row_off[r]];
}

// crow[j] = merged CSR row of the edge at CSR position cperm[j] (positions beyond the kept entries included: they are
// never read); the CSR row of position k is the sorted key of sort 1
__global__ void __launch_bounds__(256) dev_crow_kernel(int E, const int32_t *__restrict__ cperm, const int32_t *__restrict__ row_of,
                                                        int32_t *__restrict__ crow) {
  const int j = blockIdx.x * 256 + threadIdx.x;
  if (j < E) crow[j] = row_of[cperm[j]];
}

// per transpose row: 1 when it is long, and its number of chunks (entry src_rows of both arrays = 0, so that the
// exclusive sums end with the totals)
__global__ void __launch_bounds__(256) dev_long_flags_kernel(const int32_t *__restrict__ cptr, int src_rows, int32_t *__restrict__ is_long,
                                                              int32_t *__restrict__ nchunk) {
  const int c = blockIdx.x * 256 + threadIdx.x;
  if (c > src_rows) return;
  int l = 0, n = 0;
  if (c < src_rows) {
    const int len = cptr[c + 1] - cptr[c];
    if (len > kLongRow) {
      l = 1;
      n = (len + kChunk - 1) / kChunk;
    }
  }
  is_long[c] = l;
  nchunk[c] = n;
}

__global__ void __launch_bounds__(256) dev_chunk_lists_kernel(const int32_t *__restrict__ cptr, int src_rows, const int32_t *__restrict__ long_at,
                                                               const int32_t *__restrict__ chunk_at, int32_t *__restrict__ long_row,
                                                               int32_t *__restrict__ long_chunk0, int32_t *__restrict__ chunk_row,
                                                               int32_t *__restrict__ chunk_beg, int32_t *__restrict__ counts) {
  const int c = blockIdx.x * 256 + threadIdx.x;
  if (c > src_rows) return;
  if (c == src_rows) {  // the totals, and the end of the last long row's chunks
    counts[0] = long_at[c];
    counts[1] = chunk_at[c];
    long_chunk0[long_at[c]] = chunk_at[c];
    return;
  }
  const int beg = cptr[c], len = cptr[c + 1] - beg;
  if (len <= kLongRow) return;
  const int i = long_at[c], j0 = chunk_at[c];
  long_row[i] = c;
  long_chunk0[i] = j0;
  for (int m = 0, q = beg; q < beg + len; q += kChunk, ++m) {
    chunk_row[j0 + m] = c;
    chunk_beg[j0 + m] = q;
  }
}

static int bits_for(int64_t max_key) {
  int b = 1;
  while (((int64_t)1 << b) <= max_key) ++b;
  return b;
}

// Device scratch of the build, grown on demand and kept by the context.
static hgnn_status need_tmp(hgnn_ctx *ctx, size_t bytes) {
  if (ctx->dev_tmp_cap >= bytes) return HGNN_OK;
  if (ctx->dev_tmp) (void)hipFree(ctx->dev_tmp);
  ctx->dev_tmp = nullptr;
  ctx->dev_tmp_cap = 0;
  const size_t cap = bytes + bytes / 4;
  hipError_t e = hipMalloc(&ctx->dev_tmp, cap);
  if (e != hipSuccess) HGNN_FAIL(HGNN_ENOMEM, "device build scratch (%zu bytes): %s", cap, hipGetErrorString(e));
  ctx->dev_tmp_cap = cap;
  return HGNN_OK;
}

static void give_back(hgnn_ctx *ctx, hgnn_graph *g) {
  {
    std::lock_guard<std::mutex> lk(ctx->pm);
    if (g->slab.host) ctx->free_slabs.push_back(g->slab);
    if (g->ready) ctx->free_events.push_back(g->ready);
  }
  delete g;
}

}  // namespace hgnn

using namespace hgnn;

extern "C" hgnn_status hgnn_build_semantic_csr_device(hgnn_ctx *ctx, void *stream, int32_t num_layers, const hgnn_coo_layer *layers,
                                                      hgnn_graph **out, float *gpu_ms) {
  if (!ctx || !layers || !out) HGNN_FAIL(HGNN_EINVAL, "NULL argument");
  *out = nullptr;
  if (gpu_ms) *gpu_ms = 0.f;
  if (ctx->device < 0) HGNN_FAIL(HGNN_EUNSUPPORTED, "host-only context cannot run device work");
  if (num_layers < 1 || num_layers > kMaxLayers) HGNN_FAIL(HGNN_EINVAL, "num_layers %d outside [1,%d]", num_layers, kMaxLayers);
  hgnn_graph *g = new (std::nothrow) hgnn_graph();
  if (!g) HGNN_FAIL(HGNN_ENOMEM, "out of host memory");
  g->num_layers = num_layers;
  for (int l = 0; l < num_layers; ++l) g->L[l].in = layers[l];
  std::string msg;
  hgnn_status st = plan_graph(ctx, g, msg);
  if (st != HGNN_OK) {
    give_back(ctx, g);
    HGNN_FAIL(st, "%s", msg.c_str());
  }
  const int T = ctx->T, R = ctx->R;
  hipStream_t s = (hipStream_t)stream;
  auto fail = [&](hgnn_status code, const std::string &m) {
    (void)hipStreamSynchronize(s);
    give_back(ctx, g);
    set_error("%s", m.c_str());
    return code;
  };
  // the registered global edge-type table, once per registration
  bool use_table = false;
  for (int l = 0; l < num_layers; ++l) use_table |= layers[l].num_edges > 0 && !layers[l].edge_type && !layers[l].global_edge_type;
  if (use_table && ctx->dev_types8_version != ctx->types_version) {
    if (ctx->dev_types8) (void)hipFree(ctx->dev_types8);
    ctx->dev_types8 = nullptr;
    const size_t n = ctx->edge_types8.size();
    hipError_t e = hipMalloc((void **)&ctx->dev_types8, std::max<size_t>(n, 1));
    if (e == hipSuccess && n) e = hipMemcpy(ctx->dev_types8, ctx->edge_types8.data(), n, hipMemcpyHostToDevice);
    if (e != hipSuccess) return fail(HGNN_EHIP, std::string("edge-type table upload: ") + hipGetErrorString(e));
    ctx->dev_types8_version = ctx->types_version;
  }
  hipEvent_t ev0 = nullptr, ev1 = nullptr;
  if (gpu_ms) {
    if (hipEventCreate(&ev0) != hipSuccess || hipEventCreate(&ev1) != hipSuccess) return fail(HGNN_EHIP, "hipEventCreate failed");
    (void)hipEventRecord(ev0, s);
  }
  // scratch for the largest layer
  size_t max_e = 1, max_rows = 1;
  for (int l = 0; l < num_layers; ++l) {
    max_e = std::max<size_t>(max_e, (size_t)g->L[l].edges);
    max_rows = std::max<size_t>(max_rows, (size_t)std::max(g->L[l].rows, g->L[l].src_rows) + 1);
  }
  size_t sort_tmp = 0, scan_tmp = 0;
  {
    hipcub::DoubleBuffer<int32_t> dk(nullptr, nullptr), dv(nullptr, nullptr);
    (void)hipcub::DeviceRadixSort::SortPairs(nullptr, sort_tmp, dk, dv, (int)max_e, 0, 32, s);
    (void)hipcub::DeviceScan::ExclusiveSum(nullptr, scan_tmp, (int32_t *)nullptr, (int32_t *)nullptr, (int)max_rows, s);
  }
  auto up = [](size_t n) { return (n + 255) / 256 * 256; };
  const size_t e4 = up(max_e * 4), r4 = up(max_rows * 4);
  // raw input (index pairs up to 16 bytes an edge, type or id up to 8), 7 int32 arrays of E, 4 of rows, library scratch, counters
  const size_t total = up(max_e * 16) + up(max_e * 8) + 7 * e4 + 4 * r4 + up(std::max(sort_tmp, scan_tmp)) + 256 * (size_t)kMaxLayers;
  if ((st = need_tmp(ctx, total)) != HGNN_OK) {
    give_back(ctx, g);
    return st;
  }
  char *tp = (char *)ctx->dev_tmp;
  auto carve = [&](size_t bytes) { char *p = tp; tp += bytes; return p; };
  void *d_ei = carve(up(max_e * 16));
  void *d_et = carve(up(max_e * 8));
  int32_t *key_a = (int32_t *)carve(e4), *key_b = (int32_t *)carve(e4), *val_a = (int32_t *)carve(e4), *val_b = (int32_t *)carve(e4);
  int32_t *colsrc = (int32_t *)carve(e4), *key2_b = (int32_t *)carve(e4), *val2_b = (int32_t *)carve(e4);
  int32_t *is_long = (int32_t *)carve(r4), *nchunk = (int32_t *)carve(r4), *long_at = (int32_t *)carve(r4), *chunk_at = (int32_t *)carve(r4);
  void *lib_tmp = carve(up(std::max(sort_tmp, scan_tmp)));
  int32_t *d_counts = (int32_t *)carve(256 * (size_t)kMaxLayers);   // per layer: n_long, n_chunks, error flags
  size_t lib_bytes = std::max(sort_tmp, scan_tmp);
  hipError_t he = hipMemsetAsync(d_counts, 0, 256 * (size_t)kMaxLayers, s);
  int32_t *base = g->slab.dev;
  for (int l = 0; l < num_layers && he == hipSuccess; ++l) {
    LayerHost &L = g->L[l];
    const hgnn_coo_layer &in = L.in;
    const int E = (int)L.edges;
    DevSchema sc;
    std::memset(&sc, 0, sizeof(sc));
    sc.R = R; sc.T = T; sc.rows = (int32_t)L.rows; sc.src_rows = (int32_t)L.src_rows; sc.tmask = L.tmask;
    for (int t = 0; t < T; ++t) {
      sc.n_src[t] = (int32_t)L.n_src[t];
      sc.n_dst[t] = (int32_t)L.n_dst[t];
      sc.row_off[t + 1] = sc.row_off[t] + (int32_t)L.n_src[t];
    }
    for (int r = 0; r < R; ++r) {
      sc.rel_src[r] = (uint8_t)ctx->rel_src[r];
      sc.rel_dst[r] = (uint8_t)ctx->rel_dst[r];
      sc.rel_row_off[r + 1] = sc.rel_row_off[r] + (int32_t)L.n_dst[ctx->rel_dst[r]];
    }
    int32_t *counts = d_counts + 64 * l;
    int32_t *rowptr = base + L.o_rowptr, *colidx = base + L.o_colidx, *cptr = base + L.o_cptr, *crow = base + L.o_crow;
    const int eb = (E + 255) / 256;
    const int32_t *perm = val_a, *row_of = key_a, *cperm = val2_b;
    if (E > 0) {
      const size_t isz = in.index_is_i64 ? 8 : 4;
      he = hipMemcpyAsync(d_ei, in.edge_index, 2 * (size_t)E * isz, hipMemcpyHostToDevice, s);
      const int32_t *d_type = nullptr;
      const int64_t *d_id = nullptr;
      std::vector<int32_t> resolved;
      if (he == hipSuccess && in.edge_type) {
        he = hipMemcpyAsync(d_et, in.edge_type, (size_t)E * 4, hipMemcpyHostToDevice, s);
        d_type = (const int32_t *)d_et;
      } else if (he == hipSuccess && in.global_edge_type) {
        // a table of the caller's own: the lookup is done here, on the host, and the per-edge types go up
        resolved.resize(E);
        for (int e = 0; e < E; ++e) {
          const int64_t id = in.edge_id[e];
          resolved[e] = (id >= 0 && id < in.num_global_edges) ? in.global_edge_type[id] : -1;
        }
        he = hipMemcpyAsync(d_et, resolved.data(), (size_t)E * 4, hipMemcpyHostToDevice, s);
        if (he == hipSuccess) he = hipStreamSynchronize(s);  // `resolved` goes out of scope below
        d_type = (const int32_t *)d_et;
      } else if (he == hipSuccess) {
        he = hipMemcpyAsync(d_et, in.edge_id, (size_t)E * 8, hipMemcpyHostToDevice, s);
        d_id = (const int64_t *)d_et;
      }
      if (he != hipSuccess) break;
      if (in.index_is_i64)
        HGNN_LAUNCH(dev_keys_kernel<int64_t>, dim3(eb), dim3(256), 0, s, (const int64_t *)d_ei, E, d_type, d_id, ctx->dev_types8,
                    (int64_t)ctx->edge_types8.size(), sc, key_a, val_a, colsrc, counts + 2);
      else
        HGNN_LAUNCH(dev_keys_kernel<int32_t>, dim3(eb), dim3(256), 0, s, (const int32_t *)d_ei, E, d_type, d_id, ctx->dev_types8,
                    (int64_t)ctx->edge_types8.size(), sc, key_a, val_a, colsrc, counts + 2);
      {
        hipcub::DoubleBuffer<int32_t> dk(key_a, key_b), dv(val_a, val_b);
        size_t nb = lib_bytes;
        he = hipcub::DeviceRadixSort::SortPairs(lib_tmp, nb, dk, dv, E, 0, bits_for(L.rows), s);
        if (he != hipSuccess) break;
        row_of = dk.Current();
        perm = dv.Current();
      }
      // the buffers sort 1 did not end in are free for sort 2's input
      int32_t *key2_a = row_of == key_a ? key_b : key_a, *val2_a = perm == val_a ? val_b : val_a;
      HGNN_LAUNCH(dev_csr_fill_kernel, dim3(eb), dim3(256), 0, s, E, perm, colsrc, sc, colidx, key2_a, val2_a);
      {
        hipcub::DoubleBuffer<int32_t> dk(key2_a, key2_b), dv(val2_a, val2_b);
        size_t nb = lib_bytes;
        he = hipcub::DeviceRadixSort::SortPairs(lib_tmp, nb, dk, dv, E, 0, bits_for(L.src_rows), s);
        if (he != hipSuccess) break;
        HGNN_LAUNCH(dev_lower_bound_kernel, dim3((int)(L.src_rows + 256) / 256), dim3(256), 0, s, dk.Current(), E, (int)L.src_rows, cptr);
        cperm = dv.Current();
      }
      HGNN_LAUNCH(dev_crow_kernel, dim3(eb), dim3(256), 0, s, E, cperm, row_of, crow);
    } else {
      HGNN_LAUNCH(dev_lower_bound_kernel, dim3((int)(L.src_rows + 256) / 256), dim3(256), 0, s, key_a, 0, (int)L.src_rows, cptr);
    }
    HGNN_LAUNCH(dev_lower_bound_kernel, dim3((int)(L.rows + 256) / 256), dim3(256), 0, s, row_of, E, (int)L.rows, rowptr);
    HGNN_LAUNCH(dev_rel_tables_kernel, dim3(1), dim3(256), 0, s, sc, rowptr, base + L.o_rel_row_off, base + L.o_rel_edge_off);
    // long transpose rows
    const int rb = (int)(L.src_rows + 256) / 256;
    HGNN_LAUNCH(dev_long_flags_kernel, dim3(rb), dim3(256), 0, s, cptr, (int)L.src_rows, is_long, nchunk);
    {
      size_t nb = lib_bytes;
      he = hipcub::DeviceScan::ExclusiveSum(lib_tmp, nb, is_long, long_at, (int)L.src_rows + 1, s);
      nb = lib_bytes;
      if (he == hipSuccess) he = hipcub::DeviceScan::ExclusiveSum(lib_tmp, nb, nchunk, chunk_at, (int)L.src_rows + 1, s);
      if (he != hipSuccess) break;
    }
    HGNN_LAUNCH(dev_chunk_lists_kernel, dim3(rb), dim3(256), 0, s, cptr, (int)L.src_rows, long_at, chunk_at, base + L.o_long_row,
                base + L.o_long_chunk0, base + L.o_chunk_row, base + L.o_chunk_beg, counts);
    // the permutations: on the device for the attention variant (cperm), host views otherwise
    if (E > 0) {
      const bool cperm_on_device = ctx->agg == HGNN_AGG_ATTN;
      if (cperm_on_device) he = hipMemcpyAsync(base + L.o_cperm, cperm, (size_t)E * 4, hipMemcpyDeviceToDevice, s);
      else he = hipMemcpyAsync(g->slab.host + L.o_cperm, cperm, (size_t)E * 4, hipMemcpyDeviceToHost, s);
      if (he == hipSuccess) he = hipMemcpyAsync(g->slab.host + L.o_perm, perm, (size_t)E * 4, hipMemcpyDeviceToHost, s);
      // the scratch arrays are reused by the next layer: in stream order, so nothing more to wait for
    }
  }
  if (he == hipSuccess) he = hipGetLastError();
  if (he == hipSuccess && ev1) he = hipEventRecord(ev1, s);
  if (he == hipSuccess) he = hipMemcpyAsync(g->slab.host, g->slab.dev, g->used * sizeof(int32_t), hipMemcpyDeviceToHost, s);
  std::vector<int32_t> host_counts(64 * (size_t)num_layers);
  if (he == hipSuccess) he = hipStreamSynchronize(s);
  if (he == hipSuccess) he = hipMemcpy(host_counts.data(), d_counts, host_counts.size() * sizeof(int32_t), hipMemcpyDeviceToHost);
  if (gpu_ms && he == hipSuccess) (void)hipEventElapsedTime(gpu_ms, ev0, ev1);
  if (ev0) (void)hipEventDestroy(ev0);
  if (ev1) (void)hipEventDestroy(ev1);
  if (he != hipSuccess) return fail(HGNN_EHIP, std::string("device build: ") + hipGetErrorString(he));
  for (int l = 0; l < num_layers; ++l) {
    const int32_t *c = host_counts.data() + 64 * l;
    if (c[2]) {
      char buf[160];
      std::snprintf(buf, sizeof(buf), "layer %d: %s%s%s", l, (c[2] & kBadType) ? "edge type outside [0,R) " : "",
                    (c[2] & kBadSrc) ? "source index outside its type's rows " : "", (c[2] & kBadDst) ? "destination index outside its type's rows" : "");
      return fail(HGNN_EINVAL, buf);
    }
    g->L[l].n_long = c[0];
    g->L[l].n_chunks = c[1];
    g->L[l].tedges = g->slab.host[g->L[l].o_cptr + g->L[l].src_rows];
  }
  he = hipEventRecord(g->ready, s);
  if (he != hipSuccess) return fail(HGNN_EHIP, std::string("hipEventRecord: ") + hipGetErrorString(he));
  {
    std::lock_guard<std::mutex> lk(g->m);
    g->status = HGNN_OK;
    g->state = 1;
  }
  *out = g;
  return HGNN_OK;
}
