// Layer-wise neighbour sampling on the host (Section 2.3 step 1; Fig. 6's sampling thread), run as the first
// part of a builder's task so that sampling, edge index selection and upload of mini-batch i+k overlap the GPU
// work of mini-batch i.  The rule (order of visits, subset choice, generator) is the one stated with
// hgnn_sample_and_build in hgnn.h.
#include <algorithm>
#include <cstring>

#include "common.h"

namespace hgnn {

// SplitMix64 output function (Steele, Lea, Flood: "Fast splittable pseudorandom number generators", 2014)
static inline uint64_t mix64(uint64_t z) {
  z += 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

hgnn_status run_sample_job(hgnn_ctx *ctx, Builder &bd, hgnn_graph *g, std::string &msg) {
  SampleJob &job = *g->job;
  const hgnn_sampler &sm = *job.sampler;
  const int T = ctx->T, R = ctx->R, L = g->num_layers;
  for (int t = 0; t < T; ++t)
    if ((int64_t)bd.local_of[t].size() != sm.num_nodes[t]) bd.local_of[t].assign((size_t)sm.num_nodes[t], -1);
  // global ids per type of the current hop; the buffers live in the builder and in the (pooled) job, so that a
  // steady stream of mini-batches allocates nothing and touches no fresh pages
  std::vector<int64_t> *dst = bd.hop_ids[0], *src = bd.hop_ids[1];
  for (int t = 0; t < T; ++t) dst[t].clear();
  dst[job.target_type] = job.targets;
  I64Buf &ed = bd.edge_dst;
  const uint64_t k0 = mix64(job.seed);
  hgnn_status st = HGNN_OK;
  for (int h = 1; h <= L && st == HGNN_OK; ++h) {
    const int l = L - h;
    const int64_t fanout = job.fanouts[h - 1];
    const uint64_t kh = mix64(k0 ^ (uint64_t)h);
    for (int t = 0; t < T; ++t) {
      src[t] = dst[t];
      int32_t *lut = bd.local_of[t].data();
      for (size_t i = 0; i < dst[t].size(); ++i) {
        const int64_t v = dst[t][i];
        if (lut[v] >= 0) {  // only the targets can repeat: later hops' lists are distinct by construction
          msg = "target " + std::to_string(v) + " is listed twice";
          st = HGNN_EINVAL;
          src[t].resize(i);  // the entries to reset below
          break;
        }
        lut[v] = (int32_t)i;
      }
      job.n_dst[l][t] = (int64_t)dst[t].size();
    }
    I64Buf &es = job.edge_index[l];  // local sources first; the destinations are appended below
    I64Buf &eid = job.edge_id[l];
    {
      size_t bound = 0;  // every destination keeps at most `fanout` edges per relation
      for (int r = 0; r < R; ++r) bound += dst[ctx->rel_dst[r]].size() * (size_t)fanout;
      bound = std::min<size_t>(bound, (size_t)sm.edge_off[R]);
      if (!es.reserve(2 * bound + 1) || !ed.reserve(bound + 1) || !eid.reserve(bound + 1)) {
        msg = "out of host memory";
        st = HGNN_ENOMEM;
      }
    }
    int64_t *pes = es.p, *ped = ed.p, *peid = eid.p;
    size_t ne = 0;  // edges of this hop so far (the bound above holds, so the writes below need no check)
    for (int r = 0; r < R && st == HGNN_OK; ++r) {
      const int s = ctx->rel_src[r], d = ctx->rel_dst[r];
      const int64_t nd = (int64_t)dst[d].size();
      job.rel_edge_off[l][r] = (int64_t)ne;
      if (nd == 0) continue;
      const int64_t *ptr = sm.in_indptr[r];
      const int32_t *nbr = sm.in_nbr[r];
      const int64_t e0 = sm.edge_off[r];
      int32_t *lut = bd.local_of[s].data();
      std::vector<int64_t> &sl = src[s];
      const uint64_t kr = mix64(kh ^ (uint64_t)r);
      // Destination vertices are taken in blocks; inside a block every step (row pointers, neighbour positions,
      // neighbour ids, local-row table) is done for all vertices before the next, each step prefetching what the
      // next one reads: the reads are random accesses into arrays far larger than the caches, and this keeps
      // dozens of them in flight instead of one.
      constexpr int kBlock = 32, kMaxFan = 64;
      int64_t pos[kBlock][kMaxFan];
      int32_t cnt[kBlock];
      for (int64_t i0 = 0; i0 < nd; i0 += kBlock) {
        const int nb = (int)std::min<int64_t>(kBlock, nd - i0);
        for (int b = 0; b < nb; ++b) __builtin_prefetch(ptr + dst[d][i0 + b]);
        if (i0 + kBlock < nd)
          for (int b = 0; b < kBlock && i0 + kBlock + b < nd; b += 8) __builtin_prefetch(&dst[d][i0 + kBlock + b]);
        for (int b = 0; b < nb; ++b) {
          const int64_t v = dst[d][i0 + b];
          const int64_t first = ptr[v], deg = ptr[v + 1] - first;
          int64_t *pb = pos[b];
          if (deg <= fanout) {
            for (int64_t p = 0; p < deg; ++p) pb[p] = first + p;
            cnt[b] = (int32_t)deg;
            for (int64_t p = 0; p < deg; p += 16) __builtin_prefetch(nbr + first + p);
          } else {
            const uint64_t key = mix64(kr ^ (uint64_t)v);
            for (int64_t c = 0; c < fanout; ++c) {
              const int64_t j = deg - fanout + c;
              int64_t t = (int64_t)(((unsigned __int128)mix64(key + (uint64_t)c) * (uint64_t)(j + 1)) >> 64);
              bool again = false;
              for (int64_t q = 0; q < c; ++q) again |= pb[q] == first + t;  // no early exit: the loop vectorises
              if (again) t = j;
              pb[c] = first + t;
              __builtin_prefetch(nbr + first + t);
            }
            cnt[b] = (int32_t)fanout;
          }
        }
        for (int b = 0; b < nb; ++b)
          for (int c = 0; c < cnt[b]; ++c) __builtin_prefetch(lut + nbr[pos[b][c]]);
        for (int b = 0; b < nb; ++b) {
          const int64_t i = i0 + b;
          for (int c = 0; c < cnt[b]; ++c) {
            const int64_t p = pos[b][c];
            const int64_t u = nbr[p];
            int32_t loc = lut[u];
            if (loc < 0) {
              loc = (int32_t)sl.size();
              lut[u] = loc;
              sl.push_back(u);
            }
            pes[ne] = loc;
            ped[ne] = i;
            peid[ne] = e0 + p;
            ++ne;
          }
        }
      }
      if (sl.size() > (size_t)INT32_MAX - 1) {
        msg = "more than 2^31-2 source rows of one type";
        st = HGNN_EOVERFLOW;
      }
    }
    // this hop's block; the lookup tables go back to "not in the hop"
    job.rel_edge_off[l][R] = (int64_t)ne;
    if (st == HGNN_OK && ne) std::memcpy(pes + ne, ped, ne * sizeof(int64_t));
    es.n = 2 * ne;
    eid.n = ne;
    for (int t = 0; t < T; ++t) {
      job.n_src[l][t] = (int64_t)src[t].size();
      int32_t *lut = bd.local_of[t].data();
      for (int64_t v : src[t]) lut[v] = -1;
    }
    std::swap(dst, src);
  }
  if (st != HGNN_OK) return st;
  for (int t = 0; t < T; ++t) job.ids[t].assign(dst[t].begin(), dst[t].end());
  for (int l = 0; l < L; ++l) {
    hgnn_coo_layer &in = g->L[l].in;
    std::memset(&in, 0, sizeof(in));
    in.num_edges = (int64_t)job.edge_id[l].size();
    in.edge_index = job.edge_index[l].data();
    in.index_is_i64 = 1;
    in.edge_id = job.edge_id[l].data();
    in.n_src = job.n_src[l];
    in.n_dst = job.n_dst[l];
    in.transpose_types = job.transpose[l].empty() ? nullptr : job.transpose[l].data();
  }
  return HGNN_OK;
}

}  // namespace hgnn

using namespace hgnn;

hgnn_status hgnn_sampler_create(hgnn_ctx *ctx, const hgnn_host_graph *graph, hgnn_sampler **out) {
  if (!ctx || !graph || !out || !graph->num_nodes || !graph->in_indptr || !graph->in_nbr || !graph->edge_off)
    HGNN_FAIL(HGNN_EINVAL, "NULL argument");
  *out = nullptr;
  const int T = ctx->T, R = ctx->R;
  for (int t = 0; t < T; ++t)
    if (graph->num_nodes[t] < 0 || graph->num_nodes[t] > INT32_MAX)
      HGNN_FAIL(HGNN_EINVAL, "num_nodes[%d]=%lld outside [0, 2^31)", t, (long long)graph->num_nodes[t]);
  if (graph->edge_off[0] != 0) HGNN_FAIL(HGNN_EINVAL, "edge_off[0] must be 0");
  for (int r = 0; r < R; ++r) {
    const int64_t n = graph->num_nodes[ctx->rel_dst[r]], e = graph->edge_off[r + 1] - graph->edge_off[r];
    if (e < 0 || !graph->in_indptr[r] || (e > 0 && !graph->in_nbr[r])) HGNN_FAIL(HGNN_EINVAL, "relation %d: bad edge range or NULL arrays", r);
    const int64_t *p = graph->in_indptr[r];
    if (p[0] != 0 || p[n] != e) HGNN_FAIL(HGNN_EINVAL, "relation %d: in_indptr does not span its %lld edges", r, (long long)e);
    for (int64_t v = 0; v < n; ++v)
      if (p[v + 1] < p[v]) HGNN_FAIL(HGNN_EINVAL, "relation %d: in_indptr decreases at vertex %lld", r, (long long)v);
    const int64_t ns = graph->num_nodes[ctx->rel_src[r]];
    const int32_t *nb = graph->in_nbr[r];
    for (int64_t i = 0; i < e; ++i)
      if (nb[i] < 0 || nb[i] >= ns) HGNN_FAIL(HGNN_EINVAL, "relation %d: in_nbr[%lld]=%d outside its source type", r, (long long)i, nb[i]);
  }
  hgnn_sampler *s = new (std::nothrow) hgnn_sampler();
  if (!s) HGNN_FAIL(HGNN_ENOMEM, "out of host memory");
  s->num_nodes.assign(graph->num_nodes, graph->num_nodes + T);
  s->edge_off.assign(graph->edge_off, graph->edge_off + R + 1);
  s->in_indptr.assign(graph->in_indptr, graph->in_indptr + R);
  s->in_nbr.assign(graph->in_nbr, graph->in_nbr + R);
  // the edge-type table of Algorithm 2, in its compact form: edge ids of relation r are one contiguous range
  std::vector<uint8_t> types((size_t)s->edge_off[R]);
  for (int r = 0; r < R; ++r)
    std::memset(types.data() + s->edge_off[r], r, (size_t)(s->edge_off[r + 1] - s->edge_off[r]));
  ctx->edge_types8.swap(types);
  ++ctx->types_version;
  index_edge_type_runs(ctx);
  *out = s;
  return HGNN_OK;
}

void hgnn_sampler_destroy(hgnn_ctx *ctx, hgnn_sampler *s) {
  (void)ctx;
  delete s;
}
