// Host-only stress of the runtime's threaded parts, for runs under -fsanitize=thread / address: many index builds
// in flight at once over several builders (pooled buffers, queue, condition variables), from two calling threads,
// with views read and graphs released while others are still being built; then the same with mini-batches sampled
// in the loop.  Every build is checked against a single-threaded reference written out here (stable grouping by
// relation and destination), so a race that corrupts an array fails the run even without a sanitizer report.
#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <random>
#include <thread>
#include <vector>

#include "../../include/hgnn.h"

#define CHECK(x)                                                                      \
  do {                                                                                \
    if (!(x)) {                                                                       \
      std::fprintf(stderr, "FAILED %s:%d: %s (%s)\n", __FILE__, __LINE__, #x, hgnn_last_error()); \
      std::exit(1);                                                                   \
    }                                                                                 \
  } while (0)

struct Batch {
  std::vector<int64_t> ei, n_src, n_dst;
  std::vector<int32_t> et;
  int64_t E;
};

static const int T = 3, R = 5;
static const int32_t rel_src[R] = {0, 1, 1, 2, 0}, rel_dst[R] = {1, 0, 1, 1, 2};

static Batch make_batch(unsigned seed) {
  std::mt19937 rng(seed);
  Batch b;
  b.n_src = {int64_t(200 + rng() % 300), int64_t(300 + rng() % 300), int64_t(50 + rng() % 100)};
  b.n_dst = {int64_t(20 + rng() % 100), int64_t(30 + rng() % 150), int64_t(10 + rng() % 40)};
  b.E = 3000 + rng() % 4000;
  b.ei.resize(2 * b.E);
  b.et.resize(b.E);
  for (int64_t e = 0; e < b.E; ++e) {
    const int r = rng() % R;
    b.et[e] = r;
    b.ei[e] = rng() % b.n_src[rel_src[r]];
    b.ei[b.E + e] = rng() % b.n_dst[rel_dst[r]];
  }
  return b;
}

static void check_graph(hgnn_ctx *ctx, hgnn_graph *g, const Batch &b) {
  hgnn_csr_view v;
  CHECK(hgnn_graph_host_view(ctx, g, 0, &v) == HGNN_OK);
  int64_t row_off[T + 1] = {0}, rel_row_off[R + 1] = {0};
  for (int t = 0; t < T; ++t) row_off[t + 1] = row_off[t] + b.n_src[t];
  for (int r = 0; r < R; ++r) rel_row_off[r + 1] = rel_row_off[r] + b.n_dst[rel_dst[r]];
  CHECK(v.rows == rel_row_off[R] && v.edges == b.E);
  std::vector<int64_t> order(b.E);
  for (int64_t e = 0; e < b.E; ++e) order[e] = e;
  std::stable_sort(order.begin(), order.end(), [&](int64_t x, int64_t y) {
    const int64_t kx = rel_row_off[b.et[x]] + b.ei[b.E + x], ky = rel_row_off[b.et[y]] + b.ei[b.E + y];
    return kx < ky;
  });
  int64_t k = 0;
  for (int64_t rho = 0; rho < v.rows; ++rho) {
    CHECK(v.rowptr[rho] == k);
    while (k < b.E && rel_row_off[b.et[order[k]]] + b.ei[b.E + order[k]] == rho) {
      const int64_t e = order[k];
      CHECK(v.colidx[k] == row_off[rel_src[b.et[e]]] + b.ei[e]);
      if (v.perm) CHECK(v.perm[k] == e);
      ++k;
    }
  }
  CHECK(v.rowptr[v.rows] == b.E);
  // transpose: every entry's row lists the column it sits under
  for (int64_t c = 0; c < v.src_rows; ++c)
    for (int64_t j = v.cptr[c]; j < v.cptr[c + 1]; ++j) {
      const int32_t rho = v.crow[j];
      bool found = false;
      for (int32_t q = v.rowptr[rho]; q < v.rowptr[rho + 1] && !found; ++q) found = v.colidx[q] == c;
      CHECK(found);
    }
  CHECK(v.cptr[v.src_rows] == v.transpose_edges);
}

int main() {
  hgnn_schema sch = {T, R, rel_src, rel_dst, 1, HGNN_AGG_MEAN, HGNN_FUSE_SUM, HGNN_F32};
  for (int pass = 0; pass < 2; ++pass) {
    hgnn_ctx *ctx = nullptr;
    // pass 0: 4 builders of 2 threads each (parallel phases inside a build); pass 1: 6 single-threaded builders
    CHECK(hgnn_create(&ctx, &sch, -1, pass == 0 ? 8 : 6, pass == 0 ? 4 : 6) == HGNN_OK);
    CHECK(hgnn_set_build_permutation(ctx, pass == 0) == HGNN_OK);
    auto caller = [&](unsigned seed0) {
      std::vector<Batch> batches;
      for (int i = 0; i < 24; ++i) batches.push_back(make_batch(seed0 + i));
      std::vector<hgnn_graph *> graphs(batches.size(), nullptr);
      for (size_t i = 0; i < batches.size(); ++i) {
        Batch &b = batches[i];
        hgnn_coo_layer L = {};
        L.num_edges = b.E;
        L.edge_index = b.ei.data();
        L.index_is_i64 = 1;
        L.edge_type = b.et.data();
        L.n_src = b.n_src.data();
        L.n_dst = b.n_dst.data();
        CHECK(hgnn_build_semantic_csr(ctx, 1, &L, &graphs[i]) == HGNN_OK);
        if (i >= 6) {  // check and release an older one while newer ones are being built
          check_graph(ctx, graphs[i - 6], batches[i - 6]);
          hgnn_graph_release(ctx, graphs[i - 6]);
          graphs[i - 6] = nullptr;
        }
      }
      for (size_t i = 0; i < batches.size(); ++i)
        if (graphs[i]) {
          check_graph(ctx, graphs[i], batches[i]);
          hgnn_graph_release(ctx, graphs[i]);
        }
    };
    std::thread t1(caller, 1000u + 100u * pass), t2(caller, 5000u + 100u * pass);
    t1.join();
    t2.join();

    // sampling in the loop: a small graph, many mini-batches in flight
    std::mt19937 rng(7 + pass);
    std::vector<int64_t> num_nodes = {400, 500, 120};
    std::vector<std::vector<int64_t>> indptr(R);
    std::vector<std::vector<int32_t>> nbr(R);
    std::vector<int64_t> edge_off(R + 1, 0);
    for (int r = 0; r < R; ++r) {
      indptr[r].push_back(0);
      for (int64_t v = 0; v < num_nodes[rel_dst[r]]; ++v) {
        const int deg = rng() % 9;
        std::vector<int32_t> s;
        while ((int)s.size() < deg) {
          const int32_t u = rng() % num_nodes[rel_src[r]];
          if (std::find(s.begin(), s.end(), u) == s.end()) s.push_back(u);
        }
        nbr[r].insert(nbr[r].end(), s.begin(), s.end());
        indptr[r].push_back((int64_t)nbr[r].size());
      }
      edge_off[r + 1] = edge_off[r] + (int64_t)nbr[r].size();
    }
    std::vector<const int64_t *> ip(R);
    std::vector<const int32_t *> nb(R);
    for (int r = 0; r < R; ++r) {
      ip[r] = indptr[r].data();
      nb[r] = nbr[r].data();
    }
    hgnn_host_graph hg = {num_nodes.data(), ip.data(), nb.data(), edge_off.data()};
    hgnn_sampler *sm = nullptr;
    CHECK(hgnn_sampler_create(ctx, &hg, &sm) == HGNN_OK);
    const int32_t fanouts[2] = {4, 3};
    std::vector<hgnn_graph *> sg;
    for (int i = 0; i < 40; ++i) {
      std::vector<int64_t> targets;
      for (int64_t v = (i * 7) % 50; (int)targets.size() < 32; v += 3) targets.push_back(v % num_nodes[1]);
      std::sort(targets.begin(), targets.end());
      targets.erase(std::unique(targets.begin(), targets.end()), targets.end());
      hgnn_graph *g = nullptr;
      CHECK(hgnn_sample_and_build(ctx, sm, 1, targets.data(), (int64_t)targets.size(), 2, fanouts, 1000 + i, nullptr, &g) == HGNN_OK);
      sg.push_back(g);
      if (i >= 8) {
        int64_t n_rows[T];
        CHECK(hgnn_graph_ids(ctx, sg[i - 8], n_rows, nullptr, nullptr) == HGNN_OK);
        hgnn_csr_view v;
        CHECK(hgnn_graph_host_view(ctx, sg[i - 8], 0, &v) == HGNN_OK);
        CHECK(v.rowptr[v.rows] == v.edges && n_rows[1] >= 1);
        hgnn_graph_release(ctx, sg[i - 8]);
        sg[i - 8] = nullptr;
      }
    }
    for (hgnn_graph *g : sg)
      if (g) {
        CHECK(hgnn_graph_wait(ctx, g) == HGNN_OK);
        hgnn_graph_release(ctx, g);
      }
    hgnn_sampler_destroy(ctx, sm);
    hgnn_destroy(ctx);
  }
  std::puts("host stress ok");
  return 0;
}
