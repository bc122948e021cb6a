// bf16 forward GEMM of the mean layer on the LDS-DMA core (gemm_dma.h):  h_d = act([Z_r1 | Z_r1' | ... | X_d] . [W; W; ...] + b_d)
// with K-contiguous operands, as 256x128 tiles (one persistent block of 8 wavefronts per compute unit, three LDS stages)
// or 128x128 tiles (two blocks per compute unit, two stages).  An alternative to gemm_fwd_kernel that a context uses
// only when HGNN_DMA_GEMM is set in the environment: on the headline workload it measures 78-83 us against 67 us.
// The launcher returns false when a shape is outside what the kernel covers (widths that are no multiple of 8,
// more K-segments or K-steps than its LDS tables hold); the caller then runs the generic kernel.
#include <algorithm>
#include <cstdlib>
#include <cstring>

#include "gemm_dma.h"

namespace hgnn {

struct LiveMask2 {
  uint32_t w[kMaxR / 32];
};
// Where each group's K-segments sit in the LDS table, and how many K-steps they add up to.
template <int N> struct SegPlanN {
  uint16_t first[N + 1];
  uint16_t steps[N];
};
typedef SegPlanN<kMaxT> SegPlan;

template <int TM, int S>
__global__ void __launch_bounds__(dma::kThreads, S == 2 ? 2 : 1) gemm2_fwd_kernel(TypeTab tt, RelTab rt, PtrTab pt, WtTab wt, SegTab tiles, XcdMap xmap,
                                                                     SegPlan plan, LiveMask2 live, int H, int relu,
                                                                     const bf16 *__restrict__ x, const bf16 *__restrict__ z,
                                                                     const bf16 *__restrict__ zlo, const bf16 *__restrict__ wtb,
                                                                     bf16 *__restrict__ h) {
  constexpr int MI = TM / 128;
  __shared__ dma::Lds<TM, S> sm;
  // Per-type tables the tile loop indexes: copied from the kernel arguments (which sit in host memory: a first
  // touch of one of their cache lines costs a bus round trip) into LDS once, every thread an entry.
  __shared__ int s_tile_off[kMaxT + 1], s_n_dst[kMaxT], s_out_row_off[kMaxT];
  __shared__ uint16_t s_first[kMaxT + 1];
  __shared__ const bf16 *s_bias[kMaxT];
  const int R = rt.num_rels, T = tt.num_types;
  if (threadIdx.x <= T) {
    const int t = threadIdx.x;
    s_tile_off[t] = tiles.tile_off[t];
    s_first[t] = plan.first[t];
    if (t < T) {
      s_n_dst[t] = tt.n_dst[t];
      s_out_row_off[t] = tt.out_row_off[t];
      s_bias[t] = reinterpret_cast<const bf16 *>(pt.bias[t]);
    }
  }
  // K-segments of every destination type with rows: the aggregate of each relation ending in it that has an edge
  // (and its low-order plane, when the layer keeps one, against the same weights), then the root term.  Wavefront w
  // fills the types w, w + 8, ...; its lanes examine 64 relations at a time and pack the live ones with a ballot.
  {
    const int lane = threadIdx.x & 63, mult = zlo ? 2 : 1;
    for (int d = threadIdx.x >> 6; d < T; d += dma::kWaves) {
      if (tt.n_dst[d] == 0) continue;
      const int pos0 = plan.first[d];
      int cnt = 0;
      for (int cursor = 0; cursor < R; cursor += 64) {
        const int r = cursor + lane;
        bool use = r < R;
        if (use) use = rt.dst[r] == d && ((live.w[r >> 5] >> (r & 31)) & 1u);
        const unsigned long long m = __ballot(use);
        if (use) {
          const int pos = pos0 + (cnt + __popcll(m & ((1ull << lane) - 1ull))) * mult;
          const int F = tt.in_dim[rt.src[r]];
          const bf16 *B = wtb + (int64_t)wt.rel4[r] * 4;
          put_seg(sm.seg[pos], z + (int64_t)rt.z_off4[r] * 4, F, B, F, 0, F);
          if (zlo) put_seg(sm.seg[pos + 1], zlo + (int64_t)rt.z_off4[r] * 4, F, B, F, 0, F);
        }
        cnt += __popcll(m);
      }
      if (lane == 0 && pt.w_root[d]) {
        const int F = tt.in_dim[d];
        put_seg(sm.seg[pos0 + cnt * mult], x + tt.xroot_off[d], F, wtb + (int64_t)wt.root4[d] * 4, F, 0, F);
      }
    }
  }
  __syncthreads();
  // Persistent blocks: block b lives on XCD b % 8 (the hardware deals blocks out round-robin) and walks that XCD's
  // contiguous tile range in steps of the blocks per XCD.  (A block per tile leaves a compute unit idle between two
  // tiles: with ~150 KB of LDS only one block fits, and the next cannot be placed before this one has gone.)
  const int xcd = blockIdx.x & 7, per_xcd = gridDim.x >> 3;
  const int tile_first = xmap.first[xcd], tile_last = xmap.first[xcd + 1];
  const int tiles_n = (H + dma::TN - 1) / dma::TN;
  dma::run_tiles_kc<TM, S>(
      sm, tile_first + (blockIdx.x >> 3), tile_last, per_xcd,
      [&](int tile, dma::TilePlan &tp) {
        int d = 0;
        while (tile >= s_tile_off[d + 1]) ++d;
        const int local = tile - s_tile_off[d];
        tp.t.a_extent = s_n_dst[d];
        tp.t.a0 = (local / tiles_n) * TM;
        tp.t.b_extent = H;
        tp.t.b0 = (local % tiles_n) * dma::TN;
        tp.t.id = d;
        tp.seg_first = s_first[d];
        tp.nseg = s_first[d + 1] - s_first[d];
      },
      [&](f32x16(&acc)[MI][2], const dma::TileEnt &te) {
        const int d = te.id, m0 = te.a0, n0 = te.b0;
        const bf16 *bias = s_bias[d];
        const int wn = ((threadIdx.x >> 6) & 1) * 64;
        float bv[2];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          const int c = n0 + wn + j * 32 + (threadIdx.x & 31);
          bv[j] = (bias && c < H) ? to_float(bias[c]) : 0.f;
        }
        dma::store_tile_bf16<MI>(acc, h + ((int64_t)s_out_row_off[d] + m0) * H + n0, H, te.a_extent - m0, H - n0,
                                 [&](float v, int, int col) {
                                   const float o = v + bv[(col - wn) >> 5];
                                   return relu ? fmaxf(o, 0.f) : o;
                                 });
      });
}

// Compute units behind each of the 8 L2s of the current device (one persistent block per compute unit).
static int compute_units_per_xcd() {
  static int cached = 0;
  if (cached == 0) {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 8)
      cus = 256;
    cached = cus / 8;
  }
  return cached;
}

// Operand extents must keep byte offsets inside 32 bits (the loaders add them to a 64-bit base).
static bool fits32(int64_t rows, int64_t ld) { return rows * ld * 2 < ((int64_t)1 << 32); }

bool launch_gemm2_fwd(hipStream_t s, const TypeTab &tt, const RelTab &rt, const PtrTab &pt, const WtTab &wt, const uint32_t *live_mask,
                      int H, int relu, const void *x, const void *z, const void *zlo, const void *wt_buf, void *h, hgnn_status *st) {
  *st = HGNN_OK;
  const int T = tt.num_types;
  int64_t total_dst = 0;
  for (int t = 0; t < T; ++t) {
    if (tt.in_dim[t] % 8) return false;
    if (tt.in_dim[t] > 65535 || !fits32(tt.row_off[t + 1] - tt.row_off[t], tt.in_dim[t]) || !fits32(H, tt.in_dim[t])) return false;
    total_dst += tt.n_dst[t];
  }
  if (total_dst == 0) return true;
  LiveMask2 live;
  for (int i = 0; i < kMaxR / 32; ++i) live.w[i] = live_mask[i];
  // 256-row tiles when they still give every compute unit about two tiles, 128-row tiles otherwise
  const int tn = (H + dma::TN - 1) / dma::TN;
  int64_t t256 = 0;
  for (int t = 0; t < T; ++t) t256 += (int64_t)((tt.n_dst[t] + 255) / 256) * tn;
  const int TM = t256 >= 512 ? 256 : 128;
  SegTab tiles;
  std::memset(&tiles, 0, sizeof(tiles));
  tiles.num_segs = T;
  SegPlan plan;
  std::memset(&plan, 0, sizeof(plan));
  int64_t cost[kMaxT];
  for (int d = 0; d < T; ++d) {
    tiles.tile_off[d + 1] = tiles.tile_off[d] + ((tt.n_dst[d] + TM - 1) / TM) * tn;
    int steps = 0, segs = 0;
    if (tt.n_dst[d] > 0) {
      for (int r = 0; r < rt.num_rels; ++r)
        if (rt.dst[r] == d && ((live.w[r >> 5] >> (r & 31)) & 1u)) {
          steps += (zlo ? 2 : 1) * ((tt.in_dim[rt.src[r]] + dma::BK - 1) / dma::BK);
          segs += zlo ? 2 : 1;
        }
      if (pt.w_root[d]) {
        steps += (tt.in_dim[d] + dma::BK - 1) / dma::BK;
        ++segs;
      }
    }
    plan.first[d + 1] = (uint16_t)(plan.first[d] + segs);
    if (steps > dma::kStepList) return false;  // a tile's K-steps must fit the step list
    plan.steps[d] = (uint16_t)steps;
    cost[d] = steps + 1;  // K-steps plus the tile's epilogue
  }
  if (plan.first[T] > dma::kSegTable) return false;  // more K-segments than the LDS table holds
  XcdMap xmap;
  const int longest = balance_xcd(tiles.tile_off, cost, T, xmap) / 8;
  // 256-row tiles: one persistent block per compute unit with three LDS stages; 128-row tiles: two blocks per compute
  // unit with two stages each (an independent instruction stream beside each block hides its barriers and waits)
#define HGNN_FWD2(TM_, S_, BLOCKS_PER_CU)                                                                                      \
  HGNN_LAUNCH((gemm2_fwd_kernel<TM_, S_>), dim3(8 * std::min(longest, BLOCKS_PER_CU * compute_units_per_xcd())), dim3(dma::kThreads), \
              0, s, tt, rt, pt, wt, tiles, xmap, plan, live, H, relu, (const bf16 *)x, (const bf16 *)z, (const bf16 *)zlo,      \
              (const bf16 *)wt_buf, (bf16 *)h)
  if (TM == 256) HGNN_FWD2(256, 3, 1); else HGNN_FWD2(128, 2, 2);
#undef HGNN_FWD2
  if (hipGetLastError() != hipSuccess) {
    set_error("gemm2_fwd_kernel launch failed");
    *st = HGNN_EHIP;
  }
  return true;
}

}  // namespace hgnn
