// MFMA GEMMs of the layer path (gfx950, wave64):
//   forward : h_d = act( [Z_r1 | Z_r2 | ... | X_d] . [W_r1; W_r2; ...; W_0^d] + b_d )   per destination type d
//             -- projection and semantic fusion in one contraction (the K loop walks the relations that
//             end in d, then the root term), bias and activation in the epilogue;
//   dA      : dZ_s = (G' W_s^T) scaled per row by 1/|N_r(v)|                          per K-segment s
//   dW      : dW_s = A_s^T G'  (reduction over the destination rows, split and added atomically)
// One 256-thread block (2x2 wavefronts) computes a 128x128 tile; every wavefront owns 64x64 of it as
// 2x2 MFMA 32x32 accumulators.  The reduction runs as ONE flat sequence of K-steps over all segments of
// the tile, software-pipelined: operands go global -> registers -> LDS, the global loads of the next
// two K-steps are in flight while the current one is multiplied, and LDS is double-buffered so that a
// step costs one barrier.  An operand is kept in LDS the way it lies in memory: "KC" = the reduction
// index is contiguous (rows = output index), "KS" = the output index is contiguous.
// Every kernel exists in a FAST form (all operands 16-byte aligned: per-thread offsets are computed once
// per segment, a K-step is 8 vector loads from wave-uniform bases) and a generic form (element-wise,
// zero-filled loads) for unaligned shapes.
#include "bias_reduce.h"
#include "gemm_core.h"

namespace hgnn {

// ------------------------------------------------------------------------------------------
// Forward.  `live` has bit r set when relation r has at least one edge in this layer.
struct LiveMask {
  uint32_t w[kMaxR / 32];
};

template <typename T, bool FAST, int MI>
__global__ void __launch_bounds__(kThreads, MI == 1 ? 3 : 2) gemm_fwd_kernel(TypeTab tt, RelTab rt, PtrTab pt, WtTab wt, SegTab tiles, XcdMap xmap, LiveMask live,
                                                            int H, int relu, const T *__restrict__ x, const T *__restrict__ z,
                                                            const T *__restrict__ zlo, const T *__restrict__ wtb,
                                                            T *__restrict__ h, int only_seg,
                                                            float *__restrict__ acc32) {
  constexpr int BM = 64 * MI, BN = 64 * MI;
  __shared__ GemmLds<T, MI, MI> sm;
  __shared__ int s_nseg;
  const int R = rt.num_rels;
  const int tile = xcd_tile(xmap, blockIdx.x);
  if (tile < 0) return;
  int d = 0;
  while (tile >= tiles.tile_off[d + 1]) ++d;
  const int tiles_n = (H + BN - 1) / BN;
  const int local = tile - tiles.tile_off[d];
  const int m0 = (local / tiles_n) * BM, n0 = (local % tiles_n) * BN;
  const int M = tt.n_dst[d];
  f32x16 acc[MI][MI];
  zero_acc(acc);
  // K-segments of this destination type: the aggregate of every relation ending in d (and, when the layer keeps
  // it, the aggregate's low-order remainder against the same weights), then the root term.  The first wavefront
  // looks at a window of relations at once, one per lane, and packs the ones that take part with a ballot.
  for (int cursor = 0; cursor < R; cursor += kRelWindow) {
    if (threadIdx.x < 64) {
      const int lane = threadIdx.x, r = cursor + lane;
      bool use = lane < kRelWindow && r < R;
      if (use) use = rt.dst[r] == d && (only_seg < 0 || only_seg == r) && ((live.w[r >> 5] >> (r & 31)) & 1u);  // no edge: all zero
      const unsigned long long m = __ballot(use);
      const int mult = zlo ? 2 : 1;
      if (use) {
        const int pos = __popcll(m & ((1ull << lane) - 1ull)) * mult;
        const int F = tt.in_dim[rt.src[r]];
        const T *B = wtb + (int64_t)wt.rel4[r] * 4;
        put_seg(sm.seg[pos], z + (int64_t)rt.z_off4[r] * 4, F, B, F, 0, F);
        if (zlo) put_seg(sm.seg[pos + 1], zlo + (int64_t)rt.z_off4[r] * 4, F, B, F, 0, F);
      }
      if (lane == 0) {
        int n = __popcll(m) * mult;
        if (cursor + kRelWindow >= R && pt.w_root[d] && (only_seg < 0 || only_seg == R + d)) {
          const int F = tt.in_dim[d];
          put_seg(sm.seg[n++], x + tt.xroot_off[d], F, wtb + (int64_t)wt.root4[d] * 4, F, 0, F);
        }
        s_nseg = n;
      }
    }
    __syncthreads();
    gemm_run<T, FAST, true, true>(acc, sm, s_nseg, M, m0, H, n0);
  }
  const int64_t orow = tt.out_row_off[d];
  if (acc32) {
    HGNN_FOR_EACH_ACC({
      if (m0 + row < M && n0 + col < H) acc32[(orow + m0 + row) * H + n0 + col] += val;
    })
    return;
  }
  const T *bias = reinterpret_cast<const T *>(pt.bias[d]);
  float bv[MI];
  const int wn0 = ((threadIdx.x >> 6) & 1) * 32 * MI;
#pragma unroll
  for (int j = 0; j < MI; ++j) {
    const int c = n0 + wn0 + j * 32 + (threadIdx.x & 31);
    bv[j] = (bias && c < H) ? to_float(bias[c]) : 0.f;
  }
  write_tile(acc, sm, h + (orow + m0) * H + n0, H, M - m0, H - n0, [&](float v, int, int col) {
    const float o = v + bv[(col - wn0) >> 5];
    return relu ? fmaxf(o, 0.f) : o;
  });
}

hgnn_status launch_gemm_fwd(hipStream_t s, int dtype, const LayerDev &L, const TypeTab &tt, const RelTab &rt,
                            const PtrTab &pt, const WtTab &wt, const SegTab &tiles, const uint32_t *live_mask, int H,
                            int relu, const void *x, const void *z, const void *zlo, const void *wt_buf, void *h,
                            int only_seg, float *acc32, int tile_mn) {
  const int n = tiles.tile_off[tt.num_types];
  if (n == 0) return HGNN_OK;
  (void)L;
  LiveMask live;
  for (int i = 0; i < kMaxR / 32; ++i) live.w[i] = live_mask[i];
  // A tile's cost: its K-steps (destination types differ in the number of relations that end in them) plus
  // the fixed part (segment table, pipeline fill, epilogue), which is worth about four K-steps.
  int64_t cost[kMaxT];
  const int bk = dtype == HGNN_BF16 ? Mma<bf16>::BK : Mma<float>::BK;
  for (int d = 0; d < tt.num_types; ++d) {
    int64_t steps = 0;
    for (int r = 0; r < rt.num_rels; ++r)
      if (rt.dst[r] == d && (only_seg < 0 || only_seg == r) && ((live.w[r >> 5] >> (r & 31)) & 1u))
        steps += (zlo ? 2 : 1) * ((tt.in_dim[rt.src[r]] + bk - 1) / bk);
    if (pt.w_root[d] && (only_seg < 0 || only_seg == rt.num_rels + d)) steps += (tt.in_dim[d] + bk - 1) / bk;
    cost[d] = steps + 4;
  }
  XcdMap xmap;
  dim3 grid(balance_xcd(tiles.tile_off, cost, tt.num_types, xmap));
  // operands of the forward are the library's own aligned buffers (aggregates, transposed weights) and
  // x_merged, whose row widths are multiples of 16 bytes: always the FAST form
#define HGNN_FWD(TY, MI_)                                                                                        \
  HGNN_LAUNCH((gemm_fwd_kernel<TY, true, MI_>), grid, dim3(kThreads), 0, s, tt, rt, pt, wt, tiles, xmap, live, H, relu, \
              (const TY *)x, (const TY *)z, (const TY *)zlo, (const TY *)wt_buf, (TY *)h, only_seg, acc32)
  if (dtype == HGNN_BF16) {
    if (tile_mn == 64) HGNN_FWD(bf16, 1); else HGNN_FWD(bf16, 2);
  } else {
    if (tile_mn == 64) HGNN_FWD(float, 1); else HGNN_FWD(float, 2);
  }
#undef HGNN_FWD
  HGNN_HIP(hipGetLastError());
  return HGNN_OK;
}

// ------------------------------------------------------------------------------------------
__device__ __forceinline__ int find_seg(const SegTab &tiles, int tile) {
  int lo = 0, hi = tiles.num_segs;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (tiles.tile_off[mid] <= tile) lo = mid; else hi = mid;
  }
  return lo;
}

// dZ_s = (G' W_s^T) / deg.  G' has leading dimension ldg (>= H; the columns H..ldg-1 are zero), and so have
// the weights handed in through `pt` (the caller's own when H is a multiple of 16 bytes, zero-padded copies
// otherwise), so that the reduction simply runs over ldg.
// One tile of dZ_seg: destination rows m0.., columns n0.. of the segment's input width.
template <typename T, bool FAST, int MI>
__device__ __forceinline__ void da_tile_at(GemmLds<T, MI, MI> &sm, int seg, int m0, int n0, const LayerDev &L, const TypeTab &tt,
                                           const RelTab &rt, const PtrTab &pt, int ldg, const T *__restrict__ gp,
                                           T *__restrict__ dz) {
  constexpr int BM = 64 * MI;
  const int R = rt.num_rels;
  const bool is_rel = seg < R;
  const int d = is_rel ? rt.dst[seg] : seg - R;
  const int F = tt.in_dim[is_rel ? rt.src[seg] : d];
  const T *W = reinterpret_cast<const T *>(is_rel ? pt.w_rel[seg] : pt.w_root[d]);
  const int M = tt.n_dst[d];
  f32x16 acc[MI][MI];
  zero_acc(acc);
  if (threadIdx.x == 0) put_seg(sm.seg[0], gp + (int64_t)tt.out_row_off[d] * ldg, ldg, W, ldg, 0, ldg);
  if (threadIdx.x < BM) {  // 1/|N_r(v)| of the tile's rows (1 for the root term)
    float sc = 1.f;
    const int row = m0 + threadIdx.x;
    if (is_rel && row < M) {
      const int rho = L.rel_row_off[seg] + row;
      const int deg = L.rowptr[rho + 1] - L.rowptr[rho];
      sc = deg > 0 ? 1.f / (float)deg : 0.f;
    }
    sm.rowscale[threadIdx.x] = sc;
  }
  __syncthreads();
  gemm_run<T, FAST, true, true>(acc, sm, 1, M, m0, F, n0);
  T *out = dz + (int64_t)(is_rel ? rt.z_off4[seg] : rt.zroot_off4[d]) * 4;
  write_tile(acc, sm, out + (int64_t)m0 * F + n0, F, M - m0, F - n0,
             [&](float v, int row, int) { return v * sm.rowscale[row]; });
}

// Tiles in segment order (all row blocks of a segment, then the next segment).
template <typename T, bool FAST, int MI>
__device__ __forceinline__ void da_tile(GemmLds<T, MI, MI> &sm, int bid, int nblocks, const LayerDev &L, const TypeTab &tt,
                                        const RelTab &rt, const PtrTab &pt, const SegTab &tiles, int ldg,
                                        const T *__restrict__ gp, T *__restrict__ dz) {
  constexpr int BM = 64 * MI, BN = 64 * MI;
  const int tile = xcd_tile(bid, nblocks);
  const int R = rt.num_rels;
  if (tile >= tiles.tile_off[tiles.num_segs]) return;
  const int seg = find_seg(tiles, tile);
  const bool is_rel = seg < R;
  const int F = tt.in_dim[is_rel ? rt.src[seg] : seg - R];
  const int tiles_n = (F + BN - 1) / BN;
  const int local = tile - tiles.tile_off[seg];
  da_tile_at<T, FAST, MI>(sm, seg, (local / tiles_n) * BM, (local % tiles_n) * BN, L, tt, rt, pt, ldg, gp, dz);
}

// Tiles grouped by destination type and row block (the DwTab's `u` then runs over the column blocks of all the
// type's segments): the tiles that read the same 128 rows of G' are neighbours, in one XCD, and fetch them once.
template <typename T, bool FAST, int MI>
__device__ __forceinline__ void da_tile_grouped(GemmLds<T, MI, MI> &sm, int bid, int nblocks, const LayerDev &L, const TypeTab &tt,
                                                const RelTab &rt, const PtrTab &pt, const DwTab &tiles, int ldg,
                                                const T *__restrict__ gp, T *__restrict__ dz) {
  constexpr int BM = 64 * MI, BN = 64 * MI;
  const int tile = xcd_tile(bid, nblocks);
  if (tile >= tiles.tile_off[tt.num_types]) return;
  int d = 0;
  while (tile >= tiles.tile_off[d + 1]) ++d;
  const int local = tile - tiles.tile_off[d];
  const int u = local % tiles.u_total[d], mt = local / tiles.u_total[d];
  int e = tiles.first[d];
  while (e + 1 < tiles.first[d + 1] && u >= tiles.u_off[e + 1]) ++e;
  da_tile_at<T, FAST, MI>(sm, tiles.seg[e], mt * BM, (u - tiles.u_off[e]) * BN, L, tt, rt, pt, ldg, gp, dz);
}

template <typename T, bool FAST, int MI>
__global__ void __launch_bounds__(kThreads, MI == 1 ? 4 : 2) gemm_da_kernel(LayerDev L, TypeTab tt, RelTab rt, PtrTab pt, SegTab tiles, int ldg,
                                                           const T *__restrict__ gp, T *__restrict__ dz) {
  __shared__ GemmLds<T, MI, MI> sm;
  da_tile<T, FAST, MI>(sm, blockIdx.x, gridDim.x, L, tt, rt, pt, tiles, ldg, gp, dz);
}

hgnn_status launch_gemm_da(hipStream_t s, int dtype, const LayerDev &L, const TypeTab &tt, const RelTab &rt,
                           const PtrTab &pt, const SegTab &tiles, int ldg, bool fast, const void *gp, void *dz) {
  const int n = tiles.tile_off[tiles.num_segs];
  if (n == 0) return HGNN_OK;
  dim3 grid(round_up8(n)), blk(kThreads);
#define HGNN_DA(TY, FA, MI_) \
  HGNN_LAUNCH((gemm_da_kernel<TY, FA, MI_>), grid, blk, 0, s, L, tt, rt, pt, tiles, ldg, (const TY *)gp, (TY *)dz)
#define HGNN_DA2(TY, FA) { HGNN_DA(TY, FA, 2); }
  if (dtype == HGNN_BF16) {
    if (fast) HGNN_DA2(bf16, true) else HGNN_DA2(bf16, false)
  } else {
    if (fast) HGNN_DA2(float, true) else HGNN_DA2(float, false)
  }
#undef HGNN_DA2
#undef HGNN_DA
  HGNN_HIP(hipGetLastError());
  return HGNN_OK;
}

// ------------------------------------------------------------------------------------------
// dW_s += A_s^T G' over the destination-row slice [k_begin, k_end) of this block.
template <typename T, bool FAST, int MI>
__device__ __forceinline__ void dw_tile(GemmLds<T, MI, MI> &sm, int bid, const TypeTab &tt, const RelTab &rt,
                                        const GradPtrTab &gt, const DwTab &tiles, const XcdMap &xmap, int split_rows, int H,
                                        int ldg, const T *__restrict__ x, const T *__restrict__ z,
                                        const T *__restrict__ gp) {
  constexpr int BM = 64 * MI, BN = 64 * MI;
  const int tile = xcd_tile(xmap, bid);
  const int R = rt.num_rels;
  if (tile < 0) return;
  int d = 0;
  while (tile >= tiles.tile_off[d + 1]) ++d;
  // inside the type: row slice, then block of dW rows over the type's segments, then column block
  const int tiles_h = (H + BN - 1) / BN;
  int local = tile - tiles.tile_off[d];
  const int th = local % tiles_h;
  local /= tiles_h;
  const int u = local % tiles.u_total[d];
  const int sp = local / tiles.u_total[d];
  int e = tiles.first[d];
  while (e + 1 < tiles.first[d + 1] && u >= tiles.u_off[e + 1]) ++e;
  const int seg = tiles.seg[e];
  const int tf = u - tiles.u_off[e];
  const bool is_rel = seg < R;
  const int F = tt.in_dim[is_rel ? rt.src[seg] : d];
  float *dW = is_rel ? gt.dw_rel[seg] : gt.dw_root[d];
  const int M = tt.n_dst[d];
  const int f0 = tf * BM, h0 = th * BN;
  const int k_begin = sp * split_rows, k_end = min(M, k_begin + split_rows);
  f32x16 acc[MI][MI];
  zero_acc(acc);
  if (threadIdx.x == 0)
    put_seg(sm.seg[0], is_rel ? z + (int64_t)rt.z_off4[seg] * 4 : x + tt.xroot_off[d], F,
            gp + (int64_t)tt.out_row_off[d] * ldg, ldg, k_begin, k_end);
  __syncthreads();
  gemm_run<T, FAST, false, false>(acc, sm, 1, F, f0, ldg, h0);
  HGNN_FOR_EACH_ACC({
    if (f0 + row < F && h0 + col < H) atomicAdd(dW + (int64_t)(f0 + row) * H + h0 + col, val);
  })
}

template <typename T, bool FAST, int MI>
__global__ void __launch_bounds__(kThreads, MI == 1 ? 4 : 2) gemm_dw_kernel(TypeTab tt, RelTab rt, GradPtrTab gt, DwTab tiles, XcdMap xmap, int split_rows, int H,
                                                           int ldg, const T *__restrict__ x, const T *__restrict__ z,
                                                           const T *__restrict__ gp) {
  __shared__ GemmLds<T, MI, MI> sm;
  dw_tile<T, FAST, MI>(sm, blockIdx.x, tt, rt, gt, tiles, xmap, split_rows, H, ldg, x, z, gp);
}

// Both backward GEMMs of a layer in ONE launch: the first n_dw blocks compute weight-gradient tiles (long
// reductions), the others input-gradient tiles (short ones).  Each kernel alone leaves compute units idle at its
// end -- the weight gradient has fewer tiles than the chip has block slots -- and the other one's tiles fill them.
// The last n_bias blocks (when bpart is given) add up the partial bias-gradient sums that the row pass over G'
// left: a few microseconds of work that would otherwise be a launch of its own.
template <typename T, bool FAST>
__global__ void __launch_bounds__(kThreads, 2) gemm_bwd_kernel(LayerDev L, TypeTab tt, RelTab rt, PtrTab pt, DwTab da_tiles,
                                                            GradPtrTab gt, DwTab dw_tiles, XcdMap xmap, int n_dw, int split_rows,
                                                            int H, int ldg, const T *__restrict__ x, const T *__restrict__ z,
                                                            const T *__restrict__ gp, T *__restrict__ dz,
                                                            const float *__restrict__ bpart, int rpb, int n_bias) {
  __shared__ GemmLds<T, 2, 2> sm;
  const int n_gemm = (int)gridDim.x - n_bias;
  if ((int)blockIdx.x >= n_gemm) {
    bias_reduce_part(tt, gt, H, rpb, bpart, (int)blockIdx.x - n_gemm);
    return;
  }
  if ((int)blockIdx.x < n_dw) dw_tile<T, FAST, 2>(sm, blockIdx.x, tt, rt, gt, dw_tiles, xmap, split_rows, H, ldg, x, z, gp);
  else da_tile_grouped<T, FAST, 2>(sm, blockIdx.x - n_dw, n_gemm - n_dw, L, tt, rt, pt, da_tiles, ldg, gp, dz);
}

static int dw_blocks(int dtype, const TypeTab &tt, const DwTab &tiles, int split_rows, XcdMap &xmap) {
  // a tile's cost: the K-steps of its row slice (the average over the type's slices) plus the fixed part
  int64_t cost[kMaxT];
  const int bk = dtype == HGNN_BF16 ? Mma<bf16>::BK : Mma<float>::BK;
  for (int d = 0; d < tt.num_types; ++d) {
    const int64_t slices = (tt.n_dst[d] + split_rows - 1) / split_rows;
    cost[d] = 4 + (slices > 0 ? (tt.n_dst[d] / slices + bk - 1) / bk : 0);
  }
  return balance_xcd(tiles.tile_off, cost, tt.num_types, xmap);
}

hgnn_status launch_gemm_bwd(hipStream_t s, int dtype, const LayerDev &L, const TypeTab &tt, const RelTab &rt,
                            const PtrTab &pt, const DwTab &da_tiles, const GradPtrTab &gt, const DwTab &dw_tiles,
                            int split_rows, int H, int ldg, bool fast, const void *x, const void *z, const void *gp, void *dz,
                            const float *bpart, int rpb) {
  XcdMap xmap;
  const int n_dw = dw_blocks(dtype, tt, dw_tiles, split_rows, xmap);
  const int n_da = round_up8(da_tiles.tile_off[tt.num_types]);
  const int n_bias = bpart ? bias_reduce_blocks(tt.num_types, H) : 0;
  dim3 grid(n_dw + n_da + n_bias), blk(kThreads);
#define HGNN_BWD(TY, FA)                                                                                             \
  HGNN_LAUNCH((gemm_bwd_kernel<TY, FA>), grid, blk, 0, s, L, tt, rt, pt, da_tiles, gt, dw_tiles, xmap, n_dw, split_rows, H, \
              ldg, (const TY *)x, (const TY *)z, (const TY *)gp, (TY *)dz, bpart, rpb, n_bias)
  if (dtype == HGNN_BF16) {
    if (fast) HGNN_BWD(bf16, true); else HGNN_BWD(bf16, false);
  } else {
    if (fast) HGNN_BWD(float, true); else HGNN_BWD(float, false);
  }
#undef HGNN_BWD
  HGNN_HIP(hipGetLastError());
  return HGNN_OK;
}

hgnn_status launch_gemm_dw(hipStream_t s, int dtype, const LayerDev &L, const TypeTab &tt, const RelTab &rt,
                           const GradPtrTab &gt, const DwTab &tiles, int split_rows, int H, int ldg, bool fast,
                           const void *x, const void *z, const void *gp) {
  const int n = tiles.tile_off[tt.num_types];
  if (n == 0) return HGNN_OK;
  (void)L;
  XcdMap xmap;
  dim3 grid(dw_blocks(dtype, tt, tiles, split_rows, xmap)), blk(kThreads);
#define HGNN_DW(TY, FA, MI_)                                                                                  \
  HGNN_LAUNCH((gemm_dw_kernel<TY, FA, MI_>), grid, blk, 0, s, tt, rt, gt, tiles, xmap, split_rows, H, ldg, (const TY *)x, \
              (const TY *)z, (const TY *)gp)
#define HGNN_DW2(TY, FA) { HGNN_DW(TY, FA, 2); }
  if (dtype == HGNN_BF16) {
    if (fast) HGNN_DW2(bf16, true) else HGNN_DW2(bf16, false)
  } else {
    if (fast) HGNN_DW2(float, true) else HGNN_DW2(float, false)
  }
#undef HGNN_DW2
#undef HGNN_DW
  HGNN_HIP(hipGetLastError());
  return HGNN_OK;
}

}  // namespace hgnn
