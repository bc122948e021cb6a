// Gather-mean over the merged CSR and its transpose for the common case that every vertex type has the
// same feature width F (then row i of x_merged / of the aggregate starts at i * F and no per-row relation
// lookup is needed).  These are the HBM-bound kernels of the path (the paper's merged aggregation,
// Algorithm 1, evaluated without materialising per-edge feature copies).
//
// A wavefront owns 64/LPR consecutive rows (LPR = lanes per row, each lane moving C 16-byte pieces of a
// feature row).  The rows of a wavefront are consecutive in the CSR, so their edges are one contiguous
// range: the wave loads its row pointers with one load, its column indices with one or two coalesced
// loads, and hands the indices to the lanes that need them through cross-lane reads.  All feature-row
// loads of up to four edges are then in flight together.  Dependent round trips per wave: row pointers,
// indices, features -- three, however many rows and edges it owns.
#include <cstring>
#include <type_traits>

#include "common.h"
#include "device_types.h"
#include "transpose_jobs.h"

namespace hgnn {

// Column index of wave-relative edge `rel` (0 = first edge of the wave), from the two index registers.
__device__ __forceinline__ int wave_col(int c0, int c1, int rel) {
  const int r = min(max(rel, 0), 127);
  const int a = __shfl(c0, r & 63), b = __shfl(c1, r & 63);
  return r < 64 ? a : b;
}

// Source of wave-relative edge `rel` when the edges carry row ADDRESSES (two 64-bit index registers).
__device__ __forceinline__ unsigned long long wave_addr(unsigned long long c0, unsigned long long c1, int rel) {
  const int r = min(max(rel, 0), 127);
  const unsigned long long a = __shfl(c0, r & 63), b = __shfl(c1, r & 63);
  return r < 64 ? a : b;
}

// ADDR = false: `colidx` holds rows of x.  ADDR = true: `colidx` is unused and `gaddr` holds, per edge, the device
// address of the source row (in whichever per-type feature store it lives), so that no merged copy of the source
// rows is needed.
template <typename T, int LPRL, int C, bool ADDR>
__global__ void __launch_bounds__(256, (C <= 2 && !ADDR) ? 8 : 1) spmm_fwd_uniform_kernel(const int32_t *__restrict__ rowptr, const int32_t *__restrict__ colidx,
                                                                const unsigned long long *__restrict__ gaddr,
                                                                const T *__restrict__ x, T *__restrict__ z, T *__restrict__ zlo,
                                                                int F, int row_begin, int row_end, TransposeJobs tj) {
  using V = Vec16<T>;
  using Idx = std::conditional_t<ADDR, unsigned long long, int>;
  constexpr int LPR = 1 << LPRL, RPW = 64 / LPR;
  // The first tj.blocks blocks transpose the layer's weights for the GEMM that follows this launch: a few
  // microseconds of work that would otherwise be a launch of its own in front of this one.
  __shared__ T tile[32][33];
  if ((int)blockIdx.x < tj.blocks) {
    transpose_jobs_block<T>(tj, blockIdx.x, tj.blocks, tile);
    return;
  }
  const int lane = threadIdx.x & 63;
  const int row0 = row_begin + (((int)blockIdx.x - tj.blocks) * 4 + (threadIdx.x >> 6)) * RPW;
  if (row0 >= row_end) return;  // whole wave
  const int nrows = min(RPW, row_end - row0);
  const int rp = rowptr[row0 + min(lane, nrows)];
  const int e0 = __shfl(rp, 0), eN = __shfl(rp, nrows);
  Idx c0 = 0, c1 = 0;
  if constexpr (ADDR) {
    if (e0 + lane < eN) c0 = gaddr[e0 + lane];
    if (e0 + 64 + lane < eN) c1 = gaddr[e0 + 64 + lane];
  } else {
    if (e0 + lane < eN) c0 = colidx[e0 + lane];
    if (e0 + 64 + lane < eN) c1 = colidx[e0 + 64 + lane];
  }
  const int g = lane >> LPRL, sub = lane & (LPR - 1);
  const int beg = __shfl(rp, min(g, nrows)), end = __shfl(rp, min(g + 1, nrows));
  const int len = end - beg;
  int maxlen = len;
#pragma unroll
  for (int o = 32; o >= LPR; o >>= 1) maxlen = max(maxlen, __shfl_xor(maxlen, o));
  const int nvec = F / V::N;
  const uint4 *xb = reinterpret_cast<const uint4 *>(x);
  float acc[C][V::N];
#pragma unroll
  for (int p = 0; p < C; ++p)
#pragma unroll
    for (int i = 0; i < V::N; ++i) acc[p][i] = 0.f;
  for (int i = 0; i < maxlen; i += 4) {  // same trip count for every lane: the cross-lane reads need all lanes
    Idx col[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if constexpr (ADDR) col[j] = wave_addr(c0, c1, beg - e0 + i + j);
      else col[j] = wave_col(c0, c1, beg - e0 + i + j);
    }
    uint4 v[4][C];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const bool on = i + j < len;
      Idx cj = col[j];
      if (on && beg - e0 + i + j >= 128) {  // beyond the two index registers
        if constexpr (ADDR) cj = gaddr[beg + i + j];
        else cj = colidx[beg + i + j];
      }
#pragma unroll
      for (int p = 0; p < C; ++p) {
        const int q = sub + p * LPR;
        if constexpr (ADDR)
          v[j][p] = (on && q < nvec) ? reinterpret_cast<const uint4 *>(cj)[q] : make_uint4(0, 0, 0, 0);
        else
          v[j][p] = (on && q < nvec) ? xb[(int64_t)cj * nvec + q] : make_uint4(0, 0, 0, 0);
      }
    }
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int p = 0; p < C; ++p) V::add(acc[p], v[j][p]);
  }
  if (g >= nrows) return;
  const float inv = len > 0 ? 1.0f / (float)len : 0.0f;
  const int64_t zoff = (int64_t)(row0 + g) * F;
#pragma unroll
  for (int p = 0; p < C; ++p) {
    const int q = sub + p * LPR;
    if (q >= nvec) continue;
#pragma unroll
    for (int i = 0; i < V::N; ++i) acc[p][i] *= inv;
    const uint4 hi = V::pack(acc[p]);
    reinterpret_cast<uint4 *>(z + zoff)[q] = hi;
    if (zlo) reinterpret_cast<uint4 *>(zlo + zoff)[q] = V::pack_remainder(acc[p], hi);
  }
}

template <typename T, int LPRL, int C>
static void launch_fwd_uniform(hipStream_t s, const LayerDev &L, const void *x, const unsigned long long *gaddr, void *z, void *zlo, int F,
                               int row_begin, int row_end, const TransposeJobs &tj) {
  constexpr int RPB = 4 * (64 >> LPRL);
  dim3 grid(tj.blocks + (row_end - row_begin + RPB - 1) / RPB);
  if (gaddr)
    HGNN_LAUNCH((spmm_fwd_uniform_kernel<T, LPRL, C, true>), grid, dim3(256), 0, s, L.rowptr, L.colidx, gaddr, (const T *)x, (T *)z,
                (T *)zlo, F, row_begin, row_end, tj);
  else
    HGNN_LAUNCH((spmm_fwd_uniform_kernel<T, LPRL, C, false>), grid, dim3(256), 0, s, L.rowptr, L.colidx, gaddr, (const T *)x, (T *)z,
                (T *)zlo, F, row_begin, row_end, tj);
}

// Returns false when the shape is outside what the uniform kernels cover (the generic kernels then run).
// Lanes per row and 16-byte pieces per lane, measured per width on the headline's two layers: the forward's rows
// are up to `fanout` long and run best with more rows per wavefront (256-byte rows: 8 lanes x 2 pieces, 48 -> 41 us),
// the transpose's rows are mostly one or two entries long and run best with 16 lanes x 1 piece (32 vs 37 us);
// 1 KB rows take a whole wavefront each in both directions.
template <typename T, bool FWD, typename FN> static bool dispatch_width(int nvec, FN fn) {
  if (nvec <= 1) fn.template operator()<0, 1>();
  else if (nvec <= 2) fn.template operator()<1, 1>();
  else if (nvec <= 4) fn.template operator()<2, 1>();
  else if (nvec <= 8) fn.template operator()<3, 1>();
  else if (nvec <= 16) {
    if constexpr (FWD) fn.template operator()<3, 2>();
    else fn.template operator()<4, 1>();
  }
  else if (nvec <= 32) fn.template operator()<4, 2>();
  else if (nvec <= 64) fn.template operator()<6, 1>();
  else if (nvec <= 128) fn.template operator()<6, 2>();
  else if (nvec <= 256) fn.template operator()<6, 4>();
  else return false;
  return true;
}

bool launch_spmm_fwd_uniform(hipStream_t s, int dtype, const LayerDev &L, int F, const void *x, void *z, void *zlo,
                             int row_begin, int row_end, const uint64_t *gaddr, const TransposeJobs *tjp) {
  const int es = dtype == HGNN_BF16 ? 2 : 4;
  const int nvec = F * es / 16;
  const unsigned long long *ga = reinterpret_cast<const unsigned long long *>(gaddr);
  TransposeJobs none;
  if (!tjp) {
    std::memset(&none, 0, sizeof(none));
    tjp = &none;
  }
  const TransposeJobs &tj = *tjp;
  if (dtype == HGNN_BF16)
    return dispatch_width<bf16, true>(nvec, [&]<int LPRL, int C>() { launch_fwd_uniform<bf16, LPRL, C>(s, L, x, ga, z, zlo, F, row_begin, row_end, tj); });
  return dispatch_width<float, true>(nvec, [&]<int LPRL, int C>() { launch_fwd_uniform<float, LPRL, C>(s, L, x, ga, z, zlo, F, row_begin, row_end, tj); });
}

// gaddr[e] = address of the feature row that edge e reads: the row ids[t][c - row_off[t]] of store t, for the
// merged source row c = colidx[e] and its vertex type t.
__global__ void __launch_bounds__(256) gather_address_kernel(const int32_t *__restrict__ colidx, int edges, GatherSrc gs, int row_bytes,
                                                              unsigned long long *__restrict__ gaddr) {
  const int e = blockIdx.x * 256 + threadIdx.x;
  if (e >= edges) return;
  const int c = colidx[e];
  int t = 0;
  while (t + 1 < gs.num_types && c >= gs.row_off[t + 1]) ++t;
  const long long id = gs.ids[t][c - gs.row_off[t]];
  gaddr[e] = reinterpret_cast<unsigned long long>(gs.store[t]) + (unsigned long long)id * (unsigned long long)row_bytes;
}

hgnn_status launch_gather_addresses(hipStream_t s, const LayerDev &L, const GatherSrc &gs, int row_bytes, uint64_t *gaddr) {
  if (L.edges == 0) return HGNN_OK;
  HGNN_LAUNCH(gather_address_kernel, dim3((L.edges + 255) / 256), dim3(256), 0, s, L.colidx, L.edges, gs, row_bytes,
              reinterpret_cast<unsigned long long *>(gaddr));
  HGNN_HIP(hipGetLastError());
  return HGNN_OK;
}

// ------------------------------------------------------------------------------------------
// Algorithm 1 of the paper taken literally, as a baseline for the fused gather-mean above: the source rows of
// all semantic graphs are collected into one matrix FeatureCat [E x F] (IndexSelect per relation + Concat: in
// the merged CSR the edges of all relations are already one list, so this is one gather), and Aggregate then
// reduces FeatureCat by destination (one segment per merged row).  The sums run over the edges in the order
// of the fused kernel, so the two give the same bits.
template <typename T>
__global__ void __launch_bounds__(256) feature_cat_kernel(const int32_t *__restrict__ colidx, const T *__restrict__ x,
                                                           T *__restrict__ fc, int nvec, int64_t pieces) {
  const uint4 *xb = reinterpret_cast<const uint4 *>(x);
  uint4 *fb = reinterpret_cast<uint4 *>(fc);
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < pieces; i += (int64_t)gridDim.x * 256) {
    const int64_t e = i / nvec;
    const int q = (int)(i - e * nvec);
    fb[i] = xb[(int64_t)colidx[e] * nvec + q];
  }
}

// one lane per 16-byte piece of a merged row: z[row] = mean of fc[rowptr[row] .. rowptr[row + 1])
template <typename T>
__global__ void __launch_bounds__(256) segment_mean_kernel(const int32_t *__restrict__ rowptr, const T *__restrict__ fc,
                                                            T *__restrict__ z, T *__restrict__ zlo, int nvec, int64_t pieces) {
  using V = Vec16<T>;
  const uint4 *fb = reinterpret_cast<const uint4 *>(fc);
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < pieces; i += (int64_t)gridDim.x * 256) {
    const int64_t row = i / nvec;
    const int q = (int)(i - row * nvec);
    const int beg = rowptr[row], end = rowptr[row + 1];
    float acc[V::N];
#pragma unroll
    for (int k = 0; k < V::N; ++k) acc[k] = 0.f;
    for (int e = beg; e < end; ++e) V::add(acc, fb[(int64_t)e * nvec + q]);
    const float inv = end > beg ? 1.0f / (float)(end - beg) : 0.0f;
#pragma unroll
    for (int k = 0; k < V::N; ++k) acc[k] *= inv;
    const uint4 hi = V::pack(acc);
    reinterpret_cast<uint4 *>(z)[i] = hi;
    if (zlo) reinterpret_cast<uint4 *>(zlo)[i] = V::pack_remainder(acc, hi);
  }
}

hgnn_status launch_aggregate_literal(hipStream_t s, int dtype, const LayerDev &L, int F, const void *x, void *feature_cat,
                                     void *z, void *zlo) {
  const int es = dtype == HGNN_BF16 ? 2 : 4;
  const int nvec = F * es / 16;
  const int64_t pe = (int64_t)L.edges * nvec, pr = (int64_t)L.rows * nvec;
  if (pe > 0) {
    const int blocks = (int)std::min<int64_t>((pe + 255) / 256, 1 << 16);
    if (dtype == HGNN_BF16)
      HGNN_LAUNCH(feature_cat_kernel<bf16>, dim3(blocks), dim3(256), 0, s, L.colidx, (const bf16 *)x, (bf16 *)feature_cat, nvec, pe);
    else
      HGNN_LAUNCH(feature_cat_kernel<float>, dim3(blocks), dim3(256), 0, s, L.colidx, (const float *)x, (float *)feature_cat, nvec, pe);
    HGNN_HIP(hipGetLastError());
  }
  if (pr > 0) {
    const int blocks = (int)std::min<int64_t>((pr + 255) / 256, 1 << 16);
    if (dtype == HGNN_BF16)
      HGNN_LAUNCH(segment_mean_kernel<bf16>, dim3(blocks), dim3(256), 0, s, L.rowptr, (const bf16 *)feature_cat, (bf16 *)z, (bf16 *)zlo, nvec, pr);
    else
      HGNN_LAUNCH(segment_mean_kernel<float>, dim3(blocks), dim3(256), 0, s, L.rowptr, (const float *)feature_cat, (float *)z, (float *)zlo, nvec, pr);
    HGNN_HIP(hipGetLastError());
  }
  return HGNN_OK;
}

// ------------------------------------------------------------------------------------------
// Transpose: dx[c] = sum over transpose row c of dz[crow] (+ root-term gradient for destination rows).
// Only the source rows of the vertex types listed in `ranges` are produced; rows longer than kLongRow are
// left to the chunked path.
struct RowRange {
  int32_t lo, hi;        // merged source rows of one vertex type
  int32_t n_dst;         // its destination rows (prefix)
  int32_t wave0;         // first wave working on this range
  int64_t root_off;      // scalars before its root-term gradient in dz, or -1 without a root term
};
struct RowRanges {
  RowRange r[kMaxT];
  int32_t n, total_waves;
};

template <typename T, int LPRL, int C>
__global__ void __launch_bounds__(256) spmm_bwd_uniform_kernel(const int32_t *__restrict__ cptr, const int32_t *__restrict__ crow,
                                                                RowRanges rr, const T *__restrict__ dz, T *__restrict__ dx, int F,
                                                                const int32_t *__restrict__ chunk_row,
                                                                const int32_t *__restrict__ chunk_beg, int n_chunks,
                                                                float *__restrict__ partial) {
  using V = Vec16<T>;
  constexpr int LPR = 1 << LPRL, RPW = 64 / LPR;
  const int lane = threadIdx.x & 63;
  const int wave = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (wave >= rr.total_waves) {
    // The waves behind the row waves take the chunks of the long rows (kChunk entries each): fp32 partial sums
    // for the pass that adds them up.  They ride in this launch because on their own they are a launch of a few
    // blocks that the stream would run after this one.
    const int item = (wave - rr.total_waves) * RPW + (lane >> LPRL), sub = lane & (LPR - 1);
    if (item >= n_chunks) return;
    const int c = chunk_row[item];
    bool wanted = false;
    for (int i = 0; i < rr.n; ++i) wanted |= c >= rr.r[i].lo && c < rr.r[i].hi;
    if (!wanted) return;
    const int beg = chunk_beg[item], end = min(beg + kChunk, cptr[c + 1]);
    const int nvec = F / V::N;
    const uint4 *zb = reinterpret_cast<const uint4 *>(dz);
    for (int q = sub; q < nvec; q += LPR) {
      float acc[V::N];
#pragma unroll
      for (int i = 0; i < V::N; ++i) acc[i] = 0.f;
      int e = beg;
      for (; e + 4 <= end; e += 4) {
        const uint4 v0 = zb[(int64_t)crow[e] * nvec + q], v1 = zb[(int64_t)crow[e + 1] * nvec + q];
        const uint4 v2 = zb[(int64_t)crow[e + 2] * nvec + q], v3 = zb[(int64_t)crow[e + 3] * nvec + q];
        V::add(acc, v0); V::add(acc, v1); V::add(acc, v2); V::add(acc, v3);
      }
      for (; e < end; ++e) V::add(acc, zb[(int64_t)crow[e] * nvec + q]);
      float *pp = partial + (int64_t)item * F + q * V::N;
#pragma unroll
      for (int i = 0; i < V::N; ++i) pp[i] = acc[i];
    }
    return;
  }
  int ri = 0;
  while (ri + 1 < rr.n && wave >= rr.r[ri + 1].wave0) ++ri;
  const RowRange R = rr.r[ri];
  const int row0 = R.lo + (wave - R.wave0) * RPW;
  const int nrows = min(RPW, R.hi - row0);
  const int rp = cptr[row0 + min(lane, nrows)];
  const int e0 = __shfl(rp, 0), eN = __shfl(rp, nrows);
  const int c0 = e0 + lane < eN ? crow[e0 + lane] : 0;
  const int c1 = e0 + 64 + lane < eN ? crow[e0 + 64 + lane] : 0;
  const int g = lane >> LPRL, sub = lane & (LPR - 1);
  const int beg = __shfl(rp, min(g, nrows)), end = __shfl(rp, min(g + 1, nrows));
  const bool is_long = end - beg > kLongRow;
  const int len = is_long ? 0 : end - beg;
  int maxlen = len;
#pragma unroll
  for (int o = 32; o >= LPR; o >>= 1) maxlen = max(maxlen, __shfl_xor(maxlen, o));
  const int nvec = F / V::N;
  const uint4 *zb = reinterpret_cast<const uint4 *>(dz);
  float acc[C][V::N];
#pragma unroll
  for (int p = 0; p < C; ++p)
#pragma unroll
    for (int i = 0; i < V::N; ++i) acc[p][i] = 0.f;
  for (int i = 0; i < maxlen; i += 4) {
    int col[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) col[j] = wave_col(c0, c1, beg - e0 + i + j);
    uint4 v[4][C];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const bool on = i + j < len;
      int cj = col[j];
      if (on && beg - e0 + i + j >= 128) cj = crow[beg + i + j];
#pragma unroll
      for (int p = 0; p < C; ++p) {
        const int q = sub + p * LPR;
        v[j][p] = (on && q < nvec) ? zb[(int64_t)cj * nvec + q] : make_uint4(0, 0, 0, 0);
      }
    }
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int p = 0; p < C; ++p) V::add(acc[p], v[j][p]);
  }
  if (g >= nrows || is_long) return;
  const int c = row0 + g, cl = c - R.lo;
  const bool root = R.root_off >= 0 && cl < R.n_dst;
#pragma unroll
  for (int p = 0; p < C; ++p) {
    const int q = sub + p * LPR;
    if (q >= nvec) continue;
    if (root) V::add(acc[p], reinterpret_cast<const uint4 *>(dz + R.root_off + (int64_t)cl * F)[q]);
    reinterpret_cast<uint4 *>(dx + (int64_t)c * F)[q] = V::pack(acc[p]);
  }
}

template <typename T, int LPRL, int C>
static void launch_bwd_uniform(hipStream_t s, const LayerDev &L, RowRanges &rr, const void *dz, void *dx, int F, float *partial) {
  constexpr int RPW = 64 >> LPRL;
  int w = 0;
  for (int i = 0; i < rr.n; ++i) {
    rr.r[i].wave0 = w;
    w += (rr.r[i].hi - rr.r[i].lo + RPW - 1) / RPW;
  }
  rr.total_waves = w;
  w += (L.n_chunks + RPW - 1) / RPW;  // the chunk waves
  if (w == 0) return;
  HGNN_LAUNCH((spmm_bwd_uniform_kernel<T, LPRL, C>), dim3((w + 3) / 4), dim3(256), 0, s, L.cptr, L.crow, rr, (const T *)dz,
                     (T *)dx, F, L.chunk_row, L.chunk_beg, L.n_chunks, partial);
}

bool launch_spmm_bwd_uniform(hipStream_t s, int dtype, const LayerDev &L, const TypeTab &tt, const RelTab &rt, const PtrTab &pt,
                             int F, uint32_t want, const void *dz, void *dx, float *partial) {
  RowRanges rr;
  rr.n = 0;
  for (int t = 0; t < tt.num_types; ++t) {
    if (!((want >> t) & 1u) || tt.row_off[t + 1] == tt.row_off[t]) continue;
    RowRange &r = rr.r[rr.n++];
    r.lo = tt.row_off[t];
    r.hi = tt.row_off[t + 1];
    r.n_dst = tt.n_dst[t];
    r.root_off = pt.w_root[t] ? (int64_t)rt.zroot_off4[t] * 4 : -1;
    r.wave0 = 0;
  }
  rr.total_waves = 0;
  const int es = dtype == HGNN_BF16 ? 2 : 4;
  const int nvec = F * es / 16;
  if (dtype == HGNN_BF16)
    return dispatch_width<bf16, false>(nvec, [&]<int LPRL, int C>() { launch_bwd_uniform<bf16, LPRL, C>(s, L, rr, dz, dx, F, partial); });
  return dispatch_width<float, false>(nvec, [&]<int LPRL, int C>() { launch_bwd_uniform<float, LPRL, C>(s, L, rr, dz, dx, F, partial); });
}

}  // namespace hgnn
