// Memory-bound kernels of the layer path (gfx950): type-first feature gather, the relation-
// segmented gather-mean over the merged CSR (paper Algorithm 1, evaluated without materialising
// the per-edge feature copies), its transpose for the backward pass, and small element-wise
// helpers.  Every feature row is moved in 16-byte pieces by a power-of-two group of lanes.
#include <cstring>
#include "common.h"
#include "bias_reduce.h"
#include "device_types.h"
#include "transpose_jobs.h"

namespace hgnn {

// ------------------------------------------------------------------------------------------
// Stage 0: gather mini-batch rows from the per-type stores into the type-first buffer.
// ------------------------------------------------------------------------------------------
struct MergeTab {
  const void *store[kMaxT];
  const int64_t *ids[kMaxT];
  const int32_t *pos[kMaxT];   // index-first baseline: row of the interleaved buffer that holds row i of type t
  const char *inter;           // mode 2: the interleaved buffer rows are read from
  int64_t elem_off[kMaxT + 1];
  int32_t row_off[kMaxT + 1];
  int32_t dim[kMaxT];
  int32_t num_types;
  int32_t mode;                // 0: stores -> type-first buffer; 1: stores -> interleaved buffer; 2: interleaved -> type-first
};

__global__ void __launch_bounds__(256) merge_kernel(MergeTab mt, char *out, int esize, int lpr_log2) {
  const int lpr = 1 << lpr_log2;
  const int row = blockIdx.x * (256 >> lpr_log2) + (threadIdx.x >> lpr_log2);
  const int lane = threadIdx.x & (lpr - 1);
  if (row >= mt.row_off[mt.num_types]) return;
  int t = 0;
  while (row >= mt.row_off[t + 1]) ++t;
  const int i = row - mt.row_off[t];
  const int nvec = (mt.dim[t] * esize) >> 4;
  // interleaved position, clamped into the buffer (a caller's bad position cannot leave it)
  const int64_t at = mt.mode ? min(max(mt.pos[t][i], 0), mt.row_off[mt.num_types] - 1) : 0;
  const uint4 *src = mt.mode == 2 ? reinterpret_cast<const uint4 *>(mt.inter) + at * nvec
                                  : reinterpret_cast<const uint4 *>(mt.store[t]) + mt.ids[t][i] * nvec;
  uint4 *dst = mt.mode == 1 ? reinterpret_cast<uint4 *>(out) + at * nvec
                            : reinterpret_cast<uint4 *>(out + mt.elem_off[t] * esize) + (int64_t)i * nvec;
  for (int c = lane; c < nvec; c += 2 * lpr) {  // both loads before the stores
    const int c2 = c + lpr;
    const uint4 a = src[c];
    const uint4 b = c2 < nvec ? src[c2] : a;
    dst[c] = a;
    if (c2 < nvec) dst[c2] = b;
  }
}

hgnn_status launch_merge(hipStream_t s, int dtype, int T, const void *const *store, const int32_t *feat_dim,
                         const int64_t *const *ids, const int64_t *n_rows, const int64_t *elem_off, void *out, int mode,
                         const int32_t *const *pos, const void *interleaved) {
  MergeTab mt;
  std::memset(&mt, 0, sizeof(mt));
  const int es = dtype == HGNN_BF16 ? 2 : 4;
  int maxd = 0;
  mt.row_off[0] = 0;
  mt.mode = mode;
  mt.inter = (const char *)interleaved;
  for (int t = 0; t < T; ++t) {
    mt.store[t] = store ? store[t] : nullptr;
    mt.ids[t] = ids ? ids[t] : nullptr;
    mt.pos[t] = pos ? pos[t] : nullptr;
    mt.elem_off[t] = elem_off[t];
    mt.row_off[t + 1] = mt.row_off[t] + (int32_t)n_rows[t];
    mt.dim[t] = feat_dim[t];
    if (n_rows[t] > 0) maxd = std::max(maxd, feat_dim[t]);
  }
  mt.elem_off[T] = elem_off[T];
  mt.num_types = T;
  const int total = mt.row_off[T];
  if (total == 0) return HGNN_OK;
  // two 16-byte pieces per lane: both loads of a lane are in flight together (a lane per piece left the copy
  // waiting on one load at a time: 50 -> 43 us on the headline's 400k rows of 256 bytes; four per lane gain nothing)
  const int l2 = std::max(0, lanes_log2_for(maxd, es) - 1);
  const int rpb = 256 >> l2;
  HGNN_LAUNCH(merge_kernel, dim3((total + rpb - 1) / rpb), dim3(256), 0, s, mt, (char *)out, es, l2);
  HGNN_HIP(hipGetLastError());
  return HGNN_OK;
}

// ------------------------------------------------------------------------------------------
// Stage 3: z[rho] = mean over the merged CSR row rho of the source rows of x.
// One group of 2^lpr_log2 lanes owns one row; a lane owns 16-byte pieces of the feature row.
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ int rel_of_row(const int32_t *rel_row_off, int R, int row) {
  int lo = 0, hi = R;  // find r with rel_row_off[r] <= row < rel_row_off[r+1]
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (rel_row_off[mid] <= row) lo = mid; else hi = mid;
  }
  return lo;
}

template <typename T>
__global__ void __launch_bounds__(256) spmm_fwd_kernel(LayerDev L, TypeTab tt, RelTab rt, const T *__restrict__ x,
                                                        T *__restrict__ z, T *__restrict__ zlo, int row_begin, int row_end,
                                                        int lpr_log2) {
  using V = Vec16<T>;
  const int lpr = 1 << lpr_log2;
  const int row = row_begin + blockIdx.x * (256 >> lpr_log2) + (threadIdx.x >> lpr_log2);
  const int lane = threadIdx.x & (lpr - 1);
  if (row >= row_end) return;
  const int r = rel_of_row(L.rel_row_off, rt.num_rels, row);
  const int st = rt.src[r];
  const int F = tt.in_dim[st];
  const int nvec = F / V::N;
  const uint4 *xb = reinterpret_cast<const uint4 *>(x + tt.elem_off[st]);
  const int rowbase = tt.row_off[st];
  const int64_t zoff = (int64_t)rt.z_off4[r] * 4 + (int64_t)(row - L.rel_row_off[r]) * F;
  uint4 *zr = reinterpret_cast<uint4 *>(z + zoff);
  const int beg = L.rowptr[row], end = L.rowptr[row + 1];
  const float inv = end > beg ? 1.0f / (float)(end - beg) : 0.0f;
  for (int c = lane; c < nvec; c += lpr) {
    float acc[V::N];
#pragma unroll
    for (int i = 0; i < V::N; ++i) acc[i] = 0.f;
    int e = beg;
    for (; e + 4 <= end; e += 4) {
      const int c0 = L.colidx[e] - rowbase, c1 = L.colidx[e + 1] - rowbase;
      const int c2 = L.colidx[e + 2] - rowbase, c3 = L.colidx[e + 3] - rowbase;
      const uint4 v0 = xb[(int64_t)c0 * nvec + c], v1 = xb[(int64_t)c1 * nvec + c];
      const uint4 v2 = xb[(int64_t)c2 * nvec + c], v3 = xb[(int64_t)c3 * nvec + c];
      V::add(acc, v0); V::add(acc, v1); V::add(acc, v2); V::add(acc, v3);
    }
    for (; e < end; ++e) {
      const int c0 = L.colidx[e] - rowbase;
      V::add(acc, xb[(int64_t)c0 * nvec + c]);
    }
#pragma unroll
    for (int i = 0; i < V::N; ++i) acc[i] *= inv;
    const uint4 hi = V::pack(acc);
    zr[c] = hi;
    if (zlo) reinterpret_cast<uint4 *>(zlo + zoff)[c] = V::pack_remainder(acc, hi);
  }
}

hgnn_status launch_spmm_fwd(hipStream_t s, int dtype, const LayerDev &L, const TypeTab &tt, const RelTab &rt,
                            int max_dim, const void *x, void *z, void *zlo, int row_begin, int row_end,
                            const TransposeJobs *tj) {
  if (row_end <= row_begin) return tj ? launch_transpose_jobs(s, dtype, *tj) : HGNN_OK;
  const int es = dtype == HGNN_BF16 ? 2 : 4;
  bool uniform = true;
  for (int t = 0; t < tt.num_types; ++t) uniform &= tt.in_dim[t] == tt.in_dim[0];
  if (uniform && launch_spmm_fwd_uniform(s, dtype, L, tt.in_dim[0], x, z, zlo, row_begin, row_end, nullptr, tj)) {
    HGNN_HIP(hipGetLastError());
    return HGNN_OK;
  }
  if (tj) {
    hgnn_status st = launch_transpose_jobs(s, dtype, *tj);
    if (st != HGNN_OK) return st;
  }
  const int l2 = lanes_log2_for(max_dim, es);
  const int rpb = 256 >> l2;
  dim3 grid((row_end - row_begin + rpb - 1) / rpb);
  if (dtype == HGNN_BF16)
    HGNN_LAUNCH(spmm_fwd_kernel<bf16>, grid, dim3(256), 0, s, L, tt, rt, (const bf16 *)x, (bf16 *)z, (bf16 *)zlo, row_begin, row_end, l2);
  else
    HGNN_LAUNCH(spmm_fwd_kernel<float>, grid, dim3(256), 0, s, L, tt, rt, (const float *)x, (float *)z, (float *)nullptr, row_begin, row_end, l2);
  HGNN_HIP(hipGetLastError());
  return HGNN_OK;
}

// ------------------------------------------------------------------------------------------
// Backward of the aggregation: dx[c] = sum over the transpose row c of dz[crow] (dz rows arrive
// already scaled by 1/|N_r(v)|) plus, for destination rows, the root-term gradient.
// Rows longer than kLongRow are cut into chunks of kChunk edges: phase 0 handles the short rows
// and writes fp32 partial sums for the chunks, phase 1 adds up the partials of each long row.
// ------------------------------------------------------------------------------------------
template <typename T>
__device__ __forceinline__ const uint4 *dz_row(const T *dz, const LayerDev &L, const RelTab &rt, int F, int rho, bool uniform) {
  if (uniform) return reinterpret_cast<const uint4 *>(dz + (int64_t)rho * F);
  const int r = rel_of_row(L.rel_row_off, rt.num_rels, rho);
  return reinterpret_cast<const uint4 *>(dz + (int64_t)rt.z_off4[r] * 4 + (int64_t)(rho - L.rel_row_off[r]) * F);
}

template <typename T>
__global__ void __launch_bounds__(256) spmm_bwd_kernel(LayerDev L, TypeTab tt, RelTab rt, uint32_t root_mask, uint32_t want,
                                                        const T *__restrict__ dz, T *__restrict__ dx,
                                                        float *__restrict__ partial, int max_dim, int row_blocks,
                                                        int lpr_log2, int uniform) {
  using V = Vec16<T>;
  const int lpr = 1 << lpr_log2;
  const int gpb = 256 >> lpr_log2;
  const int lane = threadIdx.x & (lpr - 1);
  const bool chunk_part = (int)blockIdx.x >= row_blocks;
  const int item = (chunk_part ? (int)blockIdx.x - row_blocks : (int)blockIdx.x) * gpb + (threadIdx.x >> lpr_log2);
  int c, beg, end;
  if (!chunk_part) {
    if (item >= L.src_rows) return;
    c = item;
    beg = L.cptr[c];
    end = L.cptr[c + 1];
    if (end - beg > kLongRow) return;
  } else {
    if (item >= L.n_chunks) return;
    c = L.chunk_row[item];
    beg = L.chunk_beg[item];
    end = min(beg + kChunk, L.cptr[c + 1]);
  }
  int t = 0;
  while (c >= tt.row_off[t + 1]) ++t;
  if (!((want >> t) & 1u)) return;  // the caller does not want input gradients of this vertex type
  const int F = tt.in_dim[t];
  const int nvec = F / V::N;
  const int cl = c - tt.row_off[t];
  for (int q = lane; q < nvec; q += lpr) {
    float acc[V::N];
#pragma unroll
    for (int i = 0; i < V::N; ++i) acc[i] = 0.f;
    int e = beg;
    for (; e + 4 <= end; e += 4) {
      const uint4 *p0 = dz_row(dz, L, rt, F, L.crow[e], uniform), *p1 = dz_row(dz, L, rt, F, L.crow[e + 1], uniform);
      const uint4 *p2 = dz_row(dz, L, rt, F, L.crow[e + 2], uniform), *p3 = dz_row(dz, L, rt, F, L.crow[e + 3], uniform);
      const uint4 v0 = p0[q], v1 = p1[q], v2 = p2[q], v3 = p3[q];
      V::add(acc, v0); V::add(acc, v1); V::add(acc, v2); V::add(acc, v3);
    }
    for (; e < end; ++e) V::add(acc, dz_row(dz, L, rt, F, L.crow[e], uniform)[q]);
    if (!chunk_part) {
      if (cl < tt.n_dst[t] && ((root_mask >> t) & 1u)) {
        const T *zr = dz + (int64_t)rt.zroot_off4[t] * 4 + (int64_t)cl * F;
        V::add(acc, reinterpret_cast<const uint4 *>(zr)[q]);
      }
      reinterpret_cast<uint4 *>(dx + tt.elem_off[t] + (int64_t)cl * F)[q] = V::pack(acc);
    } else {
      float *pp = partial + (int64_t)item * max_dim + q * V::N;
#pragma unroll
      for (int i = 0; i < V::N; ++i) pp[i] = acc[i];
    }
  }
}

// Long rows: sums the chunk partials of one source row (one block per row), adds the root part and writes
// the row.  W = floats per load (4 when the row width allows).  The block's threads form `groups` groups of
// `lanes` threads; group g sums chunks g, g + groups, ... four at a time, LDS adds the groups up.
template <typename T, int W>
__global__ void __launch_bounds__(256) spmm_bwd_long_kernel(LayerDev L, TypeTab tt, RelTab rt, uint32_t root_mask, uint32_t want,
                                                             const T *__restrict__ dz, T *__restrict__ dx,
                                                             const float *__restrict__ partial, int max_dim) {
  typedef float fw __attribute__((ext_vector_type(W)));
  __shared__ float red[256 * W];
  const int i = blockIdx.x;  // one block per long row
  const int c = L.long_row[i];
  int t = 0;
  while (c >= tt.row_off[t + 1]) ++t;
  if (!((want >> t) & 1u)) return;
  const int F = tt.in_dim[t];
  const int cl = c - tt.row_off[t];
  const int j0 = L.long_chunk0[i], j1 = L.long_chunk0[i + 1];
  const bool root = cl < tt.n_dst[t] && ((root_mask >> t) & 1u);
  const int nw = F / W;                       // loads per row (W divides F)
  int lanes = 1;
  while (lanes < nw && lanes < 256) lanes <<= 1;
  const int groups = 256 / lanes, g = threadIdx.x / lanes, ln = threadIdx.x % lanes;
  for (int q0 = 0; q0 < nw; q0 += lanes) {    // more than one pass only for rows wider than 256 loads
    const int q = q0 + ln;
    fw acc = {};
    if (q < nw) {
      int j = j0 + g;
      for (; j + 3 * groups < j1; j += 4 * groups) {
        const fw v0 = *reinterpret_cast<const fw *>(partial + (int64_t)j * max_dim + q * W);
        const fw v1 = *reinterpret_cast<const fw *>(partial + (int64_t)(j + groups) * max_dim + q * W);
        const fw v2 = *reinterpret_cast<const fw *>(partial + (int64_t)(j + 2 * groups) * max_dim + q * W);
        const fw v3 = *reinterpret_cast<const fw *>(partial + (int64_t)(j + 3 * groups) * max_dim + q * W);
        acc += (v0 + v1) + (v2 + v3);
      }
      for (; j < j1; j += groups) acc += *reinterpret_cast<const fw *>(partial + (int64_t)j * max_dim + q * W);
    }
    if (groups > 1) {
      *reinterpret_cast<fw *>(red + threadIdx.x * W) = acc;
      __syncthreads();
      if (g == 0) {
        for (int o = 1; o < groups; ++o) acc += *reinterpret_cast<const fw *>(red + (o * lanes + ln) * W);
      }
    }
    if (g == 0 && q < nw) {
#pragma unroll
      for (int k = 0; k < W; ++k) {
        const int f = q * W + k;
        float v = acc[k];
        if (root) v += to_float(dz[(int64_t)rt.zroot_off4[t] * 4 + (int64_t)cl * F + f]);
        dx[tt.elem_off[t] + (int64_t)cl * F + f] = from_float<T>(v);
      }
    }
    if (groups > 1) __syncthreads();
  }
}

hgnn_status launch_spmm_bwd(hipStream_t s, int dtype, const LayerDev &L, const TypeTab &tt, const RelTab &rt,
                            const PtrTab &pt, int max_dim, uint32_t want, const void *dz, void *dx, float *partial) {
  if (L.src_rows == 0) return HGNN_OK;
  const int es = dtype == HGNN_BF16 ? 2 : 4;
  const int l2 = lanes_log2_for(max_dim, es);
  const int gpb = 256 >> l2;
  int row_blocks = (L.src_rows + gpb - 1) / gpb;
  int chunk_blocks = (L.n_chunks + gpb - 1) / gpb;
  uint32_t root_mask = 0;
  bool uniform = true;  // every relation's aggregate rows have the same width: dz row rho starts at rho * F
  for (int t = 0; t < tt.num_types; ++t) {
    if (pt.w_root[t]) root_mask |= 1u << t;
    if (tt.in_dim[t] != tt.in_dim[0]) uniform = false;
  }
  // rows up to kLongRow edges: the uniform-width kernel when it applies, else the generic one below
  // (the uniform kernel's launch also carries the chunks of the long rows; max_dim is the common width then)
  if (uniform && launch_spmm_bwd_uniform(s, dtype, L, tt, rt, pt, tt.in_dim[0], want, dz, dx, partial)) {
    HGNN_HIP(hipGetLastError());
    row_blocks = 0;
    chunk_blocks = 0;
  }
  dim3 grid(row_blocks + chunk_blocks);
  if (grid.x > 0) {
  if (dtype == HGNN_BF16)
    HGNN_LAUNCH(spmm_bwd_kernel<bf16>, grid, dim3(256), 0, s, L, tt, rt, root_mask, want, (const bf16 *)dz, (bf16 *)dx,
                       partial, max_dim, row_blocks, l2, (int)uniform);
  else
    HGNN_LAUNCH(spmm_bwd_kernel<float>, grid, dim3(256), 0, s, L, tt, rt, root_mask, want, (const float *)dz, (float *)dx,
                       partial, max_dim, row_blocks, l2, (int)uniform);
  HGNN_HIP(hipGetLastError());
  }
  if (L.n_long > 0) {
    bool w4 = (max_dim % 4) == 0;   // every row of the partial buffer starts 16-byte aligned
    for (int t = 0; t < tt.num_types; ++t)
      if (tt.in_dim[t] % 4) w4 = false;
    const dim3 g(L.n_long), b(256);
    if (dtype == HGNN_BF16) {
      if (w4) HGNN_LAUNCH((spmm_bwd_long_kernel<bf16, 4>), g, b, 0, s, L, tt, rt, root_mask, want, (const bf16 *)dz, (bf16 *)dx, partial, max_dim);
      else HGNN_LAUNCH((spmm_bwd_long_kernel<bf16, 1>), g, b, 0, s, L, tt, rt, root_mask, want, (const bf16 *)dz, (bf16 *)dx, partial, max_dim);
    } else {
      if (w4) HGNN_LAUNCH((spmm_bwd_long_kernel<float, 4>), g, b, 0, s, L, tt, rt, root_mask, want, (const float *)dz, (float *)dx, partial, max_dim);
      else HGNN_LAUNCH((spmm_bwd_long_kernel<float, 1>), g, b, 0, s, L, tt, rt, root_mask, want, (const float *)dz, (float *)dx, partial, max_dim);
    }
    HGNN_HIP(hipGetLastError());
  }
  return HGNN_OK;
}

// ------------------------------------------------------------------------------------------
// Weight transposes: Wt[h][f] = W[f][h] for every relation and root weight, as a job list.
// ------------------------------------------------------------------------------------------
void make_transpose_jobs(const TypeTab &tt, const RelTab &rt, const PtrTab &pt, const WtTab &wt, int H, void *wt_buf,
                         TransposeJobs &tj) {
  std::memset(&tj, 0, sizeof(tj));
  tj.H = H;
  tj.out = wt_buf;
  const int R = rt.num_rels, tiles_h = (H + 31) / 32;
  for (int seg = 0; seg < R + tt.num_types; ++seg) {
    const void *w = seg < R ? pt.w_rel[seg] : pt.w_root[seg - R];
    if (!w || tt.n_dst[seg < R ? rt.dst[seg] : seg - R] == 0) continue;  // no destination rows: no tile reads this weight
    const int F = tt.in_dim[seg < R ? rt.src[seg] : seg - R];
    tj.w[tj.n] = w;
    tj.F[tj.n] = F;
    tj.off4[tj.n] = seg < R ? wt.rel4[seg] : wt.root4[seg - R];
    tj.tile_off[tj.n + 1] = tj.tile_off[tj.n] + ((F + 31) / 32) * tiles_h;
    ++tj.n;
  }
  // a tile per block (two dependent memory round trips) up to 2048 blocks: over long before the launch they ride in
  tj.blocks = std::min(2048, tj.tile_off[tj.n]);
}

template <typename T>
__global__ void __launch_bounds__(256) transpose_weights_kernel(TransposeJobs tj) {
  __shared__ T tile[32][33];
  transpose_jobs_block<T>(tj, blockIdx.x, gridDim.x, tile);
}

hgnn_status launch_transpose_jobs(hipStream_t s, int dtype, const TransposeJobs &tj) {
  if (tj.blocks == 0) return HGNN_OK;
  if (dtype == HGNN_BF16) HGNN_LAUNCH(transpose_weights_kernel<bf16>, dim3(tj.blocks), dim3(256), 0, s, tj);
  else HGNN_LAUNCH(transpose_weights_kernel<float>, dim3(tj.blocks), dim3(256), 0, s, tj);
  HGNN_HIP(hipGetLastError());
  return HGNN_OK;
}

hgnn_status launch_transpose_weights(hipStream_t s, int dtype, const TypeTab &tt, const RelTab &rt,
                                     const PtrTab &pt, const WtTab &wt, int H, void *wt_buf) {
  TransposeJobs tj;
  make_transpose_jobs(tt, rt, pt, wt, H, wt_buf, tj);
  return launch_transpose_jobs(s, dtype, tj);
}

// Zero-padded copies: out[off + f*Hp + c] = c < H ? W[f*H + c] : 0  (segment = blockIdx.y).
// Block bx of gx works on segment seg.
template <typename T>
__device__ __forceinline__ void pad_weights_part(const TypeTab &tt, const RelTab &rt, const PtrTab &pt, const WtTab &wo, int H,
                                                 int Hp, T *out, int seg, int bx, int gx) {
  const int R = rt.num_rels;
  const T *w = (const T *)(seg < R ? pt.w_rel[seg] : pt.w_root[seg - R]);
  if (!w || tt.n_dst[seg < R ? rt.dst[seg] : seg - R] == 0) return;  // no destination rows: no tile reads this copy
  const int F = tt.in_dim[seg < R ? rt.src[seg] : seg - R];
  T *o = out + (int64_t)(seg < R ? wo.rel4[seg] : wo.root4[seg - R]) * 4;
  // a block takes whole rows (no division per element)
  for (int f = bx; f < F; f += gx)
    for (int c = threadIdx.x; c < Hp; c += 256) o[(int64_t)f * Hp + c] = c < H ? w[(int64_t)f * H + c] : from_float<T>(0.f);
}

template <typename T>
__global__ void __launch_bounds__(256) pad_weights_kernel(TypeTab tt, RelTab rt, PtrTab pt, WtTab wo, int H, int Hp, T *out) {
  pad_weights_part<T>(tt, rt, pt, wo, H, Hp, out, blockIdx.y, blockIdx.x, gridDim.x);
}

hgnn_status launch_pad_weights(hipStream_t s, int dtype, const TypeTab &tt, const RelTab &rt, const PtrTab &pt,
                               const WtTab &wo, int H, int Hp, void *out) {
  dim3 grid(64, rt.num_rels + tt.num_types);
  if (dtype == HGNN_BF16)
    HGNN_LAUNCH(pad_weights_kernel<bf16>, grid, dim3(256), 0, s, tt, rt, pt, wo, H, Hp, (bf16 *)out);
  else
    HGNN_LAUNCH(pad_weights_kernel<float>, grid, dim3(256), 0, s, tt, rt, pt, wo, H, Hp, (float *)out);
  HGNN_HIP(hipGetLastError());
  return HGNN_OK;
}

// ------------------------------------------------------------------------------------------
// Backward epilogue: gp = grad_h * [h > 0] (when the layer has a ReLU) and dbias_t = column sums.
// One block = kRowsPerBlock rows of one type; a thread owns columns tid, tid+256, ...  The block's column sums are added
// to dbias_t, or, when `bpart` is given, stored as row `block` of bpart [blocks x H] for a later pass that adds
// the rows of a type up (no atomics, and dbias needs no zeroing first).
// ------------------------------------------------------------------------------------------
constexpr int kVecRows = 64;  // rows per block of the 16-bytes-per-lane row pass (32: the same; 128: +3 us; 16, 256: +10 us on the headline)
constexpr int kRowsPerBlock = 8;  // of the element-wise row pass (a multiple of the eight loads in flight per lane)
template <typename T>
__device__ __forceinline__ void relu_bias_rows(const TypeTab &tt, int block, int H, int ldo, int relu, int write,
                                               const T *__restrict__ g, const T *__restrict__ h, T *__restrict__ gp,
                                               const GradPtrTab &gt, float *__restrict__ bpart) {
  int b = block, t = 0;
  for (;; ++t) {
    const int nb = (tt.n_dst[t] + kRowsPerBlock - 1) / kRowsPerBlock;
    if (b < nb) break;
    b -= nb;
  }
  const int r0 = tt.out_row_off[t] + b * kRowsPerBlock;
  const int r1 = min(r0 + kRowsPerBlock, tt.out_row_off[t] + tt.n_dst[t]);
  float *db = gt.dbias[t];
  for (int c = threadIdx.x; c < ldo; c += 256) {
    float sum = 0.f;
    if (c < H) {
      // the block's rows, eight independent loads at a time
      for (int rb = r0; rb < r1; rb += 8) {
        float v[8], hv[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int64_t i = (int64_t)min(rb + u, r1 - 1) * H + c;
          v[u] = to_float(g[i]);
          hv[u] = relu ? to_float(h[i]) : 1.f;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          if (rb + u >= r1) break;
          const float x = hv[u] > 0.f ? v[u] : 0.f;
          if (write) gp[(int64_t)(rb + u) * ldo + c] = from_float<T>(x);
          sum += x;
        }
      }
      if (bpart) bpart[(int64_t)block * H + c] = sum;
      else if (db) atomicAdd(db + c, sum);
    } else if (write) {
      for (int r = r0; r < r1; ++r) gp[(int64_t)r * ldo + c] = from_float<T>(0.f);
    }
  }
}

template <typename T>
__global__ void __launch_bounds__(256) relu_bias_bwd_kernel(TypeTab tt, int H, int ldo, int relu, int write, const T *__restrict__ g,
                                                             const T *__restrict__ h, T *__restrict__ gp, GradPtrTab gt) {
  relu_bias_rows<T>(tt, blockIdx.x, H, ldo, relu, write, g, h, gp, gt, nullptr);
}

// Same, 16 bytes per lane: a block owns kVecRows rows of one type, 256/(H/VEC) rows are in flight at a time.
template <typename T>
__device__ __forceinline__ void relu_bias_rows_vec(const TypeTab &tt, int block, int H, int relu, const T *__restrict__ g,
                                                   const T *__restrict__ h, T *__restrict__ gp, const GradPtrTab &gt,
                                                   float *__restrict__ bpart) {
  using V = Vec16<T>;
  __shared__ float red[256 * V::N];
  int b = block, t = 0;
  for (;; ++t) {
    const int nb = (tt.n_dst[t] + kVecRows - 1) / kVecRows;
    if (b < nb) break;
    b -= nb;
  }
  const int chunks = H / V::N;          // <= 256
  const int rif = 256 / chunks;         // rows in flight
  const int c = threadIdx.x % chunks, rg = threadIdx.x / chunks;
  const int r0 = tt.out_row_off[t] + b * kVecRows;
  const int r1 = min(r0 + kVecRows, tt.out_row_off[t] + tt.n_dst[t]);
  float sum[V::N];
#pragma unroll
  for (int i = 0; i < V::N; ++i) sum[i] = 0.f;
  if (rg < rif) {
    // four rows per trip: eight 16-byte loads in flight per lane (a block has few rows, so there are few
    // wavefronts per compute unit to hide the latency otherwise)
    constexpr int U = 4;
    for (int r = r0 + rg; r < r1; r += U * rif) {
      uint4 gv[U], hv4[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int ru = r + u * rif;
        const int64_t i = ((int64_t)(ru < r1 ? ru : r) * H) / V::N + c;
        gv[u] = reinterpret_cast<const uint4 *>(g)[i];
        if (relu) hv4[u] = reinterpret_cast<const uint4 *>(h)[i];
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int ru = r + u * rif;
        if (ru >= r1) break;
        const int64_t i = ((int64_t)ru * H) / V::N + c;
        float v[V::N];
#pragma unroll
        for (int k = 0; k < V::N; ++k) v[k] = 0.f;
        V::add(v, gv[u]);
        if (relu) {
          float hv[V::N];
#pragma unroll
          for (int k = 0; k < V::N; ++k) hv[k] = 0.f;
          V::add(hv, hv4[u]);
#pragma unroll
          for (int k = 0; k < V::N; ++k)
            if (!(hv[k] > 0.f)) v[k] = 0.f;
          reinterpret_cast<uint4 *>(gp)[i] = V::pack(v);
        }
#pragma unroll
        for (int k = 0; k < V::N; ++k) sum[k] += v[k];
      }
    }
  }
  float *db = gt.dbias[t];
  if (!db) return;
#pragma unroll
  for (int k = 0; k < V::N; ++k) red[threadIdx.x * V::N + k] = sum[k];
  __syncthreads();
  for (int col = threadIdx.x; col < H; col += 256) {
    const int cc = col / V::N, k = col % V::N;
    float a = 0.f;
    for (int q = 0; q < rif; ++q) a += red[(q * chunks + cc) * V::N + k];
    if (bpart) bpart[(int64_t)block * H + col] = a;
    else atomicAdd(db + col, a);
  }
}

template <typename T>
__global__ void __launch_bounds__(256) relu_bias_bwd_vec_kernel(TypeTab tt, int H, int relu, const T *__restrict__ g,
                                                                 const T *__restrict__ h, T *__restrict__ gp, GradPtrTab gt) {
  relu_bias_rows_vec<T>(tt, blockIdx.x, H, relu, g, h, gp, gt, nullptr);
}

hgnn_status launch_relu_bias_bwd(hipStream_t s, int dtype, const TypeTab &tt, int H, int ldo, int relu,
                                 const void *grad_h, const void *h, void *gp, const GradPtrTab &gt) {
  const int vec = dtype == HGNN_BF16 ? 8 : 4;
  const bool fast = ldo == H && H % vec == 0 && H / vec <= 256 && (((uintptr_t)grad_h | (uintptr_t)h | (uintptr_t)gp) & 15) == 0;
  const int rpb = fast ? kVecRows : kRowsPerBlock;
  const int write = relu || ldo != H;
  int blocks = 0;
  for (int t = 0; t < tt.num_types; ++t) blocks += (tt.n_dst[t] + rpb - 1) / rpb;
  if (blocks == 0) return HGNN_OK;
  if (fast) {
    if (dtype == HGNN_BF16)
      HGNN_LAUNCH(relu_bias_bwd_vec_kernel<bf16>, dim3(blocks), dim3(256), 0, s, tt, H, relu, (const bf16 *)grad_h,
                         (const bf16 *)h, (bf16 *)gp, gt);
    else
      HGNN_LAUNCH(relu_bias_bwd_vec_kernel<float>, dim3(blocks), dim3(256), 0, s, tt, H, relu, (const float *)grad_h,
                         (const float *)h, (float *)gp, gt);
  } else if (dtype == HGNN_BF16) {
    HGNN_LAUNCH(relu_bias_bwd_kernel<bf16>, dim3(blocks), dim3(256), 0, s, tt, H, ldo, relu, write, (const bf16 *)grad_h,
                       (const bf16 *)h, (bf16 *)gp, gt);
  } else {
    HGNN_LAUNCH(relu_bias_bwd_kernel<float>, dim3(blocks), dim3(256), 0, s, tt, H, ldo, relu, write, (const float *)grad_h,
                       (const float *)h, (float *)gp, gt);
  }
  HGNN_HIP(hipGetLastError());
  return HGNN_OK;
}

// ------------------------------------------------------------------------------------------
__device__ __forceinline__ void zero_grads_part(const TypeTab &tt, const RelTab &rt, const GradPtrTab &gt, int H, int seg,
                                                int bx, int gx, bool bias_too) {
  const int R = rt.num_rels;
  float *w;
  int64_t n;
  if (seg < R) {
    w = gt.dw_rel[seg];
    n = (int64_t)tt.in_dim[rt.src[seg]] * H;
  } else {
    const int t = seg - R;
    w = gt.dw_root[t];
    n = (int64_t)tt.in_dim[t] * H;
    float *b = gt.dbias[t];
    if (b && bias_too)
      for (int i = bx * 256 + threadIdx.x; i < H; i += gx * 256) b[i] = 0.f;
  }
  if (!w) return;
  for (int64_t i = bx * 256 + threadIdx.x; i < n; i += (int64_t)gx * 256) w[i] = 0.f;
}

__global__ void __launch_bounds__(256) zero_grads_kernel(TypeTab tt, RelTab rt, GradPtrTab gt, int H) {
  zero_grads_part(tt, rt, gt, H, blockIdx.y, blockIdx.x, gridDim.x, true);
}

hgnn_status launch_zero_grads(hipStream_t s, const TypeTab &tt, const RelTab &rt, const GradPtrTab &gt, int H) {
  HGNN_LAUNCH(zero_grads_kernel, dim3(32, rt.num_rels + tt.num_types), dim3(256), 0, s, tt, rt, gt, H);
  HGNN_HIP(hipGetLastError());
  return HGNN_OK;
}

// The start of a layer's backward pass in ONE launch: the ReLU mask / bias column sums over G (the first
// nb_relu blocks; column sums go to bpart), zeroing of the weight gradients (nb_zero blocks) and the zero-padded
// weight copies (the rest).  The three touch different memory and none is big enough to fill the chip alone.
template <typename T, bool VEC>
__global__ void __launch_bounds__(256) bwd_prep_kernel(TypeTab tt, RelTab rt, PtrTab pt, WtTab wo, GradPtrTab gt, int H, int ldo,
                                                        int relu, int write, const T *__restrict__ g, const T *__restrict__ h,
                                                        T *__restrict__ gp, float *__restrict__ bpart, int nb_relu, int nb_zero,
                                                        T *__restrict__ wpad) {
  int b = blockIdx.x;
  if (b < nb_relu) {
    if constexpr (VEC) relu_bias_rows_vec<T>(tt, b, H, relu, g, h, gp, gt, bpart);
    else relu_bias_rows<T>(tt, b, H, ldo, relu, write, g, h, gp, gt, bpart);
    return;
  }
  b -= nb_relu;
  if (b < nb_zero) {
    zero_grads_part(tt, rt, gt, H, b / 32, b % 32, 32, false);
    return;
  }
  b -= nb_zero;
  pad_weights_part<T>(tt, rt, pt, wo, H, ldo, wpad, b / 64, b % 64, 64);
}

hgnn_status launch_bwd_prep(hipStream_t s, int dtype, const TypeTab &tt, const RelTab &rt, const PtrTab &pt, const WtTab &wo,
                            const GradPtrTab &gt, int H, int ldo, int relu, bool do_rows, bool do_zero, const void *grad_h,
                            const void *h, void *gp, float *bpart, size_t bpart_rows, void *wpad, int *rows_per_block) {
  const int vec = dtype == HGNN_BF16 ? 8 : 4;
  const bool fast = ldo == H && H % vec == 0 && H / vec <= 256 && (((uintptr_t)grad_h | (uintptr_t)h | (uintptr_t)gp) & 15) == 0;
  const int rpb = fast ? kVecRows : kRowsPerBlock;
  *rows_per_block = rpb;
  const int write = relu || ldo != H;
  int nb_relu = 0;
  if (do_rows)
    for (int t = 0; t < tt.num_types; ++t) nb_relu += (tt.n_dst[t] + rpb - 1) / rpb;
  if (bpart && (size_t)nb_relu > bpart_rows) {  // the caller sized the area for another form of the row pass
    set_error("partial bias sums: %d rows for an area of %zu", nb_relu, bpart_rows);
    return HGNN_EINVAL;
  }
  const int segs = rt.num_rels + tt.num_types;
  const int nb_zero = do_zero ? 32 * segs : 0, nb_pad = wpad ? 64 * segs : 0;
  const int blocks = nb_relu + nb_zero + nb_pad;
  if (blocks == 0) return HGNN_OK;
#define HGNN_PREP(TY, VE)                                                                                              \
  HGNN_LAUNCH((bwd_prep_kernel<TY, VE>), dim3(blocks), dim3(256), 0, s, tt, rt, pt, wo, gt, H, ldo, relu, write,        \
              (const TY *)grad_h, (const TY *)h, (TY *)gp, bpart, nb_relu, nb_zero, (TY *)wpad)
  if (dtype == HGNN_BF16) {
    if (fast) HGNN_PREP(bf16, true); else HGNN_PREP(bf16, false);
  } else {
    if (fast) HGNN_PREP(float, true); else HGNN_PREP(float, false);
  }
#undef HGNN_PREP
  HGNN_HIP(hipGetLastError());
  return HGNN_OK;
}

__global__ void __launch_bounds__(256) bias_reduce_kernel(TypeTab tt, GradPtrTab gt, int H, int rpb, const float *__restrict__ bpart) {
  bias_reduce_part(tt, gt, H, rpb, bpart, blockIdx.x);
}

hgnn_status launch_bias_reduce(hipStream_t s, const TypeTab &tt, const GradPtrTab &gt, int H, int rpb, const float *bpart) {
  HGNN_LAUNCH(bias_reduce_kernel, dim3(bias_reduce_blocks(tt.num_types, H)), dim3(256), 0, s, tt, gt, H, rpb, bpart);
  HGNN_HIP(hipGetLastError());
  return HGNN_OK;
}

__global__ void __launch_bounds__(256) fill_zero_kernel(uint4 *p, size_t n16, char *tail, size_t ntail) {
  const uint4 z = make_uint4(0, 0, 0, 0);
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) p[i] = z;
  if (blockIdx.x == 0 && threadIdx.x < ntail) tail[threadIdx.x] = 0;
}

hgnn_status launch_fill_zero(hipStream_t s, void *p, size_t bytes) {
  if (bytes == 0) return HGNN_OK;
  const size_t n16 = bytes / 16;
  const int blocks = (int)std::min<size_t>(2048, (n16 + 255) / 256 + 1);
  HGNN_LAUNCH(fill_zero_kernel, dim3(blocks), dim3(256), 0, s, (uint4 *)p, n16, (char *)p + n16 * 16, bytes - n16 * 16);
  HGNN_HIP(hipGetLastError());
  return HGNN_OK;
}

// ------------------------------------------------------------------------------------------
// Storage-type conversion of a list of tensors in one launch (blockIdx.y = tensor): bf16 -> fp32 is exact,
// fp32 -> bf16 rounds to nearest even.  The attention variant computes in fp32 whatever the storage type is
// and uses this at its boundary.
struct CvtList {
  const void *src[kCvtItems];
  void *dst[kCvtItems];
  int64_t n[kCvtItems];
  int32_t count;
};
template <bool WIDEN>
__global__ void __launch_bounds__(256) convert_kernel(CvtList cl) {
  const int it = blockIdx.y;
  if (it >= cl.count) return;
  const int64_t n = cl.n[it];
  const int64_t stride = (int64_t)gridDim.x * 256;
  if constexpr (WIDEN) {
    const bf16 *a = (const bf16 *)cl.src[it];
    float *b = (float *)cl.dst[it];
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) b[i] = to_float(a[i]);
  } else {
    const float *a = (const float *)cl.src[it];
    bf16 *b = (bf16 *)cl.dst[it];
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) b[i] = from_float<bf16>(a[i]);
  }
}

hgnn_status launch_convert(hipStream_t s, bool widen, const void *const *src, void *const *dst, const int64_t *n, int count) {
  for (int i0 = 0; i0 < count; i0 += kCvtItems) {
    CvtList cl;
    std::memset(&cl, 0, sizeof(cl));
    int64_t longest = 0;
    for (int i = i0; i < count && i < i0 + kCvtItems; ++i) {
      if (n[i] <= 0) continue;
      cl.src[cl.count] = src[i];
      cl.dst[cl.count] = dst[i];
      cl.n[cl.count] = n[i];
      longest = std::max(longest, n[i]);
      ++cl.count;
    }
    if (cl.count == 0) continue;
    const int bx = (int)std::min<int64_t>(1024, (longest + 255) / 256);
    if (widen) HGNN_LAUNCH(convert_kernel<true>, dim3(bx, cl.count), dim3(256), 0, s, cl);
    else HGNN_LAUNCH(convert_kernel<false>, dim3(bx, cl.count), dim3(256), 0, s, cl);
    HGNN_HIP(hipGetLastError());
  }
  return HGNN_OK;
}

// ------------------------------------------------------------------------------------------
// Naive-structure helper: h = act(acc32 + bias) for one vertex type.
// ------------------------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(256) bias_act_kernel(int64_t row0, int64_t n_rows, int H, int relu, const float *bias,
                                                        const float *__restrict__ acc, T *__restrict__ h) {
  const int64_t n = n_rows * H;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
    float v = acc[row0 * H + i];
    if (bias) v += bias[i % H];
    if (relu) v = fmaxf(v, 0.f);
    h[row0 * H + i] = from_float<T>(v);
  }
}

template <typename T>
__global__ void __launch_bounds__(256) bias_act_typed_kernel(int64_t row0, int64_t n_rows, int H, int relu, const T *bias,
                                                              const float *__restrict__ acc, T *__restrict__ h) {
  const int64_t n = n_rows * H;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
    float v = acc[row0 * H + i];
    if (bias) v += to_float(bias[i % H]);
    if (relu) v = fmaxf(v, 0.f);
    h[row0 * H + i] = from_float<T>(v);
  }
}

hgnn_status launch_bias_act(hipStream_t s, int dtype, const TypeTab &tt, const PtrTab &pt, int H, int relu,
                            int type, const float *acc32, void *h) {
  const int64_t n_rows = tt.n_dst[type];
  if (n_rows == 0) return HGNN_OK;
  const int blocks = (int)std::min<int64_t>(4096, (n_rows * H + 255) / 256);
  if (dtype == HGNN_BF16)
    HGNN_LAUNCH(bias_act_typed_kernel<bf16>, dim3(blocks), dim3(256), 0, s, (int64_t)tt.out_row_off[type], n_rows, H,
                       relu, (const bf16 *)pt.bias[type], acc32, (bf16 *)h);
  else
    HGNN_LAUNCH(bias_act_typed_kernel<float>, dim3(blocks), dim3(256), 0, s, (int64_t)tt.out_row_off[type], n_rows, H,
                       relu, (const float *)pt.bias[type], acc32, (float *)h);
  HGNN_HIP(hipGetLastError());
  return HGNN_OK;
}

// ------------------------------------------------------------------------------------------
// Mean softmax cross-entropy and its gradient.
// ------------------------------------------------------------------------------------------
// V = values a lane keeps per row (C <= 64 V).  A wavefront takes kXentRows rows at a time: their values and labels are
// read with unconditional loads (clamped indices) that are all in flight together, so a trip costs one memory round
// trip, and the arithmetic runs out of registers.  The loss leaves a block as ONE atomic add, and the grid is kept to
// 256 blocks: adds to one address are serialised by the memory system at ~11 ns each (1024 blocks of one row per
// wavefront spent 11 of their 16 us there).  V = 0 is the form for any C, which re-reads a row for each of its passes.
constexpr int kXentRows = 4;
template <typename T, int V>
__global__ void __launch_bounds__(256) xent_kernel(const T *__restrict__ logits, const int64_t *__restrict__ labels,
                                                    int64_t rows, int C, float *loss, T *__restrict__ grad) {
  __shared__ float part[4];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const float inv_rows = 1.0f / (float)rows;
  float my_loss = 0.f;
  if constexpr (V > 0) {
    for (int64_t row0 = ((int64_t)blockIdx.x * 4 + wave) * kXentRows; row0 < rows; row0 += (int64_t)gridDim.x * 4 * kXentRows) {
      float x[kXentRows][V];
      int lab[kXentRows];
#pragma unroll
      for (int j = 0; j < kXentRows; ++j) {
        const int64_t row = min(row0 + j, rows - 1);
        lab[j] = (int)labels[row];
#pragma unroll
        for (int i = 0; i < V; ++i) {
          const int c = lane + 64 * i;
          const float v = to_float(logits[row * C + min(c, C - 1)]);
          x[j][i] = c < C ? v : -INFINITY;
        }
      }
#pragma unroll
      for (int j = 0; j < kXentRows; ++j) {
        if (row0 + j >= rows) break;
        float m = x[j][0];
#pragma unroll
        for (int i = 1; i < V; ++i) m = fmaxf(m, x[j][i]);
        for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
        float sum = 0.f, zl = 0.f;
#pragma unroll
        for (int i = 0; i < V; ++i) {
          if (lane + 64 * i == lab[j]) zl = x[j][i];
          x[j][i] = __expf(x[j][i] - m);   // exp(-inf) = 0 beyond the row
          sum += x[j][i];
        }
        for (int o = 32; o > 0; o >>= 1) {
          sum += __shfl_xor(sum, o);
          zl += __shfl_xor(zl, o);
        }
        const float inv_sum = 1.0f / sum;
#pragma unroll
        for (int i = 0; i < V; ++i) {
          const int c = lane + 64 * i;
          float p = x[j][i] * inv_sum;
          if (c == lab[j]) p -= 1.0f;
          if (c < C) grad[(row0 + j) * C + c] = from_float<T>(p * inv_rows);
        }
        my_loss += (logf(sum) + m - zl) * inv_rows;
      }
    }
  } else {
    for (int64_t row = (int64_t)blockIdx.x * 4 + wave; row < rows; row += (int64_t)gridDim.x * 4) {
      const T *z = logits + row * C;
      const int lab = (int)labels[row];
      float m = -INFINITY;
      for (int c = lane; c < C; c += 64) m = fmaxf(m, to_float(z[c]));
      for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
      float sum = 0.f;
      for (int c = lane; c < C; c += 64) sum += __expf(to_float(z[c]) - m);
      for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
      const float inv_sum = 1.0f / sum;
      for (int c = lane; c < C; c += 64) {
        float p = __expf(to_float(z[c]) - m) * inv_sum;
        if (c == lab) p -= 1.0f;
        grad[row * C + c] = from_float<T>(p * inv_rows);
      }
      my_loss += (logf(sum) + m - to_float(z[lab])) * inv_rows;
    }
  }
  if (lane == 0) part[wave] = my_loss;
  __syncthreads();
  if (threadIdx.x == 0) atomicAdd(loss, part[0] + part[1] + part[2] + part[3]);
}

template <typename T>
static void launch_xent_typed(hipStream_t s, const void *logits, const int64_t *labels, int64_t rows, int C, float *loss, void *grad) {
  dim3 grid((unsigned)std::min<int64_t>(256, (rows + 4 * kXentRows - 1) / (4 * kXentRows)));
#define HGNN_XENT(V_) HGNN_LAUNCH((xent_kernel<T, V_>), grid, dim3(256), 0, s, (const T *)logits, labels, rows, C, loss, (T *)grad)
  if (C <= 128) HGNN_XENT(2);
  else if (C <= 256) HGNN_XENT(4);
  else if (C <= 384) HGNN_XENT(6);
  else if (C <= 512) HGNN_XENT(8);
  else HGNN_XENT(0);
#undef HGNN_XENT
}

hgnn_status launch_xent(hipStream_t s, int dtype, const void *logits, const int64_t *labels, int64_t rows,
                        int classes, float *loss, void *grad) {
  hgnn_status st = launch_fill_zero(s, loss, sizeof(float));
  if (st != HGNN_OK) return st;
  if (rows == 0) return HGNN_OK;
  if (dtype == HGNN_BF16) launch_xent_typed<bf16>(s, logits, labels, rows, classes, loss, grad);
  else launch_xent_typed<float>(s, logits, labels, rows, classes, loss, grad);
  HGNN_HIP(hipGetLastError());
  return HGNN_OK;
}

}  // namespace hgnn
