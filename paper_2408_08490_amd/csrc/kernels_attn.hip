// Attention variant of the layer (the paper evaluates R-GAT, Section 5.1, and names semantic fusion as the
// layer's last stage, Section 2.2), forward part:
//   projection   Z = X W_t per vertex type, all source rows                 (MFMA GEMM, weights read in place)
//   aggregation  one launch over the merged CSR: per row and head a softmax over the row's edges of
//                LeakyReLU(a_src . z_u + a_dst . z_v), evaluated in one pass with a running maximum
//   fusion       semantic attention: tanh MLP scores per relation segment (MFMA GEMM with the row reduction
//                in its epilogue), softmax over the relations of a destination type, weighted sum + bias + act
#include <cstring>

#include "gemm_core.h"

namespace hgnn {

constexpr float kLeaky = 0.2f;
constexpr int kSemDim = 128;
constexpr int kAttnMaxH = 1024;  // widest layer output of the attention variant (64 lanes x 16 bytes)

struct AttnPtrs {
  const void *a_src[kMaxR];
  const void *a_dst[kMaxR];
};
// relations grouped by destination type
struct RelsOfType {
  uint16_t first[kMaxT + 1];
  uint8_t rel[kMaxR];
};

template <typename T> struct Piece;   // 16 bytes of a row as floats
template <> struct Piece<float> {
  static constexpr int N = 4;
  static __device__ __forceinline__ void load(float *f, const float *p) {
    const f32x4 v = *reinterpret_cast<const f32x4 *>(p);
    f[0] = v.x; f[1] = v.y; f[2] = v.z; f[3] = v.w;
  }
  static __device__ __forceinline__ void store(float *p, const float *f) {
    *reinterpret_cast<f32x4 *>(p) = f32x4{f[0], f[1], f[2], f[3]};
  }
};
template <> struct Piece<bf16> {
  static constexpr int N = 8;
  static __device__ __forceinline__ void load(float *f, const bf16 *p) {
    const u32x4 v = *reinterpret_cast<const u32x4 *>(p);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      f[2 * i] = __uint_as_float(v[i] << 16);
      f[2 * i + 1] = __uint_as_float(v[i] & 0xffff0000u);
    }
  }
  static __device__ __forceinline__ void store(bf16 *p, const float *f) {
    *reinterpret_cast<u32x4 *>(p) = u32x4{pack2(f[0], f[1]), pack2(f[2], f[3]), pack2(f[4], f[5]), pack2(f[6], f[7])};
  }
};

__device__ __forceinline__ int find_le(const int32_t *off, int n, int x) {  // largest i in [0, n) with off[i] <= x
  int lo = 0, hi = n;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (off[mid] <= x) lo = mid; else hi = mid;
  }
  return lo;
}

// ------------------------------------------------------------------------------------------
// Projection: Z[row_off[t] + i, :] = X_t[i, :] W_t for every source row of every type.
// TO = type of Z: fp32 with bf16 operands when the layer computes in fp32 on bf16 storage (the products of two bf16
// numbers are exact in fp32, so this is the fp32 projection of the widened inputs up to the order of the adds).
template <typename T, typename TO>
__global__ void __launch_bounds__(kThreads, 2) attn_proj_kernel(TypeTab tt, PtrTab pt, SegTab tiles, int H, const T *__restrict__ x,
                                                              TO *__restrict__ z) {
  __shared__ GemmLds<T> sm;
  const int tile = xcd_tile(blockIdx.x, gridDim.x);
  const int T_ = tt.num_types;
  if (tile >= tiles.tile_off[T_]) return;
  int t = 0;
  while (tile >= tiles.tile_off[t + 1]) ++t;
  const int tiles_n = (H + BN - 1) / BN;
  const int local = tile - tiles.tile_off[t];
  const int m0 = (local / tiles_n) * BM, n0 = (local % tiles_n) * BN;
  const int M = tt.row_off[t + 1] - tt.row_off[t], F = tt.in_dim[t];
  f32x16 acc[2][2];
  zero_acc(acc);
  if (threadIdx.x == 0) put_seg(sm.seg[0], x + tt.elem_off[t], F, reinterpret_cast<const T *>(pt.w_root[t]), H, 0, F);
  __syncthreads();
  gemm_run<T, true, true, false>(acc, sm, 1, M, m0, H, n0);
  write_tile(acc, sm, z + ((int64_t)tt.row_off[t] + m0) * H + n0, H, M - m0, H - n0, [](float v, int, int) { return v; });
}

// ------------------------------------------------------------------------------------------
// Aggregation.  A group of `lpr` lanes owns one merged row; lane q holds 16 bytes of the row; `hl` lanes form a
// head.  Softmax over the row's edges in one pass: running maximum m, running sum l and accumulator rescaled
// whenever the maximum grows.  Saves m and l per (row, head) for the backward pass.
template <typename T>
__global__ void __launch_bounds__(256) attn_agg_kernel(LayerDev L, TypeTab tt, RelTab rt, AttnPtrs ap, int H, int heads, int lpr_log2,
                                                       int hl, const T *__restrict__ z, T *__restrict__ mout,
                                                       float *__restrict__ mx, float *__restrict__ ls) {
  using P = Piece<T>;
  const int lpr = 1 << lpr_log2;
  const int q = threadIdx.x & (lpr - 1);
  const int64_t rho = (int64_t)blockIdx.x * (256 >> lpr_log2) + (threadIdx.x >> lpr_log2);
  if (rho >= L.rows) return;   // whole lane groups leave together
  const int r = find_le(L.rel_row_off, rt.num_rels, (int)rho);
  const int v = (int)rho - L.rel_row_off[r];
  const int d = rt.dst[r];
  const int k = (q * P::N) / (H / heads);
  float as[P::N], ad[P::N], zv[P::N], acc[P::N];
  P::load(as, reinterpret_cast<const T *>(ap.a_src[r]) + q * P::N);
  P::load(ad, reinterpret_cast<const T *>(ap.a_dst[r]) + q * P::N);
  P::load(zv, z + ((int64_t)tt.row_off[d] + v) * H + q * P::N);
  float sd = 0.f;
#pragma unroll
  for (int i = 0; i < P::N; ++i) {
    sd += ad[i] * zv[i];
    acc[i] = 0.f;
  }
  for (int o = hl >> 1; o > 0; o >>= 1) sd += __shfl_xor(sd, o);
  float m = -INFINITY, l = 0.f;
  const int e0 = L.rowptr[rho], e1 = L.rowptr[rho + 1];
  int e = e0;
  for (; e + 2 <= e1; e += 2) {   // two rows in flight
    const int u0 = L.colidx[e], u1 = L.colidx[e + 1];
    float z0[P::N], z1[P::N];
    P::load(z0, z + (int64_t)u0 * H + q * P::N);
    P::load(z1, z + (int64_t)u1 * H + q * P::N);
    float s0 = 0.f, s1 = 0.f;
#pragma unroll
    for (int i = 0; i < P::N; ++i) {
      s0 += as[i] * z0[i];
      s1 += as[i] * z1[i];
    }
    for (int o = hl >> 1; o > 0; o >>= 1) {
      s0 += __shfl_xor(s0, o);
      s1 += __shfl_xor(s1, o);
    }
    s0 += sd; s1 += sd;
    s0 = s0 > 0.f ? s0 : kLeaky * s0;
    s1 = s1 > 0.f ? s1 : kLeaky * s1;
    const float mn = fmaxf(m, fmaxf(s0, s1));
    const float c = __expf(m - mn), p0 = __expf(s0 - mn), p1 = __expf(s1 - mn);
    l = l * c + p0 + p1;
#pragma unroll
    for (int i = 0; i < P::N; ++i) acc[i] = acc[i] * c + p0 * z0[i] + p1 * z1[i];
    m = mn;
  }
  if (e < e1) {
    const int u0 = L.colidx[e];
    float z0[P::N];
    P::load(z0, z + (int64_t)u0 * H + q * P::N);
    float s0 = 0.f;
#pragma unroll
    for (int i = 0; i < P::N; ++i) s0 += as[i] * z0[i];
    for (int o = hl >> 1; o > 0; o >>= 1) s0 += __shfl_xor(s0, o);
    s0 += sd;
    s0 = s0 > 0.f ? s0 : kLeaky * s0;
    const float mn = fmaxf(m, s0);
    const float c = __expf(m - mn), p0 = __expf(s0 - mn);
    l = l * c + p0;
#pragma unroll
    for (int i = 0; i < P::N; ++i) acc[i] = acc[i] * c + p0 * z0[i];
    m = mn;
  }
  const float inv = l > 0.f ? 1.f / l : 0.f;
#pragma unroll
  for (int i = 0; i < P::N; ++i) acc[i] *= inv;
  P::store(mout + rho * H + q * P::N, acc);
  if ((q & (hl - 1)) == 0) {
    mx[rho * heads + k] = e1 > e0 ? m : 0.f;
    ls[rho * heads + k] = l;
  }
}

// ------------------------------------------------------------------------------------------
// Semantic scores: t = tanh(m W_s + b_s) stored for the backward pass; wsum[r] += sum over the segment's rows of q . t
template <typename T>
__global__ void __launch_bounds__(kThreads, 2) attn_sem_kernel(LayerDev L, TypeTab tt, RelTab rt, SegTab tiles, int H,
                                                             const T *__restrict__ mbuf, const T *__restrict__ w_sem,
                                                             const T *__restrict__ b_sem, const T *__restrict__ q_sem,
                                                             T *__restrict__ tbuf, float *__restrict__ wsum) {
  __shared__ GemmLds<T> sm;
  __shared__ float red[4];
  const int tile = xcd_tile(blockIdx.x, gridDim.x);
  const int R = rt.num_rels;
  if (tile >= tiles.tile_off[R]) return;
  const int r = find_le(tiles.tile_off, R, tile);
  const int m0 = (tile - tiles.tile_off[r]) * BM;
  const int M = tt.n_dst[rt.dst[r]];
  const int64_t row0 = L.rel_row_off[r];
  f32x16 acc[2][2];
  zero_acc(acc);
  if (threadIdx.x == 0) put_seg(sm.seg[0], mbuf + row0 * H, H, w_sem, kSemDim, 0, H);
  __syncthreads();
  gemm_run<T, true, true, false>(acc, sm, 1, M, m0, kSemDim, 0);
  float bq[2][2];
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int c = ((threadIdx.x >> 6) & 1) * 64 + j * 32 + (threadIdx.x & 31);
    bq[j][0] = to_float(b_sem[c]);
    bq[j][1] = to_float(q_sem[c]);
  }
  const int wn0 = ((threadIdx.x >> 6) & 1) * 64;
  float part = 0.f;
  const int valid = M - m0;
  write_tile(acc, sm, tbuf + (row0 + m0) * kSemDim, kSemDim, valid, kSemDim, [&](float v, int row, int col) {
    const int j = (col - wn0) >> 5;
    const float t = tanhf(v + bq[j][0]);
    if (row < valid) part += t * bq[j][1];
    return t;
  });
  for (int o = 32; o > 0; o >>= 1) part += __shfl_xor(part, o);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = part;
  __syncthreads();
  if (threadIdx.x == 0) atomicAdd(wsum + r, red[0] + red[1] + red[2] + red[3]);
}

// beta[r] = softmax over the relations with the same destination type of wsum[r] / M_d.
// mode 1 (backward): coef[r] = beta_r (dbeta_r - sum_r' beta_r' dbeta_r') / M_d, the factor of q (1 - t^2).
__global__ void attn_beta_kernel(TypeTab tt, RelTab rt, const float *__restrict__ wsum, float *__restrict__ beta,
                                 const float *__restrict__ dbeta, float *__restrict__ coef, int mode) {
  const int r = threadIdx.x;
  if (r >= rt.num_rels) return;
  const int d = rt.dst[r];
  const int M = tt.n_dst[d];
  if (M == 0) {
    if (mode == 0) beta[r] = 0.f; else coef[r] = 0.f;
    return;
  }
  if (mode == 0) {
    float mxv = -INFINITY;
    for (int o = 0; o < rt.num_rels; ++o)
      if (rt.dst[o] == d) mxv = fmaxf(mxv, wsum[o] / (float)M);
    float s = 0.f;
    for (int o = 0; o < rt.num_rels; ++o)
      if (rt.dst[o] == d) s += __expf(wsum[o] / (float)M - mxv);
    beta[r] = __expf(wsum[r] / (float)M - mxv) / s;
  } else {
    float dot = 0.f;
    for (int o = 0; o < rt.num_rels; ++o)
      if (rt.dst[o] == d) dot += beta[o] * dbeta[o];
    coef[r] = beta[r] * (dbeta[r] - dot) / (float)M;
  }
}

// h[v] = act( sum_{r -> type(v)} beta_r m[rel_row_off[r] + v] + b )
template <typename T>
__global__ void __launch_bounds__(256) attn_fuse_kernel(LayerDev L, TypeTab tt, RelsOfType ro, PtrTab pt, int H, int relu, int lpr_log2,
                                                        const T *__restrict__ mbuf, const float *__restrict__ beta,
                                                        T *__restrict__ h) {
  using P = Piece<T>;
  const int lpr = 1 << lpr_log2;
  const int q = threadIdx.x & (lpr - 1);
  const int64_t row = (int64_t)blockIdx.x * (256 >> lpr_log2) + (threadIdx.x >> lpr_log2);
  const int T_ = tt.num_types;
  if (row >= tt.out_row_off[T_]) return;
  const int d = find_le(tt.out_row_off, T_, (int)row);
  const int v = (int)row - tt.out_row_off[d];
  float acc[P::N];
  const T *bias = reinterpret_cast<const T *>(pt.bias[d]);
  if (bias) P::load(acc, bias + q * P::N);
  else {
#pragma unroll
    for (int i = 0; i < P::N; ++i) acc[i] = 0.f;
  }
  for (int j = ro.first[d]; j < ro.first[d + 1]; ++j) {
    const int r = ro.rel[j];
    const float b = beta[r];
    float mv[P::N];
    P::load(mv, mbuf + ((int64_t)L.rel_row_off[r] + v) * H + q * P::N);
#pragma unroll
    for (int i = 0; i < P::N; ++i) acc[i] += b * mv[i];
  }
  if (relu) {
#pragma unroll
    for (int i = 0; i < P::N; ++i) acc[i] = fmaxf(acc[i], 0.f);
  }
  P::store(h + row * H + q * P::N, acc);
}

// ------------------------------------------------------------------------------------------
// launchers (forward)
static int log2_exact(int n) {
  int l = 0;
  while ((1 << l) < n) ++l;
  return l;
}

hgnn_status launch_attn_proj(hipStream_t s, int dtype, const TypeTab &tt, const PtrTab &w_type_as_root, const SegTab &tiles, int H,
                             const void *x, void *z, bool z_f32) {
  const int n = tiles.tile_off[tt.num_types];
  if (n == 0) return HGNN_OK;
  dim3 grid(round_up8(n)), blk(kThreads);
  if (dtype == HGNN_BF16 && z_f32)
    HGNN_LAUNCH((attn_proj_kernel<bf16, float>), grid, blk, 0, s, tt, w_type_as_root, tiles, H, (const bf16 *)x, (float *)z);
  else if (dtype == HGNN_BF16)
    HGNN_LAUNCH((attn_proj_kernel<bf16, bf16>), grid, blk, 0, s, tt, w_type_as_root, tiles, H, (const bf16 *)x, (bf16 *)z);
  else
    HGNN_LAUNCH((attn_proj_kernel<float, float>), grid, blk, 0, s, tt, w_type_as_root, tiles, H, (const float *)x, (float *)z);
  HGNN_HIP(hipGetLastError());
  return HGNN_OK;
}

hgnn_status launch_attn_agg(hipStream_t s, int dtype, const LayerDev &L, const TypeTab &tt, const RelTab &rt,
                            const void *const *a_src, const void *const *a_dst, int H, int heads, const void *z, void *mout,
                            float *mx, float *ls) {
  if (L.rows == 0) return HGNN_OK;
  AttnPtrs ap;
  std::memset(&ap, 0, sizeof(ap));
  for (int r = 0; r < rt.num_rels; ++r) {
    ap.a_src[r] = a_src[r];
    ap.a_dst[r] = a_dst[r];
  }
  const int es = dtype == HGNN_BF16 ? 2 : 4;
  const int lpr = H * es / 16, l2 = log2_exact(lpr), hl = (H / heads) * es / 16;
  dim3 grid((unsigned)((L.rows + (256 >> l2) - 1) / (256 >> l2)));
  if (dtype == HGNN_BF16)
    HGNN_LAUNCH(attn_agg_kernel<bf16>, grid, dim3(256), 0, s, L, tt, rt, ap, H, heads, l2, hl, (const bf16 *)z, (bf16 *)mout, mx, ls);
  else
    HGNN_LAUNCH(attn_agg_kernel<float>, grid, dim3(256), 0, s, L, tt, rt, ap, H, heads, l2, hl, (const float *)z, (float *)mout, mx, ls);
  HGNN_HIP(hipGetLastError());
  return HGNN_OK;
}

hgnn_status launch_attn_sem(hipStream_t s, int dtype, const LayerDev &L, const TypeTab &tt, const RelTab &rt, int H, const void *mbuf,
                            const void *w_sem, const void *b_sem, const void *q_sem, void *tbuf, float *wsum) {
  SegTab tiles;
  std::memset(&tiles, 0, sizeof(tiles));
  for (int r = 0; r < rt.num_rels; ++r) tiles.tile_off[r + 1] = tiles.tile_off[r] + (tt.n_dst[rt.dst[r]] + BM - 1) / BM;
  tiles.num_segs = rt.num_rels;
  const int n = tiles.tile_off[rt.num_rels];
  if (n == 0) return HGNN_OK;
  dim3 grid(round_up8(n)), blk(kThreads);
  if (dtype == HGNN_BF16)
    HGNN_LAUNCH(attn_sem_kernel<bf16>, grid, blk, 0, s, L, tt, rt, tiles, H, (const bf16 *)mbuf, (const bf16 *)w_sem, (const bf16 *)b_sem,
                (const bf16 *)q_sem, (bf16 *)tbuf, wsum);
  else
    HGNN_LAUNCH(attn_sem_kernel<float>, grid, blk, 0, s, L, tt, rt, tiles, H, (const float *)mbuf, (const float *)w_sem,
                (const float *)b_sem, (const float *)q_sem, (float *)tbuf, wsum);
  HGNN_HIP(hipGetLastError());
  return HGNN_OK;
}

hgnn_status launch_attn_beta(hipStream_t s, const TypeTab &tt, const RelTab &rt, const float *wsum, float *beta, const float *dbeta,
                             float *coef, int mode) {
  HGNN_LAUNCH(attn_beta_kernel, dim3(1), dim3(kMaxR), 0, s, tt, rt, wsum, beta, dbeta, coef, mode);
  HGNN_HIP(hipGetLastError());
  return HGNN_OK;
}

static void rels_of_type(const TypeTab &tt, const RelTab &rt, RelsOfType &ro) {
  std::memset(&ro, 0, sizeof(ro));
  int n = 0;
  for (int d = 0; d < tt.num_types; ++d) {
    ro.first[d] = (uint16_t)n;
    for (int r = 0; r < rt.num_rels; ++r)
      if (rt.dst[r] == d) ro.rel[n++] = (uint8_t)r;
  }
  ro.first[tt.num_types] = (uint16_t)n;
}

hgnn_status launch_attn_fuse(hipStream_t s, int dtype, const LayerDev &L, const TypeTab &tt, const RelTab &rt, const PtrTab &pt, int H,
                             int relu, const void *mbuf, const float *beta, void *h) {
  const int64_t rows = tt.out_row_off[tt.num_types];
  if (rows == 0) return HGNN_OK;
  RelsOfType ro;
  rels_of_type(tt, rt, ro);
  const int es = dtype == HGNN_BF16 ? 2 : 4;
  const int l2 = log2_exact(H * es / 16);
  dim3 grid((unsigned)((rows + (256 >> l2) - 1) / (256 >> l2)));
  if (dtype == HGNN_BF16)
    HGNN_LAUNCH(attn_fuse_kernel<bf16>, grid, dim3(256), 0, s, L, tt, ro, pt, H, relu, l2, (const bf16 *)mbuf, beta, (bf16 *)h);
  else
    HGNN_LAUNCH(attn_fuse_kernel<float>, grid, dim3(256), 0, s, L, tt, ro, pt, H, relu, l2, (const float *)mbuf, beta, (float *)h);
  HGNN_HIP(hipGetLastError());
  return HGNN_OK;
}

// ==========================================================================================
// Backward part.
//   fusion      dbeta_r = sum_v G'_v . m_v^r ; softmax over relations backward -> coef_r (attn_beta_kernel, mode 1)
//               du = coef_r q (1 - t^2), dq, db_s (column sums) ; dW_s += m^T du (MFMA, split over rows)
//               dm = beta_r G'_v + du W_s^T (MFMA)
//   aggregation per merged row: alpha recomputed from the saved maximum and sum; sum_u alpha_u dalpha_u in a first pass;
//               per edge alpha and ds (gradient before the LeakyReLU) are stored by CSR position, da_src / da_dst
//               accumulated in registers over a run of rows; per source row (transpose): dz = sum over its edges
//               of alpha dm_v + ds a_src, plus, for a destination row, sum_r (sum_u ds) a_dst
//   projection  dW_t = X_t^T dZ_t and dX_t = dZ_t W_t^T run on the layer GEMMs of the mean variant.
// ==========================================================================================
struct ZeroList {
  float *p[2 * kMaxR + 8];
  int32_t n[2 * kMaxR + 8];
  int32_t count;
};
__global__ void attn_zero_kernel(ZeroList zl) {
  const int i = blockIdx.y;
  if (i >= zl.count) return;
  float *p = zl.p[i];
  for (int j = blockIdx.x * blockDim.x + threadIdx.x; j < zl.n[i]; j += gridDim.x * blockDim.x) p[j] = 0.f;
}

// dbeta[r] += sum over the rows of relation r of G'[v] . m[row]
template <typename T>
__global__ void __launch_bounds__(256) attn_dbeta_kernel(LayerDev L, TypeTab tt, RelTab rt, int H, int ldg, int lpr_log2, int rows_per_group,
                                                         const T *__restrict__ gp, const T *__restrict__ mbuf,
                                                         float *__restrict__ dbeta) {
  using P = Piece<T>;
  __shared__ float part[kMaxR];
  for (int i = threadIdx.x; i < kMaxR; i += 256) part[i] = 0.f;
  __syncthreads();
  const int lpr = 1 << lpr_log2;
  const int q = threadIdx.x & (lpr - 1);
  const int64_t g0 = ((int64_t)blockIdx.x * (256 >> lpr_log2) + (threadIdx.x >> lpr_log2)) * rows_per_group;
  for (int64_t rho = g0; rho < g0 + rows_per_group && rho < L.rows; ++rho) {
    const int r = find_le(L.rel_row_off, rt.num_rels, (int)rho);
    const int v = (int)rho - L.rel_row_off[r];
    float a[P::N], b[P::N];
    P::load(a, gp + ((int64_t)tt.out_row_off[rt.dst[r]] + v) * ldg + q * P::N);
    P::load(b, mbuf + rho * H + q * P::N);
    float d = 0.f;
#pragma unroll
    for (int i = 0; i < P::N; ++i) d += a[i] * b[i];
    for (int o = lpr >> 1; o > 0; o >>= 1) d += __shfl_xor(d, o);
    if (q == 0) atomicAdd(&part[r], d);
  }
  __syncthreads();
  for (int i = threadIdx.x; i < rt.num_rels; i += 256)
    if (part[i] != 0.f) atomicAdd(dbeta + i, part[i]);
}

// du = coef_r q (1 - t^2); dq[c] += coef_r sum_rows t ; db_s[c] += sum_rows du.  128 columns x 2 row lanes per block.
template <typename T>
__global__ void __launch_bounds__(256) attn_du_kernel(LayerDev L, RelTab rt, int rows_per_block, const T *__restrict__ tbuf,
                                                      const T *__restrict__ q_sem, const float *__restrict__ coef,
                                                      T *__restrict__ du, float *__restrict__ dq, float *__restrict__ dbs) {
  __shared__ float sq[256], sb[256];
  const int c = threadIdx.x & (kSemDim - 1), half = threadIdx.x >> 7;
  const float qc = to_float(q_sem[c]);
  float aq = 0.f, ab = 0.f;
  const int64_t r0 = (int64_t)blockIdx.x * rows_per_block;
  int r = -1, r_end = -1;
  float cf = 0.f;
  for (int64_t rho = r0 + half; rho < r0 + rows_per_block && rho < L.rows; rho += 2) {
    if ((int)rho >= r_end) {
      r = find_le(L.rel_row_off, rt.num_rels, (int)rho);
      r_end = L.rel_row_off[r + 1];
      cf = coef[r];
    }
    const float t = to_float(tbuf[rho * kSemDim + c]);
    const float d = cf * qc * (1.f - t * t);
    du[rho * kSemDim + c] = from_float<T>(d);
    aq += cf * t;
    ab += d;
  }
  sq[threadIdx.x] = aq;
  sb[threadIdx.x] = ab;
  __syncthreads();
  if (half == 0) {
    atomicAdd(dq + c, sq[c] + sq[c + kSemDim]);
    atomicAdd(dbs + c, sb[c] + sb[c + kSemDim]);
  }
}

// dm[row] = du[row] W_s^T + beta_r G'[v]
template <typename T>
__global__ void __launch_bounds__(kThreads, 2) attn_dm_kernel(LayerDev L, TypeTab tt, RelTab rt, SegTab tiles, int H, int ldg,
                                                            const T *__restrict__ du, const T *__restrict__ w_sem,
                                                            const T *__restrict__ gp, const float *__restrict__ beta,
                                                            T *__restrict__ dm) {
  __shared__ GemmLds<T> sm;
  const int tile = xcd_tile(blockIdx.x, gridDim.x);
  const int R = rt.num_rels;
  if (tile >= tiles.tile_off[R]) return;
  const int r = find_le(tiles.tile_off, R, tile);
  const int tiles_n = (H + BN - 1) / BN;
  const int local = tile - tiles.tile_off[r];
  const int m0 = (local / tiles_n) * BM, n0 = (local % tiles_n) * BN;
  const int d = rt.dst[r];
  const int M = tt.n_dst[d];
  const int64_t row0 = L.rel_row_off[r];
  f32x16 acc[2][2];
  zero_acc(acc);
  if (threadIdx.x == 0) put_seg(sm.seg[0], du + row0 * kSemDim, kSemDim, w_sem, kSemDim, 0, kSemDim);
  __syncthreads();
  gemm_run<T, true, true, true>(acc, sm, 1, M, m0, H, n0);
  const float b = beta[r];
  const T *g = gp + ((int64_t)tt.out_row_off[d] + m0) * ldg + n0;
  const int vr = M - m0, vc = H - n0;
  write_tile(acc, sm, dm + (row0 + m0) * H + n0, H, vr, vc, [&](float v, int row, int col) {
    return (row < vr && col < vc) ? v + b * to_float(g[(int64_t)row * ldg + col]) : 0.f;
  });
}

// dW_s += m^T du over the row slice [k_begin, k_end)
template <typename T>
__global__ void __launch_bounds__(kThreads, 2) attn_dws_kernel(int64_t rows, int split_rows, int H, const T *__restrict__ mbuf,
                                                             const T *__restrict__ du, float *__restrict__ dws) {
  __shared__ GemmLds<T> sm;
  const int tiles_f = (H + BM - 1) / BM;
  const int tf = blockIdx.x % tiles_f, sp = blockIdx.x / tiles_f;
  const int64_t k_begin = (int64_t)sp * split_rows;
  if (k_begin >= rows) return;
  const int k_end = (int)(k_begin + split_rows < rows ? k_begin + split_rows : rows);
  f32x16 acc[2][2];
  zero_acc(acc);
  if (threadIdx.x == 0) put_seg(sm.seg[0], mbuf, H, du, kSemDim, (int)k_begin, k_end);
  __syncthreads();
  const int f0 = tf * BM;
  gemm_run<T, true, false, false>(acc, sm, 1, H, f0, kSemDim, 0);
  HGNN_FOR_EACH_ACC({
    if (f0 + row < H) atomicAdd(dws + (int64_t)(f0 + row) * kSemDim + col, val);
  })
}

// Aggregation backward, by merged row.  A lane group walks `rows_per_group` consecutive rows and keeps the sums for
// da_src / da_dst of the current relation in registers; they go out with atomic adds when the relation changes.
template <typename T>
__global__ void __launch_bounds__(256) attn_agg_bwd_rows_kernel(LayerDev L, TypeTab tt, RelTab rt, AttnPtrs ap, AttnPtrs dap, int H, int heads,
                                                                int lpr_log2, int hl, int rows_per_group, const T *__restrict__ z,
                                                                const T *__restrict__ dm,
                                                                const float *__restrict__ mx, const float *__restrict__ ls,
                                                                float *__restrict__ alpha, float *__restrict__ dsb,
                                                                float *__restrict__ dsum) {
  using P = Piece<T>;
  const int lpr = 1 << lpr_log2;
  const int q = threadIdx.x & (lpr - 1);
  const int k = (q * P::N) / (H / heads);
  const bool head_lead = (q & (hl - 1)) == 0;
  const int64_t g0 = ((int64_t)blockIdx.x * (256 >> lpr_log2) + (threadIdx.x >> lpr_log2)) * rows_per_group;
  // The block's sums for da_src / da_dst meet in LDS first (nearly every block lies inside one relation); only a
  // group in another relation than the block's first row adds to global memory directly.
  __shared__ float s_das[kAttnMaxH], s_dad[kAttnMaxH];
  __shared__ int s_rel;
  for (int i = threadIdx.x; i < H; i += 256) s_das[i] = s_dad[i] = 0.f;
  if (threadIdx.x == 0) {
    const int64_t first = (int64_t)blockIdx.x * (256 >> lpr_log2) * rows_per_group;
    s_rel = first < L.rows ? find_le(L.rel_row_off, rt.num_rels, (int)first) : -1;
  }
  __syncthreads();
  int r = -1;
  float as[P::N], ad[P::N], das[P::N], dad[P::N];
  auto flush = [&]() {
    if (r < 0) return;
    if (r == s_rel) {
#pragma unroll
      for (int i = 0; i < P::N; ++i) {
        if (das[i] != 0.f) atomicAdd(&s_das[q * P::N + i], das[i]);
        if (dad[i] != 0.f) atomicAdd(&s_dad[q * P::N + i], dad[i]);
      }
      return;
    }
    float *ps = reinterpret_cast<float *>(const_cast<void *>(dap.a_src[r])) + q * P::N;
    float *pd = reinterpret_cast<float *>(const_cast<void *>(dap.a_dst[r])) + q * P::N;
#pragma unroll
    for (int i = 0; i < P::N; ++i) {
      if (das[i] != 0.f) atomicAdd(ps + i, das[i]);
      if (dad[i] != 0.f) atomicAdd(pd + i, dad[i]);
    }
  };
  for (int64_t rho = g0; rho < g0 + rows_per_group && rho < L.rows; ++rho) {
    if (r < 0 || (int)rho >= L.rel_row_off[r + 1]) {
      flush();
      r = find_le(L.rel_row_off, rt.num_rels, (int)rho);
      P::load(as, reinterpret_cast<const T *>(ap.a_src[r]) + q * P::N);
      P::load(ad, reinterpret_cast<const T *>(ap.a_dst[r]) + q * P::N);
#pragma unroll
      for (int i = 0; i < P::N; ++i) das[i] = dad[i] = 0.f;
    }
    const int e0 = L.rowptr[rho], e1 = L.rowptr[rho + 1];
    if (e1 == e0) {
      if (head_lead) dsum[rho * heads + k] = 0.f;
      continue;
    }
    const int v = (int)rho - L.rel_row_off[r];
    const int d = rt.dst[r];
    float zv[P::N], g[P::N];
    P::load(zv, z + ((int64_t)tt.row_off[d] + v) * H + q * P::N);
    P::load(g, dm + rho * H + q * P::N);
    float sd = 0.f;
#pragma unroll
    for (int i = 0; i < P::N; ++i) sd += ad[i] * zv[i];
    for (int o = hl >> 1; o > 0; o >>= 1) sd += __shfl_xor(sd, o);
    const float mxk = mx[rho * heads + k], inv_l = 1.f / ls[rho * heads + k];
    // first pass: gm = sum_u alpha_u dalpha_u, summed edge by edge.  (It equals dm . m in exact arithmetic, but the
    // stored m is rounded to the storage type and the difference would not cancel in alpha (dalpha - gm).)
    float gm = 0.f;
    // both passes take four edges at a time: their source rows are loaded together (independent loads in
    // flight), the sums are then taken edge by edge in the row's order
    constexpr int U = 4;
    auto dots = [&](const float (&zu)[P::N], float &ss, float &da) {
      ss = 0.f;
      da = 0.f;
#pragma unroll
      for (int i = 0; i < P::N; ++i) {
        ss += as[i] * zu[i];
        da += g[i] * zu[i];
      }
      for (int o = hl >> 1; o > 0; o >>= 1) {
        ss += __shfl_xor(ss, o);
        da += __shfl_xor(da, o);
      }
    };
    for (int eb = e0; eb < e1; eb += U) {
      float zu[U][P::N];
#pragma unroll
      for (int j = 0; j < U; ++j) {
        const int u = L.colidx[min(eb + j, e1 - 1)];
        P::load(zu[j], z + (int64_t)u * H + q * P::N);
      }
#pragma unroll
      for (int j = 0; j < U; ++j) {
        if (eb + j >= e1) break;
        float ss, da;
        dots(zu[j], ss, da);
        const float sc = ss + sd;
        const float ev = sc > 0.f ? sc : kLeaky * sc;
        gm += __expf(ev - mxk) * inv_l * da;
      }
    }
    float dsv_sum = 0.f;
    for (int eb = e0; eb < e1; eb += U) {
      float zu[U][P::N];
#pragma unroll
      for (int j = 0; j < U; ++j) {
        const int u = L.colidx[min(eb + j, e1 - 1)];
        P::load(zu[j], z + (int64_t)u * H + q * P::N);
      }
#pragma unroll
      for (int j = 0; j < U; ++j) {
        const int e = eb + j;
        if (e >= e1) break;
        float ss, da;
        dots(zu[j], ss, da);
        const float sc = ss + sd;
        const float ev = sc > 0.f ? sc : kLeaky * sc;
        const float a = __expf(ev - mxk) * inv_l;
        const float dsv = a * (da - gm) * (sc > 0.f ? 1.f : kLeaky);
        if (head_lead) {
          alpha[(int64_t)e * heads + k] = a;
          dsb[(int64_t)e * heads + k] = dsv;
        }
#pragma unroll
        for (int i = 0; i < P::N; ++i) das[i] += dsv * zu[j][i];
        dsv_sum += dsv;
      }
    }
#pragma unroll
    for (int i = 0; i < P::N; ++i) dad[i] += dsv_sum * zv[i];
    if (head_lead) dsum[rho * heads + k] = dsv_sum;
  }
  flush();
  __syncthreads();
  if (s_rel >= 0) {
    float *ps = reinterpret_cast<float *>(const_cast<void *>(dap.a_src[s_rel]));
    float *pd = reinterpret_cast<float *>(const_cast<void *>(dap.a_dst[s_rel]));
    for (int i = threadIdx.x; i < H; i += 256) {
      if (s_das[i] != 0.f) atomicAdd(ps + i, s_das[i]);
      if (s_dad[i] != 0.f) atomicAdd(pd + i, s_dad[i]);
    }
  }
}

// Aggregation backward, by source row (transpose): dz[c] = sum_j alpha_j dm[crow_j] + ds_j a_src[rel(crow_j)]
// (+ for a destination row: sum over the relations ending in its type of dsum[row] a_dst[r]).
// Work items: one per source row (rows longer than kLongRow entries are left to the chunk items), then one per
// chunk of a long row, which writes an fp32 partial sum; attn_agg_bwd_long_kernel adds a long row's partials up.
template <typename T>
__global__ void __launch_bounds__(256) attn_agg_bwd_cols_kernel(LayerDev L, TypeTab tt, RelTab rt, RelsOfType ro, AttnPtrs ap, int H, int heads,
                                                                int lpr_log2, const T *__restrict__ dm, const float *__restrict__ alpha,
                                                                const float *__restrict__ dsb, const float *__restrict__ dsum,
                                                                T *__restrict__ dz, float *__restrict__ partial) {
  using P = Piece<T>;
  const int lpr = 1 << lpr_log2;
  const int q = threadIdx.x & (lpr - 1);
  const int k = (q * P::N) / (H / heads);
  const int64_t item = (int64_t)blockIdx.x * (256 >> lpr_log2) + (threadIdx.x >> lpr_log2);
  if (item >= (int64_t)L.src_rows + L.n_chunks) return;
  const bool chunk = item >= L.src_rows;
  const int64_t c = chunk ? L.chunk_row[item - L.src_rows] : item;
  int j0 = L.cptr[c], j1 = L.cptr[c + 1];
  if (chunk) {
    j0 = L.chunk_beg[item - L.src_rows];
    j1 = min(j1, j0 + kChunk);
  } else if (j1 - j0 > kLongRow) {
    return;
  }
  float acc[P::N];
#pragma unroll
  for (int i = 0; i < P::N; ++i) acc[i] = 0.f;
  int r_lo = 0, r_hi = 0;
  float as[P::N];
  auto rel_of = [&](int rho) {
    if (rho < r_lo || rho >= r_hi) {
      const int r = find_le(L.rel_row_off, rt.num_rels, rho);
      r_lo = L.rel_row_off[r];
      r_hi = L.rel_row_off[r + 1];
      P::load(as, reinterpret_cast<const T *>(ap.a_src[r]) + q * P::N);
    }
  };
  int j = j0;
  for (; j + 2 <= j1; j += 2) {   // two rows of dm in flight
    const int rho0 = L.crow[j], e0 = L.cperm[j], rho1 = L.crow[j + 1], e1 = L.cperm[j + 1];
    float g0[P::N], g1[P::N];
    P::load(g0, dm + (int64_t)rho0 * H + q * P::N);
    P::load(g1, dm + (int64_t)rho1 * H + q * P::N);
    const float a0 = alpha[(int64_t)e0 * heads + k], d0 = dsb[(int64_t)e0 * heads + k];
    const float a1 = alpha[(int64_t)e1 * heads + k], d1 = dsb[(int64_t)e1 * heads + k];
    rel_of(rho0);
#pragma unroll
    for (int i = 0; i < P::N; ++i) acc[i] += a0 * g0[i] + d0 * as[i];
    rel_of(rho1);
#pragma unroll
    for (int i = 0; i < P::N; ++i) acc[i] += a1 * g1[i] + d1 * as[i];
  }
  if (j < j1) {
    const int rho0 = L.crow[j], e0 = L.cperm[j];
    float g0[P::N];
    P::load(g0, dm + (int64_t)rho0 * H + q * P::N);
    const float a0 = alpha[(int64_t)e0 * heads + k], d0 = dsb[(int64_t)e0 * heads + k];
    rel_of(rho0);
#pragma unroll
    for (int i = 0; i < P::N; ++i) acc[i] += a0 * g0[i] + d0 * as[i];
  }
  if (chunk) {
    float *pp = partial + (item - L.src_rows) * H + q * P::N;
#pragma unroll
    for (int i = 0; i < P::N; ++i) pp[i] = acc[i];
    return;
  }
  const int t = find_le(tt.row_off, tt.num_types, (int)c);
  const int v = (int)c - tt.row_off[t];
  if (v < tt.n_dst[t]) {
    for (int jj = ro.first[t]; jj < ro.first[t + 1]; ++jj) {
      const int rr = ro.rel[jj];
      const float sv = dsum[((int64_t)L.rel_row_off[rr] + v) * heads + k];
      float ad[P::N];
      P::load(ad, reinterpret_cast<const T *>(ap.a_dst[rr]) + q * P::N);
#pragma unroll
      for (int i = 0; i < P::N; ++i) acc[i] += sv * ad[i];
    }
  }
  P::store(dz + c * H + q * P::N, acc);
}

// Long rows: one block per row adds the chunk partials (threads form groups over four columns each, group g takes
// chunks g, g + groups, ...; LDS adds the groups), then the destination-side term, and writes the row.
template <typename T>
__global__ void __launch_bounds__(256) attn_agg_bwd_long_kernel(LayerDev L, TypeTab tt, RelsOfType ro, AttnPtrs ap, int H, int heads,
                                                                const float *__restrict__ partial, const float *__restrict__ dsum,
                                                                T *__restrict__ dz) {
  __shared__ float red[256 * 4];
  const int i = blockIdx.x;
  const int c = L.long_row[i];
  const int j0 = L.long_chunk0[i], j1 = L.long_chunk0[i + 1];
  const int nw = H / 4;
  int lanes = 1;
  while (lanes < nw && lanes < 256) lanes <<= 1;
  const int groups = 256 / lanes, g = threadIdx.x / lanes, ln = threadIdx.x % lanes;
  const int t = find_le(tt.row_off, tt.num_types, c);
  const int v = c - tt.row_off[t];
  for (int q0 = 0; q0 < nw; q0 += lanes) {
    const int q = q0 + ln;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    if (q < nw) {
      int j = j0 + g;
      for (; j + 3 * groups < j1; j += 4 * groups) {
        const f32x4 v0 = *reinterpret_cast<const f32x4 *>(partial + (int64_t)j * H + q * 4);
        const f32x4 v1 = *reinterpret_cast<const f32x4 *>(partial + (int64_t)(j + groups) * H + q * 4);
        const f32x4 v2 = *reinterpret_cast<const f32x4 *>(partial + (int64_t)(j + 2 * groups) * H + q * 4);
        const f32x4 v3 = *reinterpret_cast<const f32x4 *>(partial + (int64_t)(j + 3 * groups) * H + q * 4);
        acc += (v0 + v1) + (v2 + v3);
      }
      for (; j < j1; j += groups) acc += *reinterpret_cast<const f32x4 *>(partial + (int64_t)j * H + q * 4);
    }
    if (groups > 1) {
      *reinterpret_cast<f32x4 *>(red + threadIdx.x * 4) = acc;
      __syncthreads();
      if (g == 0)
        for (int o = 1; o < groups; ++o) acc += *reinterpret_cast<const f32x4 *>(red + (o * lanes + ln) * 4);
    }
    if (g == 0 && q < nw) {
      const int k = (q * 4) / (H / heads);
      if (v < tt.n_dst[t]) {
        for (int jj = ro.first[t]; jj < ro.first[t + 1]; ++jj) {
          const int rr = ro.rel[jj];
          const float sv = dsum[((int64_t)L.rel_row_off[rr] + v) * heads + k];
          const T *ad = reinterpret_cast<const T *>(ap.a_dst[rr]) + q * 4;
#pragma unroll
          for (int e = 0; e < 4; ++e) acc[e] += sv * to_float(ad[e]);
        }
      }
#pragma unroll
      for (int e = 0; e < 4; ++e) dz[(int64_t)c * H + q * 4 + e] = from_float<T>(acc[e]);
    }
    if (groups > 1) __syncthreads();
  }
}

// ------------------------------------------------------------------------------------------
// launchers (backward)
hgnn_status launch_attn_zero(hipStream_t s, float *const *ptrs, const int64_t *counts, int n) {
  ZeroList zl;
  std::memset(&zl, 0, sizeof(zl));
  for (int i = 0; i < n; ++i) {
    if (!ptrs[i] || counts[i] <= 0) continue;
    zl.p[zl.count] = ptrs[i];
    zl.n[zl.count] = (int32_t)counts[i];
    ++zl.count;
  }
  if (zl.count == 0) return HGNN_OK;
  HGNN_LAUNCH(attn_zero_kernel, dim3(32, zl.count), dim3(256), 0, s, zl);
  HGNN_HIP(hipGetLastError());
  return HGNN_OK;
}

hgnn_status launch_attn_dbeta(hipStream_t s, int dtype, const LayerDev &L, const TypeTab &tt, const RelTab &rt, int H, int ldg,
                              const void *gp, const void *mbuf, float *dbeta) {
  if (L.rows == 0) return HGNN_OK;
  const int es = dtype == HGNN_BF16 ? 2 : 4;
  const int l2 = log2_exact(H * es / 16), gpb = 256 >> l2, rpg = 16;
  dim3 grid((unsigned)((L.rows + (int64_t)gpb * rpg - 1) / ((int64_t)gpb * rpg)));
  if (dtype == HGNN_BF16) HGNN_LAUNCH(attn_dbeta_kernel<bf16>, grid, dim3(256), 0, s, L, tt, rt, H, ldg, l2, rpg, (const bf16 *)gp, (const bf16 *)mbuf, dbeta);
  else HGNN_LAUNCH(attn_dbeta_kernel<float>, grid, dim3(256), 0, s, L, tt, rt, H, ldg, l2, rpg, (const float *)gp, (const float *)mbuf, dbeta);
  HGNN_HIP(hipGetLastError());
  return HGNN_OK;
}

hgnn_status launch_attn_du(hipStream_t s, int dtype, const LayerDev &L, const RelTab &rt, const void *tbuf, const void *q_sem,
                           const float *coef, void *du, float *dq, float *dbs) {
  if (L.rows == 0) return HGNN_OK;
  const int rpb = 256;
  dim3 grid((unsigned)((L.rows + rpb - 1) / rpb));
  if (dtype == HGNN_BF16) HGNN_LAUNCH(attn_du_kernel<bf16>, grid, dim3(256), 0, s, L, rt, rpb, (const bf16 *)tbuf, (const bf16 *)q_sem, coef, (bf16 *)du, dq, dbs);
  else HGNN_LAUNCH(attn_du_kernel<float>, grid, dim3(256), 0, s, L, rt, rpb, (const float *)tbuf, (const float *)q_sem, coef, (float *)du, dq, dbs);
  HGNN_HIP(hipGetLastError());
  return HGNN_OK;
}

hgnn_status launch_attn_dm(hipStream_t s, int dtype, const LayerDev &L, const TypeTab &tt, const RelTab &rt, int H, int ldg, const void *du,
                           const void *w_sem, const void *gp, const float *beta, void *dm) {
  SegTab tiles;
  std::memset(&tiles, 0, sizeof(tiles));
  const int tn = (H + BN - 1) / BN;
  for (int r = 0; r < rt.num_rels; ++r) tiles.tile_off[r + 1] = tiles.tile_off[r] + ((tt.n_dst[rt.dst[r]] + BM - 1) / BM) * tn;
  tiles.num_segs = rt.num_rels;
  const int n = tiles.tile_off[rt.num_rels];
  if (n == 0) return HGNN_OK;
  dim3 grid(round_up8(n)), blk(kThreads);
  if (dtype == HGNN_BF16)
    HGNN_LAUNCH(attn_dm_kernel<bf16>, grid, blk, 0, s, L, tt, rt, tiles, H, ldg, (const bf16 *)du, (const bf16 *)w_sem, (const bf16 *)gp, beta, (bf16 *)dm);
  else
    HGNN_LAUNCH(attn_dm_kernel<float>, grid, blk, 0, s, L, tt, rt, tiles, H, ldg, (const float *)du, (const float *)w_sem, (const float *)gp, beta, (float *)dm);
  HGNN_HIP(hipGetLastError());
  return HGNN_OK;
}

hgnn_status launch_attn_dws(hipStream_t s, int dtype, int64_t rows, int H, const void *mbuf, const void *du, float *dws) {
  if (rows == 0) return HGNN_OK;
  const int split_rows = 2048;
  const int tiles_f = (H + BM - 1) / BM;
  dim3 grid((unsigned)(tiles_f * ((rows + split_rows - 1) / split_rows))), blk(kThreads);
  if (dtype == HGNN_BF16) HGNN_LAUNCH(attn_dws_kernel<bf16>, grid, blk, 0, s, rows, split_rows, H, (const bf16 *)mbuf, (const bf16 *)du, dws);
  else HGNN_LAUNCH(attn_dws_kernel<float>, grid, blk, 0, s, rows, split_rows, H, (const float *)mbuf, (const float *)du, dws);
  HGNN_HIP(hipGetLastError());
  return HGNN_OK;
}

hgnn_status launch_attn_agg_bwd(hipStream_t s, int dtype, const LayerDev &L, const TypeTab &tt, const RelTab &rt, const void *const *a_src,
                                const void *const *a_dst, float *const *da_src, float *const *da_dst, int H, int heads, const void *z,
                                const void *mbuf, const void *dm, const float *mx, const float *ls, float *alpha, float *dsb,
                                float *dsum, void *dz, float *partial) {
  AttnPtrs ap, dap;
  std::memset(&ap, 0, sizeof(ap));
  std::memset(&dap, 0, sizeof(dap));
  for (int r = 0; r < rt.num_rels; ++r) {
    ap.a_src[r] = a_src[r];
    ap.a_dst[r] = a_dst[r];
    dap.a_src[r] = da_src[r];
    dap.a_dst[r] = da_dst[r];
  }
  const int es = dtype == HGNN_BF16 ? 2 : 4;
  const int lpr = H * es / 16, l2 = log2_exact(lpr), hl = (H / heads) * es / 16, gpb = 256 >> l2, rpg = 8;
  if (L.rows > 0) {
    dim3 grid((unsigned)((L.rows + (int64_t)gpb * rpg - 1) / ((int64_t)gpb * rpg)));
    if (dtype == HGNN_BF16)
      HGNN_LAUNCH(attn_agg_bwd_rows_kernel<bf16>, grid, dim3(256), 0, s, L, tt, rt, ap, dap, H, heads, l2, hl, rpg, (const bf16 *)z,
                  (const bf16 *)dm, mx, ls, alpha, dsb, dsum);
    else
      HGNN_LAUNCH(attn_agg_bwd_rows_kernel<float>, grid, dim3(256), 0, s, L, tt, rt, ap, dap, H, heads, l2, hl, rpg, (const float *)z,
                  (const float *)dm, mx, ls, alpha, dsb, dsum);
    HGNN_HIP(hipGetLastError());
  }
  if (L.src_rows > 0) {
    RelsOfType ro;
    rels_of_type(tt, rt, ro);
    dim3 grid((unsigned)(((int64_t)L.src_rows + L.n_chunks + gpb - 1) / gpb));
    if (dtype == HGNN_BF16)
      HGNN_LAUNCH(attn_agg_bwd_cols_kernel<bf16>, grid, dim3(256), 0, s, L, tt, rt, ro, ap, H, heads, l2, (const bf16 *)dm, alpha, dsb, dsum,
                  (bf16 *)dz, partial);
    else
      HGNN_LAUNCH(attn_agg_bwd_cols_kernel<float>, grid, dim3(256), 0, s, L, tt, rt, ro, ap, H, heads, l2, (const float *)dm, alpha, dsb, dsum,
                  (float *)dz, partial);
    HGNN_HIP(hipGetLastError());
    if (L.n_long > 0) {
      if (dtype == HGNN_BF16)
        HGNN_LAUNCH(attn_agg_bwd_long_kernel<bf16>, dim3(L.n_long), dim3(256), 0, s, L, tt, ro, ap, H, heads, partial, dsum, (bf16 *)dz);
      else
        HGNN_LAUNCH(attn_agg_bwd_long_kernel<float>, dim3(L.n_long), dim3(256), 0, s, L, tt, ro, ap, H, heads, partial, dsum, (float *)dz);
      HGNN_HIP(hipGetLastError());
    }
  }
  return HGNN_OK;
}

}  // namespace hgnn
