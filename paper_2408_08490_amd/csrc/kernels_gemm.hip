// MFMA GEMMs of the layer path (gfx950, wave64):
//   forward : h_d = act( [Z_r1 | Z_r2 | ... | X_d] . [W_r1; W_r2; ...; W_0^d] + b_d )   per destination type d
//             -- projection and semantic fusion in one contraction (the K loop walks the relations that
//             end in d, then the root term), bias and activation in the epilogue;
//   dA      : dZ_s = (G' W_s^T) scaled per row by 1/|N_r(v)|                          per K-segment s
//   dW      : dW_s = A_s^T G'  (reduction over the destination rows, split and added atomically)
// One 256-thread block (2x2 wavefronts) computes a 128x128 tile; every wavefront owns 64x64 of it as
// 2x2 MFMA 32x32 accumulators.  Operands go global -> registers -> LDS (next tile's global loads are in
// flight while the current one is multiplied).  An operand is kept in LDS the way it lies in memory:
// "KC" = the reduction index is contiguous (rows = output index), "KS" = the output index is contiguous.
#include "common.h"
#include "device_types.h"

namespace hgnn {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));

constexpr int BM = 128, BN = 128, kThreads = 256;

template <typename T> struct Mma;
template <> struct Mma<bf16> {
  static constexpr int BK = 32, KSTEP = 16, VEC = 8, PKC = BK + 8, PKS = 128 + 4;
};
template <> struct Mma<float> {
  static constexpr int BK = 16, KSTEP = 2, VEC = 4, PKC = BK + 4, PKS = 128 + 4;
};
template <typename T> constexpr int lds_elems() {
  return (BM * Mma<T>::PKC > Mma<T>::BK * Mma<T>::PKS) ? BM * Mma<T>::PKC : Mma<T>::BK * Mma<T>::PKS;
}

// One operand tile on its way global -> registers -> LDS.  The tile is ROWS x COLS in the operand's own
// row-major orientation (COLS contiguous); out-of-range parts are zero-filled.
template <typename T, int ROWS, int COLS, int PITCH>
struct TileMover {
  static constexpr int VEC = 16 / sizeof(T), VPR = COLS / VEC, NV = ROWS * VPR / kThreads;
  static_assert(ROWS * VPR % kThreads == 0, "tile must split evenly over the block");
  uint4 reg[NV];
  __device__ __forceinline__ void load(const T *base, int64_t ld, int nrows, int ncols, int r0, int c0, bool vec_ok) {
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int v = threadIdx.x + i * kThreads;
      const int gr = r0 + v / VPR, gc = c0 + (v % VPR) * VEC;
      uint4 val = make_uint4(0, 0, 0, 0);
      if (gr < nrows && gc < ncols) {
        const T *p = base + (int64_t)gr * ld + gc;
        if (vec_ok && gc + VEC <= ncols) {
          val = *reinterpret_cast<const uint4 *>(p);
        } else {
          union { uint4 u; T e[VEC]; } tmp;
          tmp.u = make_uint4(0, 0, 0, 0);
#pragma unroll
          for (int j = 0; j < VEC; ++j)
            if (gc + j < ncols) tmp.e[j] = p[j];
          val = tmp.u;
        }
      }
      reg[i] = val;
    }
  }
  __device__ __forceinline__ void store(T *lds) const {
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int v = threadIdx.x + i * kThreads;
      T *q = lds + (v / VPR) * PITCH + (v % VPR) * VEC;
      if constexpr ((PITCH * sizeof(T)) % 16 == 0) {
        *reinterpret_cast<uint4 *>(q) = reg[i];
      } else {
        static_assert((PITCH * sizeof(T)) % 8 == 0, "LDS pitch must keep 8-byte alignment");
        reinterpret_cast<uint2 *>(q)[0] = make_uint2(reg[i].x, reg[i].y);
        reinterpret_cast<uint2 *>(q)[1] = make_uint2(reg[i].z, reg[i].w);
      }
    }
  }
};

// MFMA operand fragments out of LDS.  `o` = output index handled by this lane's fragment block.
template <bool KC> __device__ __forceinline__ bf16x8_t frag_bf16(const bf16 *s, int o, int ks, int lane) {
  using M = Mma<bf16>;
  if constexpr (KC) {
    return *reinterpret_cast<const bf16x8_t *>(s + (o + (lane & 31)) * M::PKC + ks * 16 + 8 * (lane >> 5));
  } else {
    union { bf16x8_t v; uint16_t e[8]; } u;
    const bf16 *p = s + (ks * 16 + 8 * (lane >> 5)) * M::PKS + o + (lane & 31);
#pragma unroll
    for (int j = 0; j < 8; ++j) u.e[j] = p[j * M::PKS].bits;
    return u.v;
  }
}
template <bool KC> __device__ __forceinline__ float frag_f32(const float *s, int o, int ks, int lane) {
  using M = Mma<float>;
  if constexpr (KC) return s[(o + (lane & 31)) * M::PKC + ks * 2 + (lane >> 5)];
  else return s[(ks * 2 + (lane >> 5)) * M::PKS + o + (lane & 31)];
}

template <typename T, bool AKC, bool BKC>
__device__ __forceinline__ void mma_tile(f32x16 (&acc)[2][2], const T *As, const T *Bs, int wm, int wn, int lane) {
  using M = Mma<T>;
#pragma unroll
  for (int ks = 0; ks < M::BK / M::KSTEP; ++ks) {
    if constexpr (sizeof(T) == 2) {
      bf16x8_t a[2], b[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) a[i] = frag_bf16<AKC>(reinterpret_cast<const bf16 *>(As), wm + i * 32, ks, lane);
#pragma unroll
      for (int j = 0; j < 2; ++j) b[j] = frag_bf16<BKC>(reinterpret_cast<const bf16 *>(Bs), wn + j * 32, ks, lane);
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    } else {
      float a[2], b[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) a[i] = frag_f32<AKC>(reinterpret_cast<const float *>(As), wm + i * 32, ks, lane);
#pragma unroll
      for (int j = 0; j < 2; ++j) b[j] = frag_f32<BKC>(reinterpret_cast<const float *>(Bs), wn + j * 32, ks, lane);
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i], b[j], acc[i][j], 0, 0, 0);
    }
  }
}

// Accumulates  sum_{k in [k_begin,k_end)} Aop[a0+i][k] * Bop[b0+j][k]  into the block's accumulators.
// KC operand: matrix [extent x K] row-major (ld); KS operand: matrix [K x extent] row-major (ld).
template <typename T, bool AKC, bool BKC>
__device__ __forceinline__ void gemm_segment(f32x16 (&acc)[2][2], T *As, T *Bs, const T *A, int64_t lda, int a_extent,
                                             int a0, bool a_vec, const T *B, int64_t ldb, int b_extent, int b0,
                                             bool b_vec, int k_begin, int k_end) {
  using M = Mma<T>;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;
  TileMover<T, AKC ? BM : M::BK, AKC ? M::BK : BM, AKC ? M::PKC : M::PKS> ta;
  TileMover<T, BKC ? BN : M::BK, BKC ? M::BK : BN, BKC ? M::PKC : M::PKS> tb;
  auto load = [&](int k0) {
    if constexpr (AKC) ta.load(A, lda, a_extent, k_end, a0, k0, a_vec);
    else ta.load(A, lda, k_end, a_extent, k0, a0, a_vec);
    if constexpr (BKC) tb.load(B, ldb, b_extent, k_end, b0, k0, b_vec);
    else tb.load(B, ldb, k_end, b_extent, k0, b0, b_vec);
  };
  if (k_begin >= k_end) return;
  load(k_begin);
  for (int k0 = k_begin; k0 < k_end; k0 += M::BK) {
    ta.store(As);
    tb.store(Bs);
    __syncthreads();
    if (k0 + M::BK < k_end) load(k0 + M::BK);
    mma_tile<T, AKC, BKC>(acc, As, Bs, wm, wn, lane);
    __syncthreads();
  }
}

__device__ __forceinline__ void zero_acc(f32x16 (&acc)[2][2]) {
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
}

// Element (row, col) of the block tile held in acc[i][j][v] by this lane (32x32 MFMA output layout:
// lane%32 is the column, the 16 values are rows 8*(v/4) + 4*(lane/32) + v%4).
#define HGNN_FOR_EACH_ACC(body)                                                     \
  {                                                                                 \
    const int lane_ = threadIdx.x & 63, wave_ = threadIdx.x >> 6;                   \
    _Pragma("unroll") for (int i_ = 0; i_ < 2; ++i_) _Pragma("unroll") for (int j_ = 0; j_ < 2; ++j_) \
    _Pragma("unroll") for (int v_ = 0; v_ < 16; ++v_) {                             \
      const int row = (wave_ >> 1) * 64 + i_ * 32 + 8 * (v_ >> 2) + 4 * (lane_ >> 5) + (v_ & 3); \
      const int col = (wave_ & 1) * 64 + j_ * 32 + (lane_ & 31);                    \
      const float val = acc[i_][j_][v_];                                            \
      body                                                                          \
    }                                                                               \
  }

// Blocks are spread round-robin over the 8 XCDs by the hardware; give each XCD a contiguous range of tiles
// so that tiles sharing operand rows meet in the same L2.
__device__ __forceinline__ int xcd_tile(int bid, int nblocks) {
  const int per = nblocks >> 3;
  return (bid & 7) * per + (bid >> 3);
}
static inline int round_up8(int n) { return (n + 7) & ~7; }

__device__ __forceinline__ bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

// ------------------------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(kThreads) gemm_fwd_kernel(LayerDev L, TypeTab tt, RelTab rt, PtrTab pt, WtTab wt, SegTab tiles,
                                                            int H, int relu, const T *__restrict__ x, const T *__restrict__ z,
                                                            const T *__restrict__ zlo, const T *__restrict__ wtb,
                                                            T *__restrict__ h, int only_seg,
                                                            float *__restrict__ acc32) {
  __shared__ __attribute__((aligned(16))) T As[lds_elems<T>()];
  __shared__ __attribute__((aligned(16))) T Bs[lds_elems<T>()];
  const int tile = xcd_tile(blockIdx.x, gridDim.x);
  const int T_ = tt.num_types, R = rt.num_rels;
  if (tile >= tiles.tile_off[T_]) return;
  int d = 0;
  while (tile >= tiles.tile_off[d + 1]) ++d;
  const int tiles_n = (H + BN - 1) / BN;
  const int local = tile - tiles.tile_off[d];
  const int m0 = (local / tiles_n) * BM, n0 = (local % tiles_n) * BN;
  const int M = tt.n_dst[d];
  f32x16 acc[2][2];
  zero_acc(acc);
  for (int r = 0; r < R; ++r) {
    if (rt.dst[r] != d || (only_seg >= 0 && only_seg != r)) continue;
    if (L.rel_edge_off[r + 1] == L.rel_edge_off[r]) continue;  // no edge: the aggregate is all zero
    const int F = tt.in_dim[rt.src[r]];
    gemm_segment<T, true, true>(acc, As, Bs, z + (int64_t)rt.z_off4[r] * 4, F, M, m0, true,
                                wtb + (int64_t)wt.rel4[r] * 4, F, H, n0, true, 0, F);
    if (zlo)  // low-order part of the aggregate (bf16 storage): same weights, accumulated on top
      gemm_segment<T, true, true>(acc, As, Bs, zlo + (int64_t)rt.z_off4[r] * 4, F, M, m0, true,
                                  wtb + (int64_t)wt.rel4[r] * 4, F, H, n0, true, 0, F);
  }
  if (pt.w_root[d] && (only_seg < 0 || only_seg == R + d)) {
    const int F = tt.in_dim[d];
    gemm_segment<T, true, true>(acc, As, Bs, x + tt.elem_off[d], F, M, m0, true, wtb + (int64_t)wt.root4[d] * 4, F, H,
                                n0, true, 0, F);
  }
  const T *bias = reinterpret_cast<const T *>(pt.bias[d]);
  const int64_t orow = tt.out_row_off[d];
  if (acc32) {
    HGNN_FOR_EACH_ACC({
      if (m0 + row < M && n0 + col < H) acc32[(orow + m0 + row) * H + n0 + col] += val;
    })
  } else {
    HGNN_FOR_EACH_ACC({
      if (m0 + row < M && n0 + col < H) {
        float o = val + (bias ? to_float(bias[n0 + col]) : 0.f);
        if (relu) o = fmaxf(o, 0.f);
        h[(orow + m0 + row) * H + n0 + col] = from_float<T>(o);
      }
    })
  }
}

hgnn_status launch_gemm_fwd(hipStream_t s, int dtype, const LayerDev &L, const TypeTab &tt, const RelTab &rt,
                            const PtrTab &pt, const WtTab &wt, const SegTab &tiles, int H, int relu,
                            const void *x, const void *z, const void *zlo, const void *wt_buf, void *h, int only_seg,
                            float *acc32) {
  const int n = tiles.tile_off[tt.num_types];
  if (n == 0) return HGNN_OK;
  dim3 grid(round_up8(n));
  if (dtype == HGNN_BF16)
    hipLaunchKernelGGL(gemm_fwd_kernel<bf16>, grid, dim3(kThreads), 0, s, L, tt, rt, pt, wt, tiles, H, relu, (const bf16 *)x,
                       (const bf16 *)z, (const bf16 *)zlo, (const bf16 *)wt_buf, (bf16 *)h, only_seg, acc32);
  else
    hipLaunchKernelGGL(gemm_fwd_kernel<float>, grid, dim3(kThreads), 0, s, L, tt, rt, pt, wt, tiles, H, relu, (const float *)x,
                       (const float *)z, (const float *)nullptr, (const float *)wt_buf, (float *)h, only_seg, acc32);
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

template <typename T>
__global__ void __launch_bounds__(kThreads) gemm_da_kernel(LayerDev L, TypeTab tt, RelTab rt, PtrTab pt, SegTab tiles, int H,
                                                           const T *__restrict__ gp, T *__restrict__ dz) {
  __shared__ __attribute__((aligned(16))) T As[lds_elems<T>()];
  __shared__ __attribute__((aligned(16))) T Bs[lds_elems<T>()];
  const int tile = xcd_tile(blockIdx.x, gridDim.x);
  const int R = rt.num_rels;
  if (tile >= tiles.tile_off[tiles.num_segs]) return;
  const int seg = find_seg(tiles, tile);
  const bool is_rel = seg < R;
  const int d = is_rel ? rt.dst[seg] : seg - R;
  const int F = tt.in_dim[is_rel ? rt.src[seg] : d];
  const T *W = reinterpret_cast<const T *>(is_rel ? pt.w_rel[seg] : pt.w_root[d]);
  const int M = tt.n_dst[d];
  const int tiles_n = (F + BN - 1) / BN;
  const int local = tile - tiles.tile_off[seg];
  const int m0 = (local / tiles_n) * BM, n0 = (local % tiles_n) * BN;
  f32x16 acc[2][2];
  zero_acc(acc);
  const T *A = gp + (int64_t)tt.out_row_off[d] * H;
  const bool vec = (H % Mma<T>::VEC) == 0;
  gemm_segment<T, true, true>(acc, As, Bs, A, H, M, m0, vec && aligned16(A), W, H, F, n0, vec && aligned16(W), 0, H);
  T *out = dz + (int64_t)(is_rel ? rt.z_off4[seg] : rt.zroot_off4[d]) * 4;
  const int rho0 = is_rel ? L.rel_row_off[seg] : 0;
  HGNN_FOR_EACH_ACC({
    if (m0 + row < M && n0 + col < F) {
      float sc = 1.f;
      if (is_rel) {
        const int deg = L.rowptr[rho0 + m0 + row + 1] - L.rowptr[rho0 + m0 + row];
        sc = deg > 0 ? 1.f / (float)deg : 0.f;
      }
      out[(int64_t)(m0 + row) * F + n0 + col] = from_float<T>(val * sc);
    }
  })
}

hgnn_status launch_gemm_da(hipStream_t s, int dtype, const LayerDev &L, const TypeTab &tt, const RelTab &rt,
                           const PtrTab &pt, const SegTab &tiles, int H, const void *gp, void *dz) {
  const int n = tiles.tile_off[tiles.num_segs];
  if (n == 0) return HGNN_OK;
  dim3 grid(round_up8(n));
  if (dtype == HGNN_BF16)
    hipLaunchKernelGGL(gemm_da_kernel<bf16>, grid, dim3(kThreads), 0, s, L, tt, rt, pt, tiles, H, (const bf16 *)gp, (bf16 *)dz);
  else
    hipLaunchKernelGGL(gemm_da_kernel<float>, grid, dim3(kThreads), 0, s, L, tt, rt, pt, tiles, H, (const float *)gp, (float *)dz);
  HGNN_HIP(hipGetLastError());
  return HGNN_OK;
}

// ------------------------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(kThreads) gemm_dw_kernel(LayerDev L, TypeTab tt, RelTab rt, GradPtrTab gt, SegTab tiles,
                                                           int split_rows, int H, const T *__restrict__ x,
                                                           const T *__restrict__ z, const T *__restrict__ gp) {
  __shared__ __attribute__((aligned(16))) T As[lds_elems<T>()];
  __shared__ __attribute__((aligned(16))) T Bs[lds_elems<T>()];
  const int tile = xcd_tile(blockIdx.x, gridDim.x);
  const int R = rt.num_rels;
  if (tile >= tiles.tile_off[tiles.num_segs]) return;
  const int seg = find_seg(tiles, tile);
  const bool is_rel = seg < R;
  const int d = is_rel ? rt.dst[seg] : seg - R;
  const int F = tt.in_dim[is_rel ? rt.src[seg] : d];
  float *dW = is_rel ? gt.dw_rel[seg] : gt.dw_root[d];
  const int M = tt.n_dst[d];
  const int tiles_f = (F + BM - 1) / BM, tiles_h = (H + BN - 1) / BN;
  int local = tile - tiles.tile_off[seg];
  const int th = local % tiles_h;
  local /= tiles_h;
  const int tf = local % tiles_f;
  const int sp = local / tiles_f;
  const int f0 = tf * BM, h0 = th * BN;
  const int k_begin = sp * split_rows, k_end = min(M, k_begin + split_rows);
  f32x16 acc[2][2];
  zero_acc(acc);
  const T *A = is_rel ? z + (int64_t)rt.z_off4[seg] * 4 : x + tt.elem_off[d];
  const T *B = gp + (int64_t)tt.out_row_off[d] * H;
  gemm_segment<T, false, false>(acc, As, Bs, A, F, F, f0, true, B, H, H, h0, (H % Mma<T>::VEC) == 0 && aligned16(B),
                                k_begin, k_end);
  HGNN_FOR_EACH_ACC({
    if (f0 + row < F && h0 + col < H) atomicAdd(dW + (int64_t)(f0 + row) * H + h0 + col, val);
  })
}

hgnn_status launch_gemm_dw(hipStream_t s, int dtype, const LayerDev &L, const TypeTab &tt, const RelTab &rt,
                           const GradPtrTab &gt, const SegTab &tiles, int split_rows, int H, const void *x,
                           const void *z, const void *gp) {
  const int n = tiles.tile_off[tiles.num_segs];
  if (n == 0) return HGNN_OK;
  dim3 grid(round_up8(n));
  if (dtype == HGNN_BF16)
    hipLaunchKernelGGL(gemm_dw_kernel<bf16>, grid, dim3(kThreads), 0, s, L, tt, rt, gt, tiles, split_rows, H, (const bf16 *)x,
                       (const bf16 *)z, (const bf16 *)gp);
  else
    hipLaunchKernelGGL(gemm_dw_kernel<float>, grid, dim3(kThreads), 0, s, L, tt, rt, gt, tiles, split_rows, H, (const float *)x,
                       (const float *)z, (const float *)gp);
  HGNN_HIP(hipGetLastError());
  return HGNN_OK;
}

}  // namespace hgnn
