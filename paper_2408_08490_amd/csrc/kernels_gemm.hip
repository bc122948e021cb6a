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
#include "common.h"
#include "device_types.h"

namespace hgnn {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int BM = 128, BN = 128, kThreads = 256;
constexpr int kSegCap = 96;  // K-segments staged in LDS at a time
constexpr int kRelWindow = (kSegCap - 1) / 2;  // relations examined per pass of the forward kernel (two segments each + root)

template <typename T> struct Mma;
template <> struct Mma<bf16> {
  static constexpr int BK = 64, KSTEP = 16, VEC = 8, PKC = BK + 8, PKS = 128 + 16;  // PKS: four k-rows of a transposing read on disjoint banks
};
template <> struct Mma<float> {
  static constexpr int BK = 32, KSTEP = 2, VEC = 4, PKC = BK + 4, PKS = 128 + 4;
};
template <typename T> constexpr int lds_elems() {
  return (BM * Mma<T>::PKC > Mma<T>::BK * Mma<T>::PKS) ? BM * Mma<T>::PKC : Mma<T>::BK * Mma<T>::PKS;
}

// One K-segment of a tile's reduction: sum over k in [kb, ke) of Aop[.][k] * Bop[.][k].
template <typename T> struct Seg {
  const T *A, *B;
  int lda, ldb, kb, ke;
};

// One operand tile on its way global -> registers -> LDS.  The tile is ROWS x COLS in the operand's own
// row-major orientation (COLS contiguous).
//  * FAST: per-thread byte offsets are computed once per segment (`setup`); a full K-step is NV 16-byte
//    loads from a wave-uniform base plus those offsets and nothing else.  Pieces whose OUTPUT index is out of
//    range read a clamped address and are stored as they are: they only feed output rows / columns that the
//    epilogue never writes.  Only the last, partial K-step of a segment masks (and zero-fills) pieces.
//  * generic: element-wise, zero-filled loads.
template <typename T, int ROWS, int COLS, int PITCH, bool KC>
struct TileMover {
  static constexpr int VEC = 16 / sizeof(T), VPR = COLS / VEC, NV = ROWS * VPR / kThreads;
  static_assert(ROWS * VPR % kThreads == 0, "tile must split evenly over the block");
  typedef const u32x4 __attribute__((address_space(1))) *gvec_t;
  typedef const unsigned short __attribute__((address_space(1))) *g16_t;
  typedef const unsigned int __attribute__((address_space(1))) *g32_t;
  typedef const char __attribute__((address_space(1))) *gbyte_t;
  u32x4 reg[NV];
  unsigned voff[NV];    // byte offset of this thread's pieces from the K-step's base (FAST)
  unsigned okmask = ~0u;  // pieces to keep; the others are stored as zero

  // `o0` = first output index of the tile, `extent` = number of valid output indices, ld in elements.
  __device__ __forceinline__ void setup(int ld, int extent, int o0) {
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int v = threadIdx.x + i * kThreads;
      const int r = v / VPR, c = (v % VPR) * VEC;
      if constexpr (KC) {  // rows = output index, cols = k
        const int o = o0 + r < extent ? o0 + r : 0;
        voff[i] = (unsigned)((o * ld + c) * (int)sizeof(T));
      } else {             // rows = k, cols = output index
        const int o = o0 + c < extent ? o0 + c : 0;
        voff[i] = (unsigned)((r * ld + o) * (int)sizeof(T));
      }
    }
  }
  // base = operand base advanced to the K-step (KC: + k0 elements, KS: + k0 rows); krem = ke - k0 > 0
  __device__ __forceinline__ void load_fast(const T *base, int krem) {
    gbyte_t b = (gbyte_t)base;
    if (krem >= (KC ? COLS : ROWS)) {
#pragma unroll
      for (int i = 0; i < NV; ++i) reg[i] = *(gvec_t)(b + voff[i]);
      okmask = ~0u;
    } else {
      unsigned m = 0;
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        const int v = threadIdx.x + i * kThreads;
        const int kk = KC ? (v % VPR) * VEC : v / VPR;   // first k index of the piece within the step
        const bool ok = kk < krem;                        // K extents are multiples of VEC here
        reg[i] = *(gvec_t)(b + (ok ? voff[i] : 0u));
        m |= ok ? (1u << i) : 0u;
      }
      okmask = m;
    }
  }
  __device__ __forceinline__ void load_slow(const T *base, int64_t ld, int nrows, int ncols, int r0, int c0) {
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int v = threadIdx.x + i * kThreads;
      const int gr = r0 + v / VPR, gc = c0 + (v % VPR) * VEC;
      unsigned int e[VEC];
#pragma unroll
      for (int j = 0; j < VEC; ++j) {
        const bool ok = gr < nrows && gc + j < ncols;
        const T *p = ok ? base + (int64_t)gr * ld + gc + j : base;
        unsigned int x;
        if constexpr (sizeof(T) == 2) x = *(g16_t)p; else x = *(g32_t)p;
        e[j] = ok ? x : 0u;
      }
      if constexpr (sizeof(T) == 2)
        reg[i] = u32x4{e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16), e[6] | (e[7] << 16)};
      else
        reg[i] = u32x4{e[0], e[1], e[2], e[3]};
    }
    okmask = ~0u;
  }
  __device__ __forceinline__ void store(T *lds) {
    if (okmask != ~0u) {
#pragma unroll
      for (int i = 0; i < NV; ++i)
        if (!((okmask >> i) & 1u)) reg[i] = u32x4{0u, 0u, 0u, 0u};
    }
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int v = threadIdx.x + i * kThreads;
      T *q = lds + (v / VPR) * PITCH + (v % VPR) * VEC;
      if constexpr ((PITCH * sizeof(T)) % 16 == 0) {
        *reinterpret_cast<u32x4 *>(q) = reg[i];
      } else {
        static_assert((PITCH * sizeof(T)) % 8 == 0, "LDS pitch must keep 8-byte alignment");
        reinterpret_cast<u32x2 *>(q)[0] = u32x2{reg[i].x, reg[i].y};
        reinterpret_cast<u32x2 *>(q)[1] = u32x2{reg[i].z, reg[i].w};
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
    // The operand lies in LDS with the output index contiguous; the transposing LDS read hands every lane
    // four consecutive k of one output index.  Within a group of 16 lanes, lane p passes the address of four
    // contiguous 16-bit values ("row" p) and lane i receives rows (i / 4) + 4 j, j = 0..3, at position i % 4:
    // with row p = (k0 + p / 4, outputs o16 + 4 (p % 4) ...) lane i ends up with k0..k0+3 of output o16 + i.
    typedef short v4i16 __attribute__((ext_vector_type(4)));
    typedef __attribute__((address_space(3))) v4i16 *lds_v4;
    const int p = lane & 15;
    const bf16 *q = s + (ks * 16 + 8 * (lane >> 5) + (p >> 2)) * M::PKS + o + 16 * ((lane >> 4) & 1) + 4 * (p & 3);
    union { bf16x8_t v; v4i16 h[2]; } u;
    u.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)q);
    u.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(q + 4 * M::PKS));
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

// LDS of one block: two stages of (A tile, B tile) -- reused as the output staging tile by the epilogues --
// and the K-segment table.
template <typename T> struct GemmLds {
  __attribute__((aligned(16))) T a[2][lds_elems<T>()];
  __attribute__((aligned(16))) T b[2][lds_elems<T>()];
  Seg<T> seg[kSegCap];
  float rowscale[BM];
};
constexpr int kOutPitchPad = 8;  // floats: staged rows stay 16-byte aligned, rows r and r + 4 lie 32 banks apart

// Runs the K-steps of sm.seg[0..nseg) (must be visible to the whole block) into `acc`.
// KC operand: matrix [extent x K] row-major (ld); KS operand: matrix [K x extent] row-major (ld).
template <typename T, bool FAST, bool AKC, bool BKC>
__device__ __forceinline__ void gemm_run(f32x16 (&acc)[2][2], GemmLds<T> &sm, int nseg, int a_extent, int a0,
                                         int b_extent, int b0) {
  using M = Mma<T>;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;
  using MoverA = TileMover<T, AKC ? BM : M::BK, AKC ? M::BK : BM, AKC ? M::PKC : M::PKS, AKC>;
  using MoverB = TileMover<T, BKC ? BN : M::BK, BKC ? M::BK : BN, BKC ? M::PKC : M::PKS, BKC>;
  MoverA ta0, ta1;
  MoverB tb0, tb1;
  int total = 0;
  for (int s = 0; s < nseg; ++s) total += (sm.seg[s].ke - sm.seg[s].kb + M::BK - 1) / M::BK;
  int s_ld = 0, k_ld = nseg > 0 ? sm.seg[0].kb : 0;  // cursor of the loader, two K-steps ahead of the multiplier
  int s_set0 = -1, s_set1 = -1;                      // segment each register set's offsets were computed for
  auto issue = [&](MoverA &ta, MoverB &tb, int &s_set) {
    if (s_ld >= nseg) return;
    const Seg<T> g = sm.seg[s_ld];
    if constexpr (FAST) {
      if (s_set != s_ld) {
        ta.setup(g.lda, a_extent, a0);
        tb.setup(g.ldb, b_extent, b0);
        s_set = s_ld;
      }
      ta.load_fast(AKC ? g.A + k_ld : g.A + (int64_t)k_ld * g.lda, g.ke - k_ld);
      tb.load_fast(BKC ? g.B + k_ld : g.B + (int64_t)k_ld * g.ldb, g.ke - k_ld);
    } else {
      if constexpr (AKC) ta.load_slow(g.A, g.lda, a_extent, g.ke, a0, k_ld);
      else ta.load_slow(g.A, g.lda, g.ke, a_extent, k_ld, a0);
      if constexpr (BKC) tb.load_slow(g.B, g.ldb, b_extent, g.ke, b0, k_ld);
      else tb.load_slow(g.B, g.ldb, g.ke, b_extent, k_ld, b0);
    }
    k_ld += M::BK;
    if (k_ld >= g.ke) {
      ++s_ld;
      if (s_ld < nseg) k_ld = sm.seg[s_ld].kb;
    }
  };
  issue(ta0, tb0, s_set0);
  issue(ta1, tb1, s_set1);
  for (int step = 0; step < total; step += 2) {
    ta0.store(sm.a[0]);
    tb0.store(sm.b[0]);
    __syncthreads();
    issue(ta0, tb0, s_set0);
    mma_tile<T, AKC, BKC>(acc, sm.a[0], sm.b[0], wm, wn, lane);
    if (step + 1 < total) {
      ta1.store(sm.a[1]);
      tb1.store(sm.b[1]);
      __syncthreads();
      issue(ta1, tb1, s_set1);
      mma_tile<T, AKC, BKC>(acc, sm.a[1], sm.b[1], wm, wn, lane);
    }
  }
  __syncthreads();  // the segment table and the stages may be rewritten by the caller
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

// Writes the block's 128x128 tile `out[(row0 + r) * ld + col0 + c] = f(acc, r, c)` for r < rows, c < cols.
// When rows of `out` are 16-byte aligned the tile goes through LDS (the K loop's stages are free by then)
// and leaves as whole 16-byte pieces; otherwise element by element.  `f(val, row, col)` returns the value.
// The staged tile is fp32 whatever T is: 32-bit LDS writes with a pitch that puts the two half-waves
// (rows r and r + 4 of one store) on disjoint banks; two lanes writing the halves of one dword would be
// serialised.  Conversion to T happens on the way out.
template <typename T, typename F>
__device__ __forceinline__ void write_tile(f32x16 (&acc)[2][2], GemmLds<T> &sm, T *out, int64_t ld, int rows, int cols, F f) {
  constexpr int V = 16 / sizeof(T), P = BN + kOutPitchPad;
  static_assert(sizeof(sm.a) + sizeof(sm.b) >= sizeof(float) * P * BM, "fp32 output tile must fit the stages");
  const bool vec = (ld % V) == 0 && (reinterpret_cast<uintptr_t>(out) & 15) == 0;
  if (vec) {
    float *stage = reinterpret_cast<float *>(&sm.a[0][0]);
    HGNN_FOR_EACH_ACC({ stage[row * P + col] = f(val, row, col); })
    __syncthreads();
    constexpr int VPR = BN / V;
#pragma unroll
    for (int i = 0; i < BM * VPR / kThreads; ++i) {
      const int v = threadIdx.x + i * kThreads;
      const int r = v / VPR, c = (v % VPR) * V;
      if (r < rows && c < cols) {
        const float *sp = stage + r * P + c;
        u32x4 piece;
        if constexpr (sizeof(T) == 4) {
          piece = *reinterpret_cast<const u32x4 *>(sp);
        } else {
          const f32x4 lo = *reinterpret_cast<const f32x4 *>(sp), hi = *reinterpret_cast<const f32x4 *>(sp + 4);
          piece = u32x4{pack2(lo.x, lo.y), pack2(lo.z, lo.w), pack2(hi.x, hi.y), pack2(hi.z, hi.w)};
        }
        T *dst = out + (int64_t)r * ld + c;
        if (c + V <= cols) {
          *reinterpret_cast<u32x4 *>(dst) = piece;
        } else {  // last, partial piece of a row: element by element out of the registers
#pragma unroll
          for (int j = 0; j < V; ++j) {
            if (c + j < cols) {
              if constexpr (sizeof(T) == 4) {
                reinterpret_cast<unsigned *>(dst)[j] = piece[j];
              } else {
                const unsigned w = piece[j >> 1];
                reinterpret_cast<unsigned short *>(dst)[j] = (unsigned short)((j & 1) ? (w >> 16) : (w & 0xffffu));
              }
            }
          }
        }
      }
    }
  } else {
    HGNN_FOR_EACH_ACC({
      if (row < rows && col < cols) out[(int64_t)row * ld + col] = from_float<T>(f(val, row, col));
    })
  }
}

// Blocks are spread round-robin over the 8 XCDs by the hardware; give each XCD a contiguous range of tiles
// so that tiles sharing operand rows meet in the same L2.
__device__ __forceinline__ int xcd_tile(int bid, int nblocks) {
  const int per = nblocks >> 3;
  return (bid & 7) * per + (bid >> 3);
}
static inline int round_up8(int n) { return (n + 7) & ~7; }

template <typename T>
__device__ __forceinline__ void put_seg(Seg<T> &g, const T *A, int lda, const T *B, int ldb, int kb, int ke) {
  g.A = A; g.B = B; g.lda = lda; g.ldb = ldb; g.kb = kb; g.ke = ke;
}

// ------------------------------------------------------------------------------------------
// Forward.  `live` has bit r set when relation r has at least one edge in this layer.
struct LiveMask {
  uint32_t w[kMaxR / 32];
};

template <typename T, bool FAST>
__global__ void __launch_bounds__(kThreads, 2) gemm_fwd_kernel(TypeTab tt, RelTab rt, PtrTab pt, WtTab wt, SegTab tiles, LiveMask live,
                                                            int H, int relu, const T *__restrict__ x, const T *__restrict__ z,
                                                            const T *__restrict__ zlo, const T *__restrict__ wtb,
                                                            T *__restrict__ h, int only_seg,
                                                            float *__restrict__ acc32) {
  __shared__ GemmLds<T> sm;
  __shared__ int s_nseg;
  const int T_ = tt.num_types, R = rt.num_rels;
  const int tile = xcd_tile(blockIdx.x, gridDim.x);
  if (tile >= tiles.tile_off[T_]) return;
  int d = 0;
  while (tile >= tiles.tile_off[d + 1]) ++d;
  const int tiles_n = (H + BN - 1) / BN;
  const int local = tile - tiles.tile_off[d];
  const int m0 = (local / tiles_n) * BM, n0 = (local % tiles_n) * BN;
  const int M = tt.n_dst[d];
  f32x16 acc[2][2];
  zero_acc(acc);
  // K-segments of this destination type: every relation ending in d (aggregate, and for bf16 storage its
  // low-order remainder against the same weights), then the root term.  The first wavefront looks at a
  // window of relations at once, one per lane, and packs the ones that take part with a ballot.
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
          put_seg(sm.seg[n++], x + tt.elem_off[d], F, wtb + (int64_t)wt.root4[d] * 4, F, 0, F);
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
  float bv[2];
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int c = n0 + ((threadIdx.x >> 6) & 1) * 64 + j * 32 + (threadIdx.x & 31);
    bv[j] = (bias && c < H) ? to_float(bias[c]) : 0.f;
  }
  const int wn0 = ((threadIdx.x >> 6) & 1) * 64;
  write_tile(acc, sm, h + (orow + m0) * H + n0, H, M - m0, H - n0, [&](float v, int, int col) {
    const float o = v + bv[(col - wn0) >> 5];
    return relu ? fmaxf(o, 0.f) : o;
  });
}

hgnn_status launch_gemm_fwd(hipStream_t s, int dtype, const LayerDev &L, const TypeTab &tt, const RelTab &rt,
                            const PtrTab &pt, const WtTab &wt, const SegTab &tiles, const uint32_t *live_mask, int H,
                            int relu, const void *x, const void *z, const void *zlo, const void *wt_buf, void *h,
                            int only_seg, float *acc32) {
  const int n = tiles.tile_off[tt.num_types];
  if (n == 0) return HGNN_OK;
  (void)L;
  LiveMask live;
  for (int i = 0; i < kMaxR / 32; ++i) live.w[i] = live_mask[i];
  dim3 grid(round_up8(n));
  // operands of the forward are the library's own aligned buffers (aggregates, transposed weights) and
  // x_merged, whose row widths are multiples of 16 bytes: always the FAST form
  if (dtype == HGNN_BF16)
    HGNN_LAUNCH((gemm_fwd_kernel<bf16, true>), grid, dim3(kThreads), 0, s, tt, rt, pt, wt, tiles, live, H, relu,
                       (const bf16 *)x, (const bf16 *)z, (const bf16 *)zlo, (const bf16 *)wt_buf, (bf16 *)h, only_seg, acc32);
  else
    HGNN_LAUNCH((gemm_fwd_kernel<float, true>), grid, dim3(kThreads), 0, s, tt, rt, pt, wt, tiles, live, H, relu,
                       (const float *)x, (const float *)z, (const float *)nullptr, (const float *)wt_buf, (float *)h,
                       only_seg, acc32);
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
template <typename T, bool FAST>
__global__ void __launch_bounds__(kThreads, 2) gemm_da_kernel(LayerDev L, TypeTab tt, RelTab rt, PtrTab pt, SegTab tiles, int ldg,
                                                           const T *__restrict__ gp, T *__restrict__ dz) {
  __shared__ GemmLds<T> sm;
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

hgnn_status launch_gemm_da(hipStream_t s, int dtype, const LayerDev &L, const TypeTab &tt, const RelTab &rt,
                           const PtrTab &pt, const SegTab &tiles, int ldg, bool fast, const void *gp, void *dz) {
  const int n = tiles.tile_off[tiles.num_segs];
  if (n == 0) return HGNN_OK;
  dim3 grid(round_up8(n)), blk(kThreads);
  if (dtype == HGNN_BF16) {
    if (fast) HGNN_LAUNCH((gemm_da_kernel<bf16, true>), grid, blk, 0, s, L, tt, rt, pt, tiles, ldg, (const bf16 *)gp, (bf16 *)dz);
    else HGNN_LAUNCH((gemm_da_kernel<bf16, false>), grid, blk, 0, s, L, tt, rt, pt, tiles, ldg, (const bf16 *)gp, (bf16 *)dz);
  } else {
    if (fast) HGNN_LAUNCH((gemm_da_kernel<float, true>), grid, blk, 0, s, L, tt, rt, pt, tiles, ldg, (const float *)gp, (float *)dz);
    else HGNN_LAUNCH((gemm_da_kernel<float, false>), grid, blk, 0, s, L, tt, rt, pt, tiles, ldg, (const float *)gp, (float *)dz);
  }
  HGNN_HIP(hipGetLastError());
  return HGNN_OK;
}

// ------------------------------------------------------------------------------------------
// dW_s += A_s^T G' over the destination-row slice [k_begin, k_end) of this block.
template <typename T, bool FAST>
__global__ void __launch_bounds__(kThreads, 2) gemm_dw_kernel(TypeTab tt, RelTab rt, GradPtrTab gt, DwTab tiles, int split_rows, int H,
                                                           int ldg, const T *__restrict__ x, const T *__restrict__ z,
                                                           const T *__restrict__ gp) {
  __shared__ GemmLds<T> sm;
  const int tile = xcd_tile(blockIdx.x, gridDim.x);
  const int R = rt.num_rels, T_ = tt.num_types;
  if (tile >= tiles.tile_off[T_]) return;
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
  f32x16 acc[2][2];
  zero_acc(acc);
  if (threadIdx.x == 0)
    put_seg(sm.seg[0], is_rel ? z + (int64_t)rt.z_off4[seg] * 4 : x + tt.elem_off[d], F,
            gp + (int64_t)tt.out_row_off[d] * ldg, ldg, k_begin, k_end);
  __syncthreads();
  gemm_run<T, FAST, false, false>(acc, sm, 1, F, f0, ldg, h0);
  HGNN_FOR_EACH_ACC({
    if (f0 + row < F && h0 + col < H) atomicAdd(dW + (int64_t)(f0 + row) * H + h0 + col, val);
  })
}

hgnn_status launch_gemm_dw(hipStream_t s, int dtype, const LayerDev &L, const TypeTab &tt, const RelTab &rt,
                           const GradPtrTab &gt, const DwTab &tiles, int split_rows, int H, int ldg, bool fast,
                           const void *x, const void *z, const void *gp) {
  const int n = tiles.tile_off[tt.num_types];
  if (n == 0) return HGNN_OK;
  (void)L;
  dim3 grid(round_up8(n)), blk(kThreads);
  if (dtype == HGNN_BF16) {
    if (fast) HGNN_LAUNCH((gemm_dw_kernel<bf16, true>), grid, blk, 0, s, tt, rt, gt, tiles, split_rows, H, ldg, (const bf16 *)x, (const bf16 *)z, (const bf16 *)gp);
    else HGNN_LAUNCH((gemm_dw_kernel<bf16, false>), grid, blk, 0, s, tt, rt, gt, tiles, split_rows, H, ldg, (const bf16 *)x, (const bf16 *)z, (const bf16 *)gp);
  } else {
    if (fast) HGNN_LAUNCH((gemm_dw_kernel<float, true>), grid, blk, 0, s, tt, rt, gt, tiles, split_rows, H, ldg, (const float *)x, (const float *)z, (const float *)gp);
    else HGNN_LAUNCH((gemm_dw_kernel<float, false>), grid, blk, 0, s, tt, rt, gt, tiles, split_rows, H, ldg, (const float *)x, (const float *)z, (const float *)gp);
  }
  HGNN_HIP(hipGetLastError());
  return HGNN_OK;
}

}  // namespace hgnn
