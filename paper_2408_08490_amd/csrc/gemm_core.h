// MFMA GEMM core shared by the layer GEMMs: tile movers (global -> registers -> LDS), MFMA fragment reads,
// the software-pipelined K loop over a segment table, and the LDS-staged epilogue.
#pragma once
#include "common.h"
#include "device_types.h"

namespace hgnn {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// A block is 2x2 wavefronts; every wavefront owns MI x NI accumulators of 32x32, so the block tile is
// (64 MI) x (64 NI).  BM x BN is the default tile (MI = NI = 2); launches that would not fill the chip with
// those use 64x64 tiles (MI = NI = 1).
constexpr int BM = 128, BN = 128, kThreads = 256;
constexpr int kSegCap = 96;  // K-segments staged in LDS at a time
constexpr int kRelWindow = (kSegCap - 1) / 2;  // relations examined per pass of the forward kernel (up to two segments each, and the root)

template <typename T> struct Mma;
template <> struct Mma<bf16> {
  static constexpr int BK = 64, KSTEP = 16, VEC = 8, PKC = BK + 8, KSPAD = 16;  // KS pitch = extent + KSPAD: four k-rows of a transposing read on disjoint banks
};
template <> struct Mma<float> {
  static constexpr int BK = 32, KSTEP = 2, VEC = 4, PKC = BK + 4, KSPAD = 4;
};
// LDS pitch (elements) of an operand tile kept with its OUTPUT index contiguous ("KS": rows = k).  A 128-wide bf16
// tile is kept unpadded (a row = 64 dwords = the LDS's 64 banks) with the four 64-byte column blocks of a row
// XOR-swizzled by the row's low two bits: the transposing fragment read touches four consecutive k-rows at one
// column block per 32 lanes, which then sit on four different quarters of the banks (with a 16-element pad they
// overlapped in pairs: a quarter of the weight-gradient kernel's LDS cycles were bank conflicts).  Other shapes
// keep the pad.
template <typename T> constexpr bool ks_swizzled(int extent) { return sizeof(T) == 2 && extent == 128; }
template <typename T> constexpr int ks_pitch(int extent) { return ks_swizzled<T>(extent) ? extent : extent + Mma<T>::KSPAD; }
__device__ __forceinline__ int ks_swizzle_col(int col, int row) { return (((col >> 5) ^ (row & 3)) << 5) | (col & 31); }
// elements of one LDS stage of an operand tile with `extent` output indices, in either orientation
template <typename T> constexpr int lds_elems(int extent) {
  return (extent * Mma<T>::PKC > Mma<T>::BK * ks_pitch<T>(extent)) ? extent * Mma<T>::PKC : Mma<T>::BK * ks_pitch<T>(extent);
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
      int col = (v % VPR) * VEC;
      if constexpr (!KC && ks_swizzled<T>(COLS)) col = ks_swizzle_col(col, v / VPR);
      T *q = lds + (v / VPR) * PITCH + col;
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
template <bool KC, int PITCH> __device__ __forceinline__ bf16x8_t frag_bf16(const bf16 *s, int o, int ks, int lane) {
  if constexpr (KC) {
    return *reinterpret_cast<const bf16x8_t *>(s + (o + (lane & 31)) * PITCH + ks * 16 + 8 * (lane >> 5));
  } else {
    // The operand lies in LDS with the output index contiguous; the transposing LDS read hands every lane
    // four consecutive k of one output index.  Within a group of 16 lanes, lane p passes the address of four
    // contiguous 16-bit values ("row" p) and lane i receives rows (i / 4) + 4 j, j = 0..3, at position i % 4:
    // with row p = (k0 + p / 4, outputs o16 + 4 (p % 4) ...) lane i ends up with k0..k0+3 of output o16 + i.
    typedef short v4i16 __attribute__((ext_vector_type(4)));
    typedef __attribute__((address_space(3))) v4i16 *lds_v4;
    const int p = lane & 15;
    const int row = ks * 16 + 8 * (lane >> 5) + (p >> 2);
    int col = o + 16 * ((lane >> 4) & 1) + 4 * (p & 3);
    if constexpr (PITCH == 128) col = ks_swizzle_col(col, row);  // the unpadded, swizzled 128-wide tile (row + 4 has the same low bits)
    const bf16 *q = s + row * PITCH + col;
    union { bf16x8_t v; v4i16 h[2]; } u;
    u.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)q);
    u.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(q + 4 * PITCH));
    return u.v;
  }
}
template <bool KC, int PITCH> __device__ __forceinline__ float frag_f32(const float *s, int o, int ks, int lane) {
  if constexpr (KC) return s[(o + (lane & 31)) * PITCH + ks * 2 + (lane >> 5)];
  else return s[(ks * 2 + (lane >> 5)) * PITCH + o + (lane & 31)];
}

template <typename T, bool AKC, bool BKC, int MI, int NI>
__device__ __forceinline__ void mma_tile(f32x16 (&acc)[MI][NI], const T *As, const T *Bs, int wm, int wn, int lane) {
  using M = Mma<T>;
  constexpr int PA = AKC ? M::PKC : ks_pitch<T>(64 * MI), PB = BKC ? M::PKC : ks_pitch<T>(64 * NI);
#pragma unroll
  for (int ks = 0; ks < M::BK / M::KSTEP; ++ks) {
    if constexpr (sizeof(T) == 2) {
      bf16x8_t a[MI], b[NI];
#pragma unroll
      for (int i = 0; i < MI; ++i) a[i] = frag_bf16<AKC, PA>(reinterpret_cast<const bf16 *>(As), wm + i * 32, ks, lane);
#pragma unroll
      for (int j = 0; j < NI; ++j) b[j] = frag_bf16<BKC, PB>(reinterpret_cast<const bf16 *>(Bs), wn + j * 32, ks, lane);
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    } else {
      float a[MI], b[NI];
#pragma unroll
      for (int i = 0; i < MI; ++i) a[i] = frag_f32<AKC, PA>(reinterpret_cast<const float *>(As), wm + i * 32, ks, lane);
#pragma unroll
      for (int j = 0; j < NI; ++j) b[j] = frag_f32<BKC, PB>(reinterpret_cast<const float *>(Bs), wn + j * 32, ks, lane);
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i], b[j], acc[i][j], 0, 0, 0);
    }
  }
}

// LDS of one block: two stages of (A tile, B tile) -- reused as the output staging tile by the epilogues --
// and the K-segment table.
template <typename T, int MI = 2, int NI = 2> struct GemmLds {
  __attribute__((aligned(16))) T a[2][lds_elems<T>(64 * MI)];
  __attribute__((aligned(16))) T b[2][lds_elems<T>(64 * NI)];
  Seg<T> seg[kSegCap];
  float rowscale[64 * MI];
};
constexpr int kOutPitchPad = 8;  // floats: staged rows stay 16-byte aligned, rows r and r + 4 lie 32 banks apart

// A pointer that is the same in every lane, moved to scalar registers.
template <typename P> __device__ __forceinline__ const P *uniform_ptr(const P *p) {
  const uint64_t v = reinterpret_cast<uint64_t>(p);
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
  return reinterpret_cast<const P *>(((uint64_t)hi << 32) | lo);
}

// Runs the K-steps of sm.seg[0..nseg) (must be visible to the whole block) into `acc`.
// KC operand: matrix [extent x K] row-major (ld); KS operand: matrix [K x extent] row-major (ld).
template <typename T, bool FAST, bool AKC, bool BKC, int MI, int NI>
__device__ __forceinline__ void gemm_run(f32x16 (&acc)[MI][NI], GemmLds<T, MI, NI> &sm, int nseg, int a_extent, int a0,
                                         int b_extent, int b0) {
  using M = Mma<T>;
  constexpr int TM = 64 * MI, TN = 64 * NI;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = (wave >> 1) * 32 * MI, wn = (wave & 1) * 32 * NI;
  using MoverA = TileMover<T, AKC ? TM : M::BK, AKC ? M::BK : TM, AKC ? M::PKC : ks_pitch<T>(TM), AKC>;
  using MoverB = TileMover<T, BKC ? TN : M::BK, BKC ? M::BK : TN, BKC ? M::PKC : ks_pitch<T>(TN), BKC>;
  MoverA ta0, ta1;
  MoverB tb0, tb1;
  int total = 0;
  for (int s = 0; s < nseg; ++s) total += (sm.seg[s].ke - sm.seg[s].kb + M::BK - 1) / M::BK;
  int s_ld = 0, k_ld = nseg > 0 ? sm.seg[0].kb : 0;  // cursor of the loader, two K-steps ahead of the multiplier
  int s_set0 = -1, s_set1 = -1;                      // segment each register set's offsets were computed for
  // The loader's segment is kept in scalar registers and read from LDS only when the loader moves on to the next
  // one: read per K-step, the LDS round trip sits in the step's chain of dependent operations.
  Seg<T> g;
  int s_cached = -1;
  auto issue = [&](MoverA &ta, MoverB &tb, int &s_set) {
    if (s_ld >= nseg) return;
    if (s_cached != s_ld) {
      const Seg<T> v = sm.seg[s_ld];
      g.A = uniform_ptr(v.A);
      g.B = uniform_ptr(v.B);
      g.lda = __builtin_amdgcn_readfirstlane(v.lda);
      g.ldb = __builtin_amdgcn_readfirstlane(v.ldb);
      g.kb = __builtin_amdgcn_readfirstlane(v.kb);
      g.ke = __builtin_amdgcn_readfirstlane(v.ke);
      s_cached = s_ld;
    }
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

template <int MI, int NI> __device__ __forceinline__ void zero_acc(f32x16 (&acc)[MI][NI]) {
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NI; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
}

// Element (row, col) of the block tile held in acc[i][j][v] by this lane (32x32 MFMA output layout:
// lane%32 is the column, the 16 values are rows 8*(v/4) + 4*(lane/32) + v%4).
#define HGNN_FOR_EACH_ACC(body)                                                     \
  {                                                                                 \
    const int lane_ = threadIdx.x & 63, wave_ = threadIdx.x >> 6;                   \
    constexpr int MI_ = sizeof(acc) / sizeof(acc[0]), NI_ = sizeof(acc[0]) / sizeof(acc[0][0]); \
    _Pragma("unroll") for (int i_ = 0; i_ < MI_; ++i_) _Pragma("unroll") for (int j_ = 0; j_ < NI_; ++j_) \
    _Pragma("unroll") for (int v_ = 0; v_ < 16; ++v_) {                             \
      const int row = (wave_ >> 1) * 32 * MI_ + i_ * 32 + 8 * (v_ >> 2) + 4 * (lane_ >> 5) + (v_ & 3); \
      const int col = (wave_ & 1) * 32 * NI_ + j_ * 32 + (lane_ & 31);              \
      const float val = acc[i_][j_][v_];                                            \
      body                                                                          \
    }                                                                               \
  }

// Writes the block's tile `out[(row0 + r) * ld + col0 + c] = f(acc, r, c)` for r < rows, c < cols.
// When rows of `out` are 16-byte aligned the tile goes through LDS (the K loop's stages are free by then)
// and leaves as whole 16-byte pieces; otherwise element by element.  `f(val, row, col)` returns the value.
// The output type TO may differ from the operands' T (bf16 operands, fp32 result).  The staged tile is fp32 whatever T is: 32-bit LDS writes with a pitch that puts the two half-waves
// (rows r and r + 4 of one store) on disjoint banks; two lanes writing the halves of one dword would be
// serialised.  Conversion to T happens on the way out.
template <typename T, typename TO, typename F, int MI, int NI>
__device__ __forceinline__ void write_tile(f32x16 (&acc)[MI][NI], GemmLds<T, MI, NI> &sm, TO *out, int64_t ld, int rows, int cols, F f) {
  constexpr int TM = 64 * MI, TN = 64 * NI;
  constexpr int V = 16 / sizeof(TO), P = TN + kOutPitchPad;
  static_assert(sizeof(sm.a) + sizeof(sm.b) >= sizeof(float) * P * TM, "fp32 output tile must fit the stages");
  const bool vec = (ld % V) == 0 && (reinterpret_cast<uintptr_t>(out) & 15) == 0;
  if (vec) {
    float *stage = reinterpret_cast<float *>(&sm.a[0][0]);
    HGNN_FOR_EACH_ACC({ stage[row * P + col] = f(val, row, col); })
    __syncthreads();
    constexpr int VPR = TN / V;
#pragma unroll
    for (int i = 0; i < TM * VPR / kThreads; ++i) {
      const int v = threadIdx.x + i * kThreads;
      const int r = v / VPR, c = (v % VPR) * V;
      if (r < rows && c < cols) {
        const float *sp = stage + r * P + c;
        u32x4 piece;
        if constexpr (sizeof(TO) == 4) {
          piece = *reinterpret_cast<const u32x4 *>(sp);
        } else {
          const f32x4 lo = *reinterpret_cast<const f32x4 *>(sp), hi = *reinterpret_cast<const f32x4 *>(sp + 4);
          piece = u32x4{pack2(lo.x, lo.y), pack2(lo.z, lo.w), pack2(hi.x, hi.y), pack2(hi.z, hi.w)};
        }
        TO *dst = out + (int64_t)r * ld + c;
        if (c + V <= cols) {
          *reinterpret_cast<u32x4 *>(dst) = piece;
        } else {  // last, partial piece of a row: element by element out of the registers
#pragma unroll
          for (int j = 0; j < V; ++j) {
            if (c + j < cols) {
              if constexpr (sizeof(TO) == 4) {
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
      if (row < rows && col < cols) out[(int64_t)row * ld + col] = from_float<TO>(f(val, row, col));
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

// The same idea for tiles of unequal cost: group g holds tiles [tile_off[g], tile_off[g+1]) of cost[g] each;
// every XCD gets a contiguous range of about one eighth of the total cost.  Block b works on tile
// first[b & 7] + (b >> 3) when that lies below first[(b & 7) + 1], else on nothing.
struct XcdMap {
  int32_t first[9];
};
__device__ __forceinline__ int xcd_tile(const XcdMap &m, int bid) {
  const int x = bid & 7, t = m.first[x] + (bid >> 3);
  return t < m.first[x + 1] ? t : -1;
}
// Returns the number of blocks to launch.
static inline int balance_xcd(const int32_t *tile_off, const int64_t *cost, int ngroups, XcdMap &m) {
  int64_t total = 0;
  for (int g = 0; g < ngroups; ++g) total += (int64_t)(tile_off[g + 1] - tile_off[g]) * cost[g];
  const int ntiles = tile_off[ngroups];
  m.first[0] = 0;
  int g = 0, longest = 0;
  int64_t before = 0;  // cost of the tiles before group g
  for (int x = 1; x <= 8; ++x) {
    int t = ntiles;
    if (x < 8) {
      const int64_t target = (total * x + 7) / 8;  // first tile whose preceding cost reaches the target
      while (g < ngroups && before + (int64_t)(tile_off[g + 1] - tile_off[g]) * cost[g] < target) {
        before += (int64_t)(tile_off[g + 1] - tile_off[g]) * cost[g];
        ++g;
      }
      t = g < ngroups ? tile_off[g] + (int)((target - before + cost[g] - 1) / cost[g]) : ntiles;
      if (t < m.first[x - 1]) t = m.first[x - 1];
      if (t > ntiles) t = ntiles;
    }
    m.first[x] = t;
    if (t - m.first[x - 1] > longest) longest = t - m.first[x - 1];
  }
  return longest * 8;
}

template <typename T>
__device__ __forceinline__ void put_seg(Seg<T> &g, const T *A, int lda, const T *B, int ldb, int kb, int ke) {
  g.A = A; g.B = B; g.lda = lda; g.ldb = ldb; g.kb = kb; g.ke = ke;
}

}  // namespace hgnn
