// bf16 MFMA GEMM core with operand tiles that go from global memory straight into LDS (gfx950's 16-byte
// per-lane LDS-DMA loads): no register staging, S LDS stages, the loads of the next S - 1 K-steps in flight
// while the current one is multiplied.  A block of 8 wavefronts computes a TM x 128 tile (TM = 256: every
// wavefront owns 64x64 of it as 2x2 MFMA 32x32 accumulators; TM = 128: 32x64).
//
// LDS layout of a K-contiguous operand tile (rows = output index, 64 bf16 = 128 bytes = eight 16-byte pieces per
// row, rows back to back): piece p of row r sits in slot p ^ swz(r) of its row, swz(r) = (r & 7) ^ ((r >> 3) & 1).
// A wave-wide LDS-DMA load writes lane l's 16 bytes at base + 16 l, i.e. 8 whole rows per instruction, so lane l
// of the instruction that fills rows r0..r0+7 fetches piece (l & 7) ^ swz(r0 + l / 8) of row r0 + l / 8.  An MFMA
// fragment read (lane l: row o + l % 32, piece 2 ks + l / 32) then touches, in any 16 consecutive lanes, 16
// different 16-byte bank groups of the 64-bank LDS (and 8 different ones of a 32-bank half in any 8 lanes).
#pragma once
#include "gemm_core.h"

namespace hgnn {
namespace dma {

constexpr int kThreads = 512, kWaves = 8;
constexpr int BK = 64, TN = 128;
constexpr int kRowBytes = BK * 2;  // one tile row of one K-step

__device__ __forceinline__ int swz(int r) { return (r & 7) ^ ((r >> 3) & 1); }

// Source of pieces that must read as zero (beyond the end of a K-segment).
static __device__ __attribute__((used)) const unsigned int g_zero_piece[4] = {0u, 0u, 0u, 0u};

// One wave-wide LDS-DMA load: lane l's 16 bytes at `gaddr` land at LDS byte address lds_base + 16 l (lds_base is
// wave-uniform).  Written as assembly so that the compiler does not pair every later LDS read with a wait for ALL
// outstanding loads; completion is tracked by hand with wait_loads<N>() (the loads retire in order).
__device__ __forceinline__ void load16_to_lds(const void *gaddr, unsigned lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_base), "v"(gaddr) : "memory", "m0");
}
// Waits until at most N of this wavefront's vector-memory loads are outstanding.
template <int N> __device__ __forceinline__ void wait_loads() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }
// Workgroup barrier without the memory fence of __syncthreads (which would wait for every outstanding load).
// LDS accesses of a wavefront are complete before it issues anything after its own lgkmcnt wait, which the
// compiler places before the values are used.
__device__ __forceinline__ void barrier_only() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }
__device__ __forceinline__ unsigned lds_address(const void *p) {
  return (unsigned)(unsigned long)(__attribute__((address_space(3))) const char *)p;
}

constexpr int kSegTable = 128;   // K-segments of a whole launch kept in LDS
constexpr int kStepList = 288;   // K-steps of one batch of tiles
constexpr int kTileList = 32;    // tiles of one batch

// One K-step of the block's work, ready to be loaded: operand pointers already advanced to the step.
struct alignas(16) StepEnt {
  const bf16 *A, *B;
  uint16_t lda, ldb;  // leading dimensions in elements
  uint16_t krem;      // k extent of the step: 64, or less at the end of a segment (the rest reads as zero)
  uint16_t tile;      // index into the tile list
  unsigned pad[2];
};
// What the pipeline needs to know about one output tile.
struct alignas(16) TileEnt {
  int a0, a_extent;   // first row of the tile in the A operand, valid rows of that operand
  int b0, b_extent;   // the same for B (= output columns)
  int id;             // kernel-specific (destination type / segment)
  int last_step;      // index of the tile's last K-step in the step list, -1 when it has none
  int pad[2];
};
struct TilePlan {     // filled by a kernel's `decode`: the tile and where its K-segments sit in the segment table
  TileEnt t;
  int seg_first, nseg;
};

template <int TM, int S> struct Lds {  // S = LDS stages: the loads run S - 1 K-steps ahead
  __attribute__((aligned(1024))) unsigned char a[S][TM * kRowBytes];
  __attribute__((aligned(1024))) unsigned char b[S][TN * kRowBytes];
  Seg<bf16> seg[kSegTable];
  StepEnt step[kStepList];
  TileEnt tile[kTileList];
  int n_steps, n_tiles;
};

// Loads of one K-step: TM / 64 + TN / 64 wave-wide LDS-DMA instructions per wavefront.  Instruction i of wavefront w
// fills tile rows 8 (8 i + w) .. + 7 of an operand; lane l fetches the piece (l & 7) ^ swz(row) of row 8 (8 i + w) + l / 8.
// Rows beyond an operand's extent read a clamped row (they only feed outputs that are never written); pieces beyond
// the step's k extent read zeros.
template <int TM, int S> __device__ __forceinline__ void issue_step(const Lds<TM, S> &sm, int j, unsigned a_stage, unsigned b_stage) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const u32x4 e0 = *reinterpret_cast<const u32x4 *>(&sm.step[j]);
  const u32x2 e1 = *(reinterpret_cast<const u32x2 *>(&sm.step[j]) + 2);
  // (the intrinsic returns a signed int: every word goes through uint32_t before it is widened or shifted, or the
  // low word of a pointer with bit 31 set would sign-extend into the high word)
  const uint32_t w_tile = (uint32_t)__builtin_amdgcn_readfirstlane((int)e1.y);
  const unsigned tl = w_tile >> 16;
  const u32x4 t0 = *reinterpret_cast<const u32x4 *>(&sm.tile[tl]);
  const uint64_t pa = ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)e0.y) << 32) | (uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)e0.x);
  const uint64_t pb = ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)e0.w) << 32) | (uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)e0.z);
  const uint32_t ld2 = (uint32_t)__builtin_amdgcn_readfirstlane((int)e1.x);
  const int lda = (int)(ld2 & 0xffffu), ldb = (int)(ld2 >> 16);
  const int krem = (int)(w_tile & 0xffffu);
  const int a0 = __builtin_amdgcn_readfirstlane((int)t0.x), a_last = __builtin_amdgcn_readfirstlane((int)t0.y) - 1;
  const int b0 = __builtin_amdgcn_readfirstlane((int)t0.z), b_last = __builtin_amdgcn_readfirstlane((int)t0.w) - 1;
  const int rsub = lane >> 3;
  const int kpiece = ((lane & 7) ^ rsub ^ (wave & 1)) * 8;  // (lane & 7) ^ swz(row): row & 7 = rsub, (row >> 3) & 1 = wave & 1
  const bool live = kpiece < krem;  // k extents are multiples of 8: a piece is inside or outside as a whole
  const char *za = reinterpret_cast<const char *>(pa), *zb = reinterpret_cast<const char *>(pb);
#pragma unroll
  for (int i = 0; i < TM / 64; ++i) {
    const int r = (8 * i + wave) * 8 + rsub;
    const unsigned off = (unsigned)(min(a0 + r, a_last) * lda + kpiece) * 2u;
    const void *src = live ? static_cast<const void *>(za + off) : static_cast<const void *>(g_zero_piece);
    load16_to_lds(src, __builtin_amdgcn_readfirstlane(a_stage + (unsigned)(8 * i + wave) * 1024u));
  }
#pragma unroll
  for (int i = 0; i < TN / 64; ++i) {
    const int r = (8 * i + wave) * 8 + rsub;
    const unsigned off = (unsigned)(min(b0 + r, b_last) * ldb + kpiece) * 2u;
    const void *src = live ? static_cast<const void *>(zb + off) : static_cast<const void *>(g_zero_piece);
    load16_to_lds(src, __builtin_amdgcn_readfirstlane(b_stage + (unsigned)(8 * i + wave) * 1024u));
  }
}

// Persistent pipeline over the block's tiles tile0, tile0 + stride, ... < tile_end.  `decode(tile, plan)` describes a
// tile (its K-segments must be in sm.seg, visible to the block); `finish(acc, tile entry)` writes it out straight
// from the accumulators (no LDS, no barrier: the loads of the next tile, already in flight, keep landing meanwhile).
// The tiles are taken in batches; for a batch, every K-step of every tile is written into a step list first (one
// thread per tile), so that the loop itself does no bookkeeping: it reads a step's entry and issues its loads.  All
// steps of a batch form ONE sequence, the loads run S - 1 steps ahead of the multiplication across tile
// boundaries.  Both operands are K-contiguous.  Wavefronts that share a SIMD (w and w + 4) take the two halves of a
// step in opposite order -- one issues its loads, then multiplies, the other multiplies first -- so that the matrix
// unit is busy while the other wavefront computes addresses.
template <int TM, int S, typename Decode, typename Finish>
__device__ __forceinline__ void run_tiles_kc(Lds<TM, S> &sm, int tile0, int tile_end, int stride, Decode decode, Finish finish) {
  constexpr int MI = TM / 128, NL = TM / 64 + TN / 64;  // loads per wavefront and K-step
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = (wave >> 1) * 32 * MI, wn = (wave & 1) * 64;
  const unsigned a_lds = lds_address(&sm.a[0][0]), b_lds = lds_address(&sm.b[0][0]);
  const int sw = swz(lane & 31);
  int koff[BK / 16];
#pragma unroll
  for (int ks = 0; ks < BK / 16; ++ks) koff[ks] = ((2 * ks + (lane >> 5)) ^ sw) * 16;
  const int arow = (wm + (lane & 31)) * kRowBytes, brow = (wn + (lane & 31)) * kRowBytes;
  const bool loads_first = ((wave >> 2) & 1) == 0;

  for (int batch0 = tile0; batch0 < tile_end;) {
    // ---- the batch's tile and step lists ----
    if (threadIdx.x < kTileList) {
      const int tile = batch0 + (int)threadIdx.x * stride;
      int steps = 0;
      if (tile < tile_end) {
        TilePlan tp;
        decode(tile, tp);
        for (int s = 0; s < tp.nseg; ++s) steps += (sm.seg[tp.seg_first + s].ke - sm.seg[tp.seg_first + s].kb + BK - 1) / BK;
        tp.t.last_step = -1;
        sm.tile[threadIdx.x] = tp.t;
      }
      // inclusive prefix sum over the (at most 32) tiles of the batch, inside the first wavefront
      int incl = steps;
#pragma unroll
      for (int o = 1; o < kTileList; o <<= 1) {
        const int up = __shfl_up(incl, o);
        if ((int)threadIdx.x >= o) incl += up;
      }
      // the batch ends before the first tile that would overflow the step list (a tile alone always fits: the
      // launcher checks) and at the end of the block's tiles
      const bool fits = tile < tile_end && incl <= kStepList;
      const unsigned long long m = __ballot(fits);
      const int ntile = __popcll(m & 0xffffffffull);  // `fits` is monotone over the lanes: a prefix of them
      if (threadIdx.x == 0) sm.n_tiles = ntile;
      if ((int)threadIdx.x == ntile - 1) sm.n_steps = incl;
      if (fits) {
        TilePlan tp;
        decode(tile, tp);
        int e = incl - steps;
        for (int s = 0; s < tp.nseg; ++s) {
          const Seg<bf16> g = sm.seg[tp.seg_first + s];
          for (int k = g.kb; k < g.ke; k += BK, ++e) {
            StepEnt st;
            st.A = g.A + k;
            st.B = g.B + k;
            st.lda = (uint16_t)g.lda;
            st.ldb = (uint16_t)g.ldb;
            st.krem = (uint16_t)min(g.ke - k, BK);
            st.tile = (uint16_t)threadIdx.x;
            sm.step[e] = st;
          }
        }
        if (steps > 0) sm.tile[threadIdx.x].last_step = e - 1;
      }
    }
    __syncthreads();
    const int n_steps = sm.n_steps, n_tiles = sm.n_tiles;
    // ---- the pipeline ----
    f32x16 acc[MI][2];
    zero_acc(acc);
    int issued = 0;
    auto issue = [&]() {
      if (issued < n_steps) {
        const unsigned st = (unsigned)(issued % S);
        issue_step<TM, S>(sm, issued, a_lds + st * (unsigned)(TM * kRowBytes), b_lds + st * (unsigned)(TN * kRowBytes));
      }
      if (issued < n_steps) ++issued;
    };
    issue();
    if (S > 2) issue();
    for (int j = 0; j < n_steps; ++j) {
      if (S > 2 && issued > j + 1) wait_loads<NL>();  // all but the newest step's loads of this wavefront have landed
      else wait_loads<0>();
      barrier_only();  // ... and everybody's; all wavefronts are done reading the stage that is refilled next
      if (loads_first) issue();
      {
        const unsigned char *as = sm.a[j % S], *bs = sm.b[j % S];
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
          bf16x8_t a[MI], b[2];
#pragma unroll
          for (int i = 0; i < MI; ++i) a[i] = *reinterpret_cast<const bf16x8_t *>(as + arow + i * 32 * kRowBytes + koff[ks]);
#pragma unroll
          for (int jj = 0; jj < 2; ++jj) b[jj] = *reinterpret_cast<const bf16x8_t *>(bs + brow + jj * 32 * kRowBytes + koff[ks]);
#pragma unroll
          for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int jj = 0; jj < 2; ++jj) acc[i][jj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[jj], acc[i][jj], 0, 0, 0);
        }
      }
      if (!loads_first) issue();
      const int tl = __builtin_amdgcn_readfirstlane((int)sm.step[j].tile);
      if (__builtin_amdgcn_readfirstlane(sm.tile[tl].last_step) == j) {
        finish(acc, sm.tile[tl]);
        zero_acc(acc);
      }
    }
    // tiles without any K-step (no live segment): their output is the epilogue's alone; acc is zero here
    for (int t = 0; t < n_tiles; ++t)
      if (__builtin_amdgcn_readfirstlane(sm.tile[t].last_step) < 0) finish(acc, sm.tile[t]);
    batch0 += n_tiles * stride;
    __syncthreads();  // the lists are rewritten for the next batch
  }
}

// Swaps a value with the neighbouring lane (lane ^ 1).
__device__ __forceinline__ float swap_with_neighbour(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, false));
}

// Writes this wavefront's part of the tile, out[r * ld + c] = f(acc value, r, c) for r < rows, c < cols, straight from
// the accumulators (32x32 MFMA layout: lane % 32 is the column, the 16 values of a lane are rows
// 8 (v / 4) + 4 (lane / 32) + v % 4).  With an even leading dimension and a 4-byte aligned base, neighbouring lanes
// first exchange one value of every row pair, so that a lane stores two adjacent columns of one row at once and 16
// lanes write 64 contiguous bytes; otherwise element by element.
template <int MI, typename F>
__device__ __forceinline__ void store_tile_bf16(f32x16 (&acc)[MI][2], bf16 *out, int64_t ld, int rows, int cols, F f) {
  int tid = threadIdx.x;
  asm volatile("" : "+v"(tid));  // opaque: keeps the per-lane row / column / address terms of the 32 stores from being
                                 // hoisted out of the caller's K loop, where they would occupy ~100 registers
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = (wave >> 1) * 32 * MI, wn = (wave & 1) * 64;
  const bool paired = (ld & 1) == 0 && (reinterpret_cast<uintptr_t>(out) & 3) == 0;
  const int odd = lane & 1;
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int col = wn + j * 32 + (lane & 31);
#pragma unroll
      for (int v = 0; v < 16; v += 2) {
        const int row = wm + i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);  // acc[v]: (row, col), acc[v + 1]: (row + 1, col)
        const float x0 = f(acc[i][j][v], row, col), x1 = f(acc[i][j][v + 1], row + 1, col);
        if (paired) {
          // the even lane keeps row `row` (columns col, col + 1), the odd lane row + 1 (columns col - 1, col)
          const float got = swap_with_neighbour(odd ? x0 : x1);
          const int r = row + odd, c = col - odd;
          const unsigned w = odd ? pack2(got, x1) : pack2(x0, got);
          if (r < rows && c + 1 < cols) *reinterpret_cast<unsigned *>(out + (int64_t)r * ld + c) = w;
          else if (r < rows && c < cols) out[(int64_t)r * ld + c].bits = (uint16_t)(w & 0xffffu);
        } else {
          if (row < rows && col < cols) out[(int64_t)row * ld + col] = from_float<bf16>(x0);
          if (row + 1 < rows && col < cols) out[(int64_t)(row + 1) * ld + col] = from_float<bf16>(x1);
        }
      }
    }
}

}  // namespace dma
}  // namespace hgnn
