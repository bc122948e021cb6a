// Second stage of the bias gradient: the row pass over G' leaves one row of column sums per block in
// bpart [blocks x H] (the blocks of vertex type t are consecutive, ceil(n_dst[t] / rpb) of them); this adds a
// type's rows up and STORES dbias_t.  Shared by the stand-alone launch and by the blocks that the merged
// backward GEMM launch sets aside for it.
#pragma once
#include "common.h"

namespace hgnn {

// Block bx (256 threads) of bias_reduce_blocks(): 32 columns of one type; eight groups of 32 lanes sum every
// eighth row each, four independent loads per trip.
__device__ __forceinline__ void bias_reduce_part(const TypeTab &tt, const GradPtrTab &gt, int H, int rpb,
                                                 const float *__restrict__ bpart, int bx) {
  __shared__ float red[256];
  const int cb = (H + 31) / 32;
  const int t = bx / cb, lane32 = threadIdx.x & 31, part = threadIdx.x >> 5;
  const int c = (bx % cb) * 32 + lane32;
  float *db = gt.dbias[t];
  if (!db) return;  // whole block
  int b0 = 0;
  for (int u = 0; u < t; ++u) b0 += (tt.n_dst[u] + rpb - 1) / rpb;
  const int nb = (tt.n_dst[t] + rpb - 1) / rpb;
  float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
  if (c < H) {
    const float *p = bpart + (int64_t)b0 * H + c;
    int i = part;
    for (; i + 24 < nb; i += 32) {
      a0 += p[(int64_t)i * H];
      a1 += p[(int64_t)(i + 8) * H];
      a2 += p[(int64_t)(i + 16) * H];
      a3 += p[(int64_t)(i + 24) * H];
    }
    for (; i < nb; i += 8) a0 += p[(int64_t)i * H];
  }
  red[threadIdx.x] = (a0 + a1) + (a2 + a3);
  __syncthreads();
  if (part == 0 && c < H) {
    float sum = 0.f;
#pragma unroll
    for (int q = 0; q < 8; ++q) sum += red[q * 32 + lane32];
    db[c] = sum;
  }
}

}  // namespace hgnn
