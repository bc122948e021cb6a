// Work of one block on a list of weight transposes (TransposeJobs): block b of nb takes the 32x32 tiles b, b + nb, ...
// of all jobs.  `tile` is a 32x33 LDS buffer of the calling kernel; every thread of the (256-thread) block calls this.
#pragma once
#include "common.h"
#include "device_types.h"

namespace hgnn {

template <typename T>
__device__ __forceinline__ void transpose_jobs_block(const TransposeJobs &tj, int b, int nb, T (*tile)[33]) {
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;  // 32 x 8
  const int total = tj.tile_off[tj.n];
  const int H = tj.H, tiles_h = (H + 31) / 32;
  int job = 0;
  for (int tl = b; tl < total; tl += nb) {
    while (tl >= tj.tile_off[job + 1]) ++job;
    const int local = tl - tj.tile_off[job];
    const int F = tj.F[job];
    const T *w = reinterpret_cast<const T *>(tj.w[job]);
    T *out = reinterpret_cast<T *>(tj.out) + (int64_t)tj.off4[job] * 4;
    const int f0 = (local / tiles_h) * 32, h0 = (local % tiles_h) * 32;
    for (int i = ty; i < 32; i += 8) {
      const int f = f0 + i, h = h0 + tx;
      if (f < F && h < H) tile[i][tx] = w[(int64_t)f * H + h];
    }
    __syncthreads();
    for (int i = ty; i < 32; i += 8) {
      const int h = h0 + i, f = f0 + tx;
      if (f < F && h < H) out[(int64_t)h * F + f] = tile[tx][i];
    }
    __syncthreads();
  }
}

}  // namespace hgnn
