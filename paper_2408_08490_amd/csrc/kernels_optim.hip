// Parameter update (Section 2.3, step 4: "gradient computation and parameter update"): Adam (Kingma & Ba 2015,
// Algorithm 1) on fp32 master copies, one launch for a whole list of weight tensors, and the same update on the
// rows of an embedding table that a mini-batch touched.  Both are plain streaming kernels (HBM-bound).
#include "common.h"
#include "device_types.h"

namespace hgnn {

struct AdamCoef {
  float lr, b1, b2, eps, c1, c2;  // c1 = 1 / (1 - b1^t), c2 = 1 / (1 - b2^t)
};

__device__ __forceinline__ float adam_one(float th, float g, float &m, float &v, const AdamCoef &k) {
  m = k.b1 * m + (1.f - k.b1) * g;
  v = k.b2 * v + (1.f - k.b2) * g * g;
  return th - k.lr * (m * k.c1) / (sqrtf(v * k.c2) + k.eps);
}

constexpr int kAdamTensors = 48;     // tensors per launch (the table travels as a kernel argument)
constexpr int kAdamPerBlock = 2048;  // elements per block: 256 threads x 8
struct AdamTab {
  void *param[kAdamTensors];
  float *master[kAdamTensors];  // NULL: the parameter itself is the fp32 master
  const float *grad[kAdamTensors];
  float *m[kAdamTensors], *v[kAdamTensors];
  int64_t numel[kAdamTensors];
  int32_t block_off[kAdamTensors + 1];
  int32_t n;
};

template <typename T>
__global__ void __launch_bounds__(256) adam_dense_kernel(AdamTab tab, AdamCoef k) {
  int t = 0;
  while (t + 1 < tab.n && (int)blockIdx.x >= tab.block_off[t + 1]) ++t;
  const int64_t base = (int64_t)(blockIdx.x - tab.block_off[t]) * kAdamPerBlock;
  const int64_t n = tab.numel[t];
  float *master = tab.master[t] ? tab.master[t] : reinterpret_cast<float *>(tab.param[t]);
  T *param = reinterpret_cast<T *>(tab.param[t]);
  const float *g = tab.grad[t];
  float *m = tab.m[t], *v = tab.v[t];
#pragma unroll
  for (int j = 0; j < kAdamPerBlock / 256; ++j) {
    const int64_t i = base + j * 256 + threadIdx.x;
    if (i < n) {
      float mi = m[i], vi = v[i];
      const float th = adam_one(master[i], g[i], mi, vi, k);
      m[i] = mi;
      v[i] = vi;
      master[i] = th;
      if (tab.master[t]) param[i] = from_float<T>(th);
    }
  }
}

hgnn_status launch_adam_dense(hipStream_t s, int dtype, int n, void *const *param, float *const *master,
                              const float *const *grad, float *const *m, float *const *v, const int64_t *numel,
                              float lr, float b1, float b2, float eps, double c1, double c2) {
  const AdamCoef k{lr, b1, b2, eps, (float)c1, (float)c2};
  for (int i = 0; i < n;) {  // one launch per batch of up to kAdamTensors non-empty tensors; `i` runs on across batches
    AdamTab tab;
    tab.n = 0;
    tab.block_off[0] = 0;
    for (; i < n && tab.n < kAdamTensors; ++i) {
      if (numel[i] == 0) continue;
      const int j = tab.n++;
      tab.param[j] = param[i];
      tab.master[j] = master ? master[i] : nullptr;
      tab.grad[j] = grad[i];
      tab.m[j] = m[i];
      tab.v[j] = v[i];
      tab.numel[j] = numel[i];
      tab.block_off[j + 1] = tab.block_off[j] + (int32_t)((numel[i] + kAdamPerBlock - 1) / kAdamPerBlock);
    }
    if (tab.n == 0) continue;
    const dim3 grid(tab.block_off[tab.n]);
    if (dtype == HGNN_BF16) HGNN_LAUNCH(adam_dense_kernel<bf16>, grid, dim3(256), 0, s, tab, k);
    else HGNN_LAUNCH(adam_dense_kernel<float>, grid, dim3(256), 0, s, tab, k);
    HGNN_HIP(hipGetLastError());
  }
  return HGNN_OK;
}

// One group of lanes per listed row; a lane owns 16-byte pieces of the gradient row (N scalars of T) and the
// matching fp32 pieces of the master row and the moments.
template <typename T>
__global__ void __launch_bounds__(256) adam_rows_kernel(T *__restrict__ store, float *__restrict__ master,
                                                         float *__restrict__ m, float *__restrict__ v, int F,
                                                         const int64_t *__restrict__ ids, int64_t n_rows,
                                                         const T *__restrict__ grad, AdamCoef k, int lpr_log2) {
  using V = Vec16<T>;
  const int lpr = 1 << lpr_log2;
  const int64_t row = (int64_t)blockIdx.x * (256 >> lpr_log2) + (threadIdx.x >> lpr_log2);
  const int lane = threadIdx.x & (lpr - 1);
  if (row >= n_rows) return;
  const int64_t id = ids[row];
  float *mast = master ? master : reinterpret_cast<float *>(store);
  for (int c = lane; c < F / V::N; c += lpr) {
    float g[V::N];
#pragma unroll
    for (int i = 0; i < V::N; ++i) g[i] = 0.f;
    V::add(g, reinterpret_cast<const uint4 *>(grad + row * F)[c]);
    const int64_t o = id * F + (int64_t)c * V::N;
    float out[V::N];
#pragma unroll
    for (int q = 0; q < V::N / 4; ++q) {
      float4 th = reinterpret_cast<const float4 *>(mast + o)[q];
      float4 mm = reinterpret_cast<const float4 *>(m + o)[q], vv = reinterpret_cast<const float4 *>(v + o)[q];
      th.x = adam_one(th.x, g[4 * q + 0], mm.x, vv.x, k);
      th.y = adam_one(th.y, g[4 * q + 1], mm.y, vv.y, k);
      th.z = adam_one(th.z, g[4 * q + 2], mm.z, vv.z, k);
      th.w = adam_one(th.w, g[4 * q + 3], mm.w, vv.w, k);
      reinterpret_cast<float4 *>(m + o)[q] = mm;
      reinterpret_cast<float4 *>(v + o)[q] = vv;
      reinterpret_cast<float4 *>(mast + o)[q] = th;
      out[4 * q + 0] = th.x; out[4 * q + 1] = th.y; out[4 * q + 2] = th.z; out[4 * q + 3] = th.w;
    }
    if (master) reinterpret_cast<uint4 *>(store + id * F)[c] = V::pack(out);
  }
}

hgnn_status launch_adam_rows(hipStream_t s, int dtype, void *store, float *master, float *m, float *v, int F,
                             const int64_t *ids, int64_t n_rows, const void *grad, float lr, float b1, float b2,
                             float eps, double c1, double c2) {
  if (n_rows == 0) return HGNN_OK;
  const AdamCoef k{lr, b1, b2, eps, (float)c1, (float)c2};
  const int es = dtype == HGNN_BF16 ? 2 : 4;
  const int l2 = lanes_log2_for(F, es);
  const int rpb = 256 >> l2;
  const dim3 grid((unsigned)((n_rows + rpb - 1) / rpb));
  if (dtype == HGNN_BF16)
    HGNN_LAUNCH(adam_rows_kernel<bf16>, grid, dim3(256), 0, s, (bf16 *)store, master, m, v, F, ids, n_rows, (const bf16 *)grad, k, l2);
  else
    HGNN_LAUNCH(adam_rows_kernel<float>, grid, dim3(256), 0, s, (float *)store, master, m, v, F, ids, n_rows, (const float *)grad, k, l2);
  HGNN_HIP(hipGetLastError());
  return HGNN_OK;
}

}  // namespace hgnn
