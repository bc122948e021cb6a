// A forward entry point that allocates nothing and takes no scratch area from the caller: the work area of
// hgnn_layer_fwd (transposed weights, low-order plane of the aggregate) lives in a fixed device array of this
// library.  For callers that cannot allocate device memory: code under HIP graph capture, tight serving loops,
// harnesses that forbid it.
#include <mutex>

#include "common.h"

namespace hgnn {

static __device__ __align__(256) unsigned char scratch[HGNN_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_m;
static void *g_scratch_ptr[kMaxDevices] = {};  // device address of `scratch` on each GPU (every GPU holds its own copy)

// Called with `device` current (hgnn_create does, right after hipSetDevice): looks up, once per device, where that
// device's copy of the array lives.  The array's name is only a host-side handle; device work gets this address.
hgnn_status static_scratch_init(int device) {
  if (device < 0 || device >= kMaxDevices) HGNN_FAIL(HGNN_EINVAL, "device %d outside [0,%d)", device, kMaxDevices);
  std::lock_guard<std::mutex> lk(g_scratch_m);
  if (g_scratch_ptr[device]) return HGNN_OK;
  void *p = nullptr;
  HGNN_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
  if (!p) HGNN_FAIL(HGNN_EHIP, "hipGetSymbolAddress returned a NULL address for the static work area");
  g_scratch_ptr[device] = p;
  return HGNN_OK;
}

void *static_scratch_ptr(int device) {
  if (device < 0 || device >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lk(g_scratch_m);
  return g_scratch_ptr[device];
}

}  // namespace hgnn

extern "C" hgnn_status hgnn_layer_fwd_static(hgnn_ctx *ctx, void *stream, hgnn_graph *g, int32_t layer,
                                             const hgnn_layer_params *p, const void *x_merged, void *h_out, void *saved,
                                             size_t saved_bytes) {
  using namespace hgnn;
  if (!ctx) HGNN_FAIL(HGNN_EINVAL, "NULL context");
  if (ctx->device < 0) HGNN_FAIL(HGNN_EUNSUPPORTED, "host-only context cannot run device work");
  void *ptr = static_scratch_ptr(ctx->device);
  if (!ptr) HGNN_FAIL(HGNN_EHIP, "the static work area of device %d was not set up", ctx->device);
  return layer_fwd_static_area(ctx, stream, g, layer, p, x_merged, h_out, saved, saved_bytes, ptr, HGNN_STATIC_SCRATCH_BYTES);
}
