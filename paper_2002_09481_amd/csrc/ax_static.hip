// ax_layer_run_static: the per-call part of a prepared layer with the scratch taken from a
// file-scope device array instead of a caller-provided workspace, for callers that cannot
// allocate device memory (code under HIP graph capture, serving loops that forbid allocation).
//
// The array's name is a host-side stand-in for a device symbol, not a device address: its
// address on the current device is looked up once per device with hipGetSymbolAddress and that
// pointer, never the name, is what the kernels receive.
#include <mutex>

#include "ax_internal.h"

namespace ax {
namespace {

constexpr size_t kStaticScratchBytes = (size_t)64 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_mu;
void* g_scratch_ptr[kMaxDevices];  // device address of `scratch` on each device, once looked up

// Address of the array on the current device (every device holds its own copy at its own address).
int scratch_on_current_device(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return AX_ERR_HIP;
  std::lock_guard<std::mutex> lock(g_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return AX_ERR_HIP;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return AX_OK;
}

}  // namespace
}  // namespace ax

extern "C" size_t ax_static_scratch_bytes(void) { return ax::kStaticScratchBytes; }

extern "C" int ax_layer_run_static(const ax_layer_t* layer, const void* x, int32_t* acc_out, float* y_out,
                                   void* hip_stream) {
  using namespace ax;
  if (!layer) return AX_ERR_NULL;
  if (!layer->ready) return AX_ERR_STATE;
  if (scratch_need(layer, x) > kStaticScratchBytes) return AX_ERR_WORKSPACE;
  void* ptr = nullptr;
  const int rc = scratch_on_current_device(&ptr);
  if (rc) return rc;
  // Nothing in the scratch has to start at zero: every part a call reads (materialized or packed
  // activations, their sums, pieces of shared tiles) is written by the same call first.
  return run_prepared(layer, x, acc_out, y_out, ptr, kStaticScratchBytes, kPhCall | kPhMain | kPhFixup, 1,
                      (hipStream_t)hip_stream);
}
