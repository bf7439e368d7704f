// fupr_forward_static: the forward pass for callers that cannot allocate device
// memory (code under HIP-graph capture, tight serving loops, harnesses that
// forbid it).  The workspace that fupr_forward takes from its caller is here a
// fixed array in device memory that belongs to the library.
#include <hip/hip_runtime.h>

#include <mutex>

#include "fupr.h"

namespace {

// The workspace: one copy per GPU, at that GPU's own address, held until the
// process ends.  Host code never uses this name as an address: it asks the
// runtime for the device address once per device (below) and uses that.
static __device__ __align__(256) unsigned char scratch[FUPR_STATIC_WORKSPACE_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_mutex;
void* g_ptr[kMaxDevices] = {};   // device address of `scratch` on each GPU, nullptr = not asked yet

// The current device's copy of the array; nullptr (and *st set) when the runtime
// cannot say where it is.
void* static_workspace(fupr_status* st) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    (void)hipGetLastError();
    *st = FUPR_ERR_LAUNCH;
    return nullptr;
  }
  std::lock_guard<std::mutex> lock(g_mutex);
  if (!g_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
      (void)hipGetLastError();
      *st = FUPR_ERR_LAUNCH;
      return nullptr;
    }
    g_ptr[dev] = ptr;
  }
  return g_ptr[dev];
}

}  // namespace

extern "C" size_t fupr_static_workspace_bytes(void) { return FUPR_STATIC_WORKSPACE_BYTES; }

extern "C" fupr_status fupr_forward_static(const fupr_model* m, const fupr_tensor* input,
                                           const fupr_tensor* output, void* stream) {
  if (!m || !input || !output) return FUPR_ERR_NULL;
  // the size check comes first: a batch that does not fit is refused before anything else happens
  if (input->N <= 0) return FUPR_ERR_SHAPE;
  const size_t need = fupr_model_workspace_bytes(m, input->N);
  if (need == 0 || need > (size_t)FUPR_STATIC_WORKSPACE_BYTES) return FUPR_ERR_WORKSPACE;
  fupr_status st = FUPR_OK;
  void* ws = static_workspace(&st);
  if (!ws) return st;
  // Every tensor in the workspace is written in full by the operator that
  // produces it before any operator reads it, so what the previous call left
  // there needs no clearing.
  return fupr_forward(m, input, output, ws, (size_t)FUPR_STATIC_WORKSPACE_BYTES, stream);
}
