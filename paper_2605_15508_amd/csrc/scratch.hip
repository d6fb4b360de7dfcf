// Scratch memory of sts_sparse_attn_static, the entry point that allocates nothing: one array in
// the device memory of every GPU this code object is loaded on, held until the process ends.
#include <mutex>

#include "common.h"

// In host code the array's name is only a handle, not a device address: the address of a
// device's copy is asked from the runtime once, with that device current, and kept.
static __device__ __align__(256) unsigned char scratch[STS_STATIC_SCRATCH_BYTES];

namespace {
constexpr int MAX_DEVICES = 64;
std::mutex g_mu;
void *g_ptr[MAX_DEVICES] = {nullptr};
}  // namespace

sts_status sts_static_scratch(void **out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return STS_EHIP;
  std::lock_guard<std::mutex> lk(g_mu);
  if (!g_ptr[dev]) {
    void *ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return STS_EHIP;
    g_ptr[dev] = ptr;
  }
  *out = g_ptr[dev];
  return STS_OK;
}
