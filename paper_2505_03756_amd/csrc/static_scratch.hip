// The one entry point that allocates nothing: flp_lora_apply_paged with its intermediates (segment lists,
// the fp32 shrink output, the transposed / unrounded dense base where it fits) in a file-scope device array
// instead of the pool's growing workspace.  For callers that cannot call hipMalloc: code under graph capture,
// tight serving loops, harnesses that forbid allocation.
#include <hip/hip_runtime.h>

#include <mutex>

#include "flp_internal.h"

namespace {

constexpr size_t kScratchBytes = (size_t)64 << 20;   // 64 MiB per GPU, held until the process ends

}  // namespace

// Every GPU that loads the library holds its own copy of this array at its own address.  In host code the name is
// only a handle for hipGetSymbolAddress; kernels and copies get the looked-up device pointer.
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_mu;
void* g_scratch_ptr[kMaxDevices] = {};   // device address of `scratch` on device i, null until looked up

flp_status resolve_for_pool(flp_pool* p, void** out) {
  int cur = -1;
  FLP_TRY_HIP(hipGetDevice(&cur));
  if (cur != p->device) {
    flp_set_error("flp_lora_apply_paged_static: device %d is current, the pool lives on device %d", cur, p->device);
    return FLP_EINVAL;
  }
  return flp_static_scratch_setup(cur, out);
}

}  // namespace

// Looks the array's device address up once per device, with that device current.
flp_status flp_static_scratch_setup(int device, void** out) {
  if (device < 0 || device >= kMaxDevices) {
    flp_set_error("static scratch: device index %d outside 0..%d", device, kMaxDevices - 1);
    return FLP_EINVAL;
  }
  std::lock_guard<std::mutex> lk(g_mu);
  if (!g_scratch_ptr[device]) {
    int cur = -1;
    FLP_TRY_HIP(hipGetDevice(&cur));
    if (cur != device) {
      flp_set_error("static scratch: device %d must be current for the look-up (device %d is)", device, cur);
      return FLP_EINVAL;
    }
    void* ptr = nullptr;
    FLP_TRY_HIP(hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch)));
    if (!ptr || ((uintptr_t)ptr & 255)) {
      flp_set_error("static scratch: look-up returned %p", ptr);
      return FLP_EHIP;
    }
    g_scratch_ptr[device] = ptr;
  }
  if (out) *out = g_scratch_ptr[device];
  return FLP_OK;
}

extern "C" int64_t flp_static_scratch_bytes(void) { return (int64_t)kScratchBytes; }

extern "C" flp_status flp_lora_apply_paged_static(flp_pool* pool, const flp_lora_batch* batch, void* hip_stream) {
  const FlpFixedWorkspace ws{kScratchBytes, resolve_for_pool, "flp_lora_apply_paged_static"};
  return flp_lora_apply_fixed(pool, batch, hip_stream, ws);
}
