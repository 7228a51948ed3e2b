// lvx_xattn_fwd_static: lvx_xattn_fwd for callers that cannot allocate device memory (code under
// HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).  The KV-split partial
// results that lvx_xattn_fwd keeps in a caller workspace live here in a device array of fixed size
// that belongs to the library; everything else is the same code path and the same kernels.
#include "lvx_internal.h"

namespace {

// The scratch array: one copy per GPU the library runs on, held until the process ends.
static __device__ __align__(256) unsigned char scratch[LVX_STATIC_SCRATCH_BYTES];

// Device address of `scratch` on each device (the array's name is only a host-side stand-in).
constexpr int MAX_DEVICES = 64;
void* scratch_ptr[MAX_DEVICES] = {};

// Address of the current device's copy, resolved on that device's first call.  A race between
// host threads only repeats the query; both get the same address.
hipError_t scratch_of_current_device(void** out) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
  if (!scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    scratch_ptr[dev] = p;
  }
  *out = scratch_ptr[dev];
  return hipSuccess;
}

}  // namespace

extern "C" lvx_status lvx_xattn_fwd_static(const lvx_problem* p, lvx_dtype dtype, const void* q,
                                           const void* k, const void* v, const lvx_mask* mask,
                                           void* o, lvx_dtype o_dtype, float* lse, void* hip_stream) {
  // what this very call needs (invalid arguments give 0: lvx_xattn_fwd below then names the error)
  const size_t need = lvx::fwd_workspace_need(p, dtype, mask);
  if (need > (size_t)LVX_STATIC_SCRATCH_BYTES) return LVX_ERR_WORKSPACE;
  void* ws = nullptr;
  if (scratch_of_current_device(&ws) != hipSuccess) return LVX_ERR_HIP;
  // Nothing in the scratch has to start at zero: every slice of partial results that the combine
  // reads is written in full by the launch before it.
  return lvx_xattn_fwd(p, dtype, q, k, v, mask, o, o_dtype, lse, ws, (size_t)LVX_STATIC_SCRATCH_BYTES,
                       hip_stream);
}
