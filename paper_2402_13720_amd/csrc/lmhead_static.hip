// ouro_lmhead_argmax for callers that cannot allocate: the cross-slab (value, id) partials live in a buffer that is
// part of this library's device image instead of a caller-provided workspace.  Everything else -- validation, launch
// plan, kernels -- is the ordinary entry point's.
#include "ouro_internal.hpp"

namespace ouro {

namespace {

// One copy of this array exists on every GPU the library's code object is loaded on, at that GPU's own address.  In host
// code the name is only a handle for hipGetSymbolAddress; the device address it returns is what kernels and copies get.
static __device__ __align__(256) unsigned char scratch[OURO_LMHEAD_STATIC_SCRATCH_BYTES];

DeviceOnce g_once;
void* g_scratch_ptr[kMaxDevices];      // device address of `scratch` on each GPU, filled once per device

// Device address of the current device's copy of the buffer (looked up on the first call on that device, with that
// device current).
int scratch_address(void** out) {
  int dev = 0;
  const hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_failed(e);
  if (dev < 0 || dev >= kMaxDevices) return OURO_E_BAD_SHAPE;
  const int st = device_once(g_once, [dev] {
    void* p = nullptr;
    const hipError_t err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (err != hipSuccess) return hip_failed(err);
    if (!p) return hip_failed(hipErrorInvalidSymbol);
    g_scratch_ptr[dev] = p;
    return static_cast<int>(OURO_OK);
  });
  if (st != OURO_OK) return st;
  *out = g_scratch_ptr[dev];
  return OURO_OK;
}

}  // namespace

}  // namespace ouro

using namespace ouro;

extern "C" int ouro_lmhead_argmax_static(const ouro_lmhead_desc* desc, void* hip_stream) {
  ouro_lmhead_desc d;
  {
    // validated as given, except that no workspace is asked of the caller
    if (!desc) return OURO_E_NULLPTR;
    if (desc->struct_size != sizeof(ouro_lmhead_desc)) return OURO_E_BAD_STRUCT;
    d = *desc;
    d.workspace = nullptr;
    d.workspace_bytes = 0;
    const int st = validate_lmhead(&d, true);
    if (st != OURO_OK) return st;
  }
  if (d.R == 0) return OURO_OK;
  const LmPlan p = plan_lmhead(d);
  if (p.total() > OURO_LMHEAD_STATIC_SCRATCH_BYTES) return OURO_E_STATIC_SCRATCH_TOO_SMALL;
  void* ptr = nullptr;
  const int st = scratch_address(&ptr);
  if (st != OURO_OK) return st;
  d.workspace = ptr;
  d.workspace_bytes = OURO_LMHEAD_STATIC_SCRATCH_BYTES;
  return enqueue_lmhead(d, p, static_cast<hipStream_t>(hip_stream));
}
