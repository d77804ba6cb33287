// lrqk_sparse_attend_noalloc: step a5 for callers that can neither allocate device memory nor
// hand over a workspace (code under HIP graph capture, tight serving loops, harnesses that
// forbid hipMalloc).  Same kernels as lrqk_sparse_attend; the partial softmax states that the
// split attention hands from its first launch to its second live in a file-scope device array
// instead of a caller's workspace.
//
// The array exists once per GPU (every device that loads this code object holds its own copy
// at its own address, until the process ends).  In host code the array's name is only a
// stand-in for that address: the device address is looked up once per device with
// hipGetSymbolAddress, with that device current, and only that pointer is ever handed to a
// kernel.
#include <mutex>

#include "lrqk_internal.h"

namespace lrqk {
namespace {

constexpr size_t kScratchBytes = LRQK_NOALLOC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_mu;
void* g_scratch_ptr[kMaxDevices];  // device address of `scratch` on each GPU, once known

// Device address of this GPU's scratch array (looked up on the first call on each device).
int scratch_for_current_device(void** out) {
  int dev = -1;
  LRQK_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return LRQK_EINVAL;
  std::lock_guard<std::mutex> g(g_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    LRQK_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p || !aligned256(p)) return LRQK_EINVAL;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return LRQK_OK;
}

}  // namespace
}  // namespace lrqk

extern "C" __attribute__((visibility("default"))) int lrqk_sparse_attend_noalloc(
    const lrqk_shape* shape, const float* q, const void* cacheK, const void* cacheV,
    const int32_t* sel_slot, const void* liteK, const void* liteV, float* out, void* stream) {
  using namespace lrqk;
  const int rc = lrqk_validate_shape(shape);
  if (rc != LRQK_OK) return rc;
  auto ok16 = [](const void* p) { return p && aligned16(p); };
  if (!ok16(q) || !ok16(cacheK) || !ok16(cacheV) || !ok16(sel_slot) || !ok16(out))
    return LRQK_EINVAL;
  if (shape->w > 0 && (!ok16(liteK) || !ok16(liteV))) return LRQK_EINVAL;
  const int BHq = shape->B * shape->Hq;
  // sizes beyond the fixed array are refused before anything is enqueued
  if (attend_ws_bytes(BHq, shape->k, shape->w, 1) > kScratchBytes) return LRQK_ENOMEM;
  void* ptr = nullptr;
  const int rs = scratch_for_current_device(&ptr);
  if (rs != LRQK_OK) return rs;
  const AttendGeom g = attend_geometry(BHq, shape->k, shape->w);
  hipStream_t st = static_cast<hipStream_t>(stream);
  // every partial that the merge reads is written by the first launch: nothing to clear
  float* partials = static_cast<float*>(ptr);
  LRQK_HIP(launch_attend_partial(*shape, kAttendAll, q, cacheK, cacheV, sel_slot, nullptr, nullptr,
                                 nullptr, liteK, liteV, partials, g.nsplit, g.rows_per_block,
                                 g.nsplit, 0, st));
  LRQK_HIP(launch_attend_combine(*shape, partials, g.nsplit, g.nsplit, out, st));
  return LRQK_OK;
}
