// Instrumentation only: a plain copy kernel of known traffic, used to calibrate the
// HBM byte counters (FETCH_SIZE / WRITE_SIZE) that the roofline figures are checked with.
#include "lrqk_internal.h"

namespace lrqk {
namespace {
__global__ __launch_bounds__(256) void calib_copy_kernel(const uint4* __restrict__ src,
                                                         uint4* __restrict__ dst, size_t n16) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n16) dst[i] = src[i];
}
}  // namespace
}  // namespace lrqk

extern "C" __attribute__((visibility("default"))) int lrqk_calib_copy(void* dst, const void* src,
                                                                      size_t bytes, void* stream) {
  using namespace lrqk;
  if (!dst || !src || !aligned16(dst) || !aligned16(src) || bytes % 16 != 0) return LRQK_EINVAL;
  const size_t n16 = bytes / 16;
  if (n16 == 0) return LRQK_OK;
  if ((n16 + 255) / 256 > 0x7fffffffull) return LRQK_ESHAPE;
  hipLaunchKernelGGL(calib_copy_kernel, dim3((unsigned)((n16 + 255) / 256)), dim3(256), 0,
                     static_cast<hipStream_t>(stream), static_cast<const uint4*>(src),
                     static_cast<uint4*>(dst), n16);
  LRQK_HIP(hipGetLastError());
  return LRQK_OK;
}
