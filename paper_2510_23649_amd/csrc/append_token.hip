// u2 -- the new token joins the context (Alg. 2: "concatenate" k_hat_t to A_K, append k_t, v_t
// to the rows kept on the GPU, "Async k_t, v_t to CPU").
//
// One small kernel, one workgroup per (batch, KV head):
//   * row l of A_K receives k_hat_t;
//   * row l of the K and V stores receives k_t and v_t.  The stores are pinned host memory
//     mapped into the device's address space, so these are ordinary vector stores that
//     travel over the host link and are complete when the kernel has finished: the copy
//     is asynchronous to the host, as the paper asks, and ordered with the later fetches
//     of the same row by the stream;
//   * the lite rows are a ring of w rows: row l mod w, which holds the position l - w that
//     now leaves the window, is overwritten with k_t, v_t;
//   * slot_of[., l] = -1 for the G query heads: the new token is not in the cache (its rows
//     are reachable through the lite window, and through the host store once it has left it).
#include "lrqk_internal.h"

namespace lrqk {
namespace {

constexpr int kAppendThreads = 64;

__global__ __launch_bounds__(kAppendThreads) void append_token_kernel(
    float* __restrict__ A_K, uint4* __restrict__ K_host, uint4* __restrict__ V_host,
    uint4* __restrict__ liteK, uint4* __restrict__ liteV, int32_t* __restrict__ slot_of,
    const float* __restrict__ k_hat, const uint4* __restrict__ k_new,
    const uint4* __restrict__ v_new, int Hq, int Hkv, int l, int lrows, int r, int w, int row16) {
  const int bkv = blockIdx.x, t = threadIdx.x;
  const int b = bkv / Hkv, kvh = bkv - b * Hkv;
  const int G = Hq / Hkv;
  for (int c = t; c < r; c += kAppendThreads)
    A_K[((size_t)bkv * lrows + l) * r + c] = k_hat[(size_t)bkv * r + c];
  for (int c = t; c < row16; c += kAppendThreads) {
    const uint4 kx = k_new[(size_t)bkv * row16 + c];
    const uint4 vx = v_new[(size_t)bkv * row16 + c];
    K_host[((size_t)bkv * lrows + l) * row16 + c] = kx;
    V_host[((size_t)bkv * lrows + l) * row16 + c] = vx;
    if (w > 0) {
      liteK[((size_t)bkv * w + l % w) * row16 + c] = kx;
      liteV[((size_t)bkv * w + l % w) * row16 + c] = vx;
    }
  }
  if (t < G) slot_of[((size_t)b * Hq + (size_t)kvh * G + t) * lrows + l] = -1;
}

}  // namespace

hipError_t launch_append_token(const lrqk_shape& s, float* A_K, void* K_host, void* V_host,
                               void* liteK, void* liteV, int32_t* slot_of, const float* k_hat,
                               const void* k_new, const void* v_new, hipStream_t st) {
  const int row16 = (int)(kD * kv_elem_bytes(s.kv_dtype) / 16);
  hipLaunchKernelGGL(append_token_kernel, dim3(s.B * s.Hkv), dim3(kAppendThreads), 0, st, A_K,
                     static_cast<uint4*>(K_host), static_cast<uint4*>(V_host),
                     static_cast<uint4*>(liteK), static_cast<uint4*>(liteV), slot_of, k_hat,
                     static_cast<const uint4*>(k_new), static_cast<const uint4*>(v_new), s.Hq,
                     s.Hkv, s.l, row_cap(s), s.r, s.w, row16);
  return hipGetLastError();
}

}  // namespace lrqk
