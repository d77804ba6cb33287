// Small dense linear algebra inside one wavefront (gfx950): r x r symmetric positive definite
// systems with r <= 64, lane i holding row i of the matrix in registers.  Used by the
// decode-time factor update and by the prefill factorisation.
#pragma once

#include <hip/hip_runtime.h>

#include <utility>

namespace lrqk {
namespace linalg {

__device__ __forceinline__ float lane_value(float v, int lane) {
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}

// m[c] -= l * (l of lane c) for c >= C0.  The lane reads are issued in groups ahead of the
// multiply-adds that use them: a lane read followed at once by its use waits for the scalar
// register, and the compiler keeps the order written here.
template <int R, int C0>
__device__ __forceinline__ void rank_one_downdate(float (&m)[R], float l) {
  constexpr int kGroup = 8;
#pragma unroll
  for (int cb = C0 / kGroup * kGroup; cb < R; cb += kGroup) {
    float lc[kGroup];
#pragma unroll
    for (int u = 0; u < kGroup; ++u) lc[u] = cb + u < R ? lane_value(l, cb + u) : 0.0f;
#pragma unroll
    for (int u = 0; u < kGroup; ++u)
      if (cb + u >= C0 && cb + u < R) m[cb + u] = __builtin_fmaf(-l, lc[u], m[cb + u]);
  }
}

// Building blocks; lane i (< R) holds row i of the matrix in m[], element i of a vector in a
// scalar.  Every register index is a compile-time constant: the column loops of the
// factorisations are written as pack expansions over the column number (a loop of that size
// is beyond what the compiler agrees to unroll at r = 64), the others are fully unrolled.
//
// Column J of a right-looking Cholesky factorisation M = L L^T, in place.
template <int R, int J>
__device__ __forceinline__ void chol_column(float (&m)[R], float& dinv, int lane) {
  const float inv = __builtin_amdgcn_rsqf(lane_value(m[J], J));
  const float l = m[J] * inv;
  m[J] = l;
  if (lane == J) dinv = inv;
  rank_one_downdate<R, J + 1>(m, l);
}
template <int R, int... J>
__device__ __forceinline__ void chol_columns(float (&m)[R], float& dinv, int lane,
                                             std::integer_sequence<int, J...>) {
  (chol_column<R, J>(m, dinv, lane), ...);
}
template <int R, int... J>
__device__ __forceinline__ void chol_columns2(float (&m0)[R], float (&m1)[R], float& dinv0,
                                              float& dinv1, int lane,
                                              std::integer_sequence<int, J...>) {
  ((chol_column<R, J>(m0, dinv0, lane), chol_column<R, J>(m1, dinv1, lane)), ...);
}
// M = L L^T in place: afterwards m[j] of lane i >= j holds L[i][j].  Returns, in lane j,
// 1 / L[j][j].  The two-matrix form factorises two independent matrices column by column in
// turn, so that their dependency chains interleave.
template <int R>
__device__ __forceinline__ void chol_factor2(float (&m0)[R], float (&m1)[R], float& dinv0,
                                             float& dinv1, int lane) {
  dinv0 = dinv1 = 0.0f;
  chol_columns2<R>(m0, m1, dinv0, dinv1, lane, std::make_integer_sequence<int, R>{});
}
template <int R>
__device__ __forceinline__ float chol_factor(float (&m)[R], int lane) {
  float dinv = 0.0f;
  chol_columns<R>(m, dinv, lane, std::make_integer_sequence<int, R>{});
  return dinv;
}
// L y = b with L[i][j] = L[j] of lane i
template <int R>
__device__ __forceinline__ float tri_forward(const float (&L)[R], float dinv, float b, int lane) {
  float y = 0.0f;
#pragma unroll
  for (int j = 0; j < R; ++j) {
    const float yj = lane_value(b * dinv, j);
    if (lane == j) y = yj;
    b = __builtin_fmaf(-L[j], yj, b);
  }
  return y;
}
// L^T x = y with the transposed factor: Lt[j] of lane i = L[j][i]
template <int R>
__device__ __forceinline__ float tri_backward(const float (&Lt)[R], float dinv, float y, int lane) {
  float x = 0.0f;
#pragma unroll
  for (int j = R - 1; j >= 0; --j) {
    const float xj = lane_value(y * dinv, j);
    if (lane == j) x = xj;
    y = __builtin_fmaf(-Lt[j], xj, y);
  }
  return x;
}
// out[c] of lane i = in[i] of lane c, through R * (R + 1) floats of LDS owned by the wavefront
// (in and out may be the same array)
template <int R>
__device__ __forceinline__ void transpose_rows(const float (&in)[R], float (&out)[R], float* lt,
                                               int lane) {
  __builtin_amdgcn_wave_barrier();
  if (lane < R) {
#pragma unroll
    for (int c = 0; c < R; ++c) lt[lane * (R + 1) + c] = in[c];
  }
  __builtin_amdgcn_wave_barrier();
  if (lane < R) {
#pragma unroll
    for (int c = 0; c < R; ++c) out[c] = lt[c * (R + 1) + lane];
  }
  __builtin_amdgcn_wave_barrier();
}

}  // namespace linalg
}  // namespace lrqk
