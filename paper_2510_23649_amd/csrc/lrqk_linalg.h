// Small dense linear algebra inside one wavefront (gfx950): r x r symmetric positive definite
// systems with r <= 64, lane i holding row i of the matrix in registers.  Used by the
// decode-time factor update and by the prefill factorisation.
#pragma once

#include <hip/hip_runtime.h>

namespace lrqk {
namespace linalg {

__device__ __forceinline__ float lane_value(float v, int lane) {
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}

// Building blocks; lane i (< R) holds row i of the matrix in m[], element i of a vector in a
// scalar.  All loops are fully unrolled, so every register index is a constant.
//
// Right-looking Cholesky factorisation M = L L^T, in place: afterwards m[j] of lane i >= j
// holds L[i][j].  Returns, in lane j, 1 / L[j][j].  Two independent matrices are factorised
// together so that their dependency chains interleave.
template <int R>
__device__ __forceinline__ void chol_factor2(float (&m0)[R], float (&m1)[R], float& dinv0,
                                             float& dinv1, int lane) {
  dinv0 = dinv1 = 0.0f;
#pragma unroll
  for (int j = 0; j < R; ++j) {
    const float inv0 = __builtin_amdgcn_rsqf(lane_value(m0[j], j));
    const float inv1 = __builtin_amdgcn_rsqf(lane_value(m1[j], j));
    const float l0 = m0[j] * inv0, l1 = m1[j] * inv1;
    m0[j] = l0;
    m1[j] = l1;
    if (lane == j) {
      dinv0 = inv0;
      dinv1 = inv1;
    }
#pragma unroll
    for (int c = j + 1; c < R; ++c) {
      m0[c] = __builtin_fmaf(-l0, lane_value(l0, c), m0[c]);
      m1[c] = __builtin_fmaf(-l1, lane_value(l1, c), m1[c]);
    }
  }
}
template <int R>
__device__ __forceinline__ float chol_factor(float (&m)[R], int lane) {
  float dinv = 0.0f;
#pragma unroll
  for (int j = 0; j < R; ++j) {
    const float inv = __builtin_amdgcn_rsqf(lane_value(m[j], j));
    const float lij = m[j] * inv;
    m[j] = lij;
    if (lane == j) dinv = inv;
#pragma unroll
    for (int c = j + 1; c < R; ++c) m[c] = __builtin_fmaf(-lij, lane_value(lij, c), m[c]);
  }
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
