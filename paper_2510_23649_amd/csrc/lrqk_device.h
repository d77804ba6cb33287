// Device-side helpers shared by the selection kernels (gfx950, 64-wide wavefronts).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lrqk {
namespace dev {

// Order-preserving key of a score: larger score <=> larger key; -0.0f ranks with +0.0f.
__device__ __forceinline__ uint32_t order_key(float s) {
  uint32_t u = __float_as_uint(s);
  if (u == 0x80000000u) u = 0u;
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Inverse of order_key (the key of -0.0f comes back as +0.0f).
__device__ __forceinline__ float key_to_float(uint32_t key) {
  return __uint_as_float((key & 0x80000000u) ? (key & 0x7fffffffu) : ~key);
}

// In-LDS bitonic sort, ascending, n a power of two; every thread of the workgroup takes part.
template <typename T>
__device__ __forceinline__ void bitonic_sort_lds(T* a, int n) {
  for (int size = 2; size <= n; size <<= 1) {
    for (int stride = size >> 1; stride > 0; stride >>= 1) {
      __syncthreads();
      for (int i = threadIdx.x; i < (n >> 1); i += blockDim.x) {
        const int pos = 2 * i - (i & (stride - 1));
        const int j = pos + stride;
        const bool up = (pos & size) == 0;
        const T x = a[pos], y = a[j];
        if ((x > y) == up) {
          a[pos] = y;
          a[j] = x;
        }
      }
    }
  }
  __syncthreads();
}

template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xf, 0xf, false);
}

// OR over aligned groups of 8 lanes; every lane of the group gets the result.
__device__ __forceinline__ uint32_t or_reduce8(uint32_t v) {
  v |= dpp_u32<0xB1>(v);   // quad_perm [1,0,3,2]
  v |= dpp_u32<0x4E>(v);   // quad_perm [2,3,0,1]
  v |= dpp_u32<0x141>(v);  // row_half_mirror: lane i <-> 7-i within 8 lanes
  return v;
}

// Inclusive prefix sum over the 64 lanes of a wavefront with DPP moves only: a
// shift-and-add scan inside each row of 16 lanes, then the row totals are passed on
// with row_bcast15 (rows 1 and 3) and row_bcast31 (rows 2 and 3).
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint32_t dpp_zero_fill(uint32_t v) {
  // lanes that receive nothing (shifted in from outside the row, or rows masked off) get 0
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, ROW_MASK, 0xf, false);
}
__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t v) {
  v += dpp_zero_fill<0x111, 0xf>(v);  // row_shr:1
  v += dpp_zero_fill<0x112, 0xf>(v);  // row_shr:2
  v += dpp_zero_fill<0x114, 0xf>(v);  // row_shr:4
  v += dpp_zero_fill<0x118, 0xf>(v);  // row_shr:8
  v += dpp_zero_fill<0x142, 0xa>(v);  // row_bcast15 into rows 1 and 3
  v += dpp_zero_fill<0x143, 0xc>(v);  // row_bcast31 into rows 2 and 3
  return v;
}

// Exclusive prefix sum of v over a 1024-thread workgroup (thread order) and the block
// total.  wave_tot: 16 words of LDS.
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t* wave_tot,
                                                         uint32_t* total) {
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const uint32_t incl = wave_inclusive_scan(v);
  __syncthreads();  // wave_tot may still be read from an earlier call
  if (lane == 63) wave_tot[wv] = incl;
  __syncthreads();
  uint32_t before = 0, tot = 0;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const uint32_t c = wave_tot[i];
    before += i < wv ? c : 0u;
    tot += c;
  }
  *total = tot;
  return before + incl - v;
}

// Scan a histogram of 2048 bins from the top with 1024 threads: the bin d with
// (count in bins above d) < want <= (count in bins >= d).  Thread t owns bins 2t, 2t+1.
// res[0] = d, res[1] = count above d, res[2] = total.  If the total is smaller than
// `want`, res[0] is 0xffffffff.  Callers read res and synchronise before the next call.
__device__ __forceinline__ void find_from_top(const uint32_t* hist, uint32_t want,
                                              uint32_t* wave_tot, uint32_t* res) {
  const int t = threadIdx.x;
  const uint32_t c0 = hist[2 * t], c1 = hist[2 * t + 1];
  if (t == 0) res[0] = 0xffffffffu;  // ordered before the writes below by the scan's barriers
  uint32_t total;
  const uint32_t below = block_exclusive_scan(c0 + c1, wave_tot, &total);
  const uint32_t above1 = total - below - c0 - c1;  // above bin 2t+1
  const uint32_t above0 = above1 + c1;              // above bin 2t
  if (t == 0) res[2] = total;
  if (above1 < want && want <= above1 + c1) {
    res[0] = 2 * t + 1;
    res[1] = above1;
  } else if (above0 < want && want <= above0 + c0) {
    res[0] = 2 * t;
    res[1] = above0;
  }
  __syncthreads();
}

// The same over 4096 bins (two halves).  Returns the bin through *bin (0 if even the
// whole histogram holds fewer than `want`) and the count above it through *above.
__device__ __forceinline__ void find_from_top_4096(const uint32_t* hist, uint32_t want,
                                                   uint32_t* wave_tot, uint32_t* res,
                                                   uint32_t* bin, uint32_t* above) {
  find_from_top(hist + 2048, want, wave_tot, res);
  const uint32_t d = res[0], a = res[1], upper_total = res[2];
  __syncthreads();
  if (d != 0xffffffffu) {
    *bin = 2048 + d;
    *above = a;
    return;
  }
  find_from_top(hist, want - upper_total, wave_tot, res);
  const uint32_t d2 = res[0], a2 = res[1];
  __syncthreads();
  *bin = d2 == 0xffffffffu ? 0u : d2;
  *above = d2 == 0xffffffffu ? 0u : upper_total + a2;
}

}  // namespace dev
}  // namespace lrqk
