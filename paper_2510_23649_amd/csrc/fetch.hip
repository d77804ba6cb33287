// a4 — fetch the missing K/V rows from the host store into their cache slots
// (Alg. 2: "Fetch missing k_i, v_i from CPU K, V" and "merge").  Byte copies.
//
// Two ways to move the rows:
//   direct  one kernel gathers rows straight out of pinned (device-visible) host
//           memory over the host link and writes them into the slots: 16 lanes per
//           row, 16 bytes per lane per load, K and V of a row by the same lanes;
//   staged  the host has packed the rows into a pinned staging buffer and copied
//           it with one hipMemcpyAsync; this kernel scatters the device copy into
//           the slots.
#include "lrqk_internal.h"

namespace lrqk {
namespace {

constexpr int kFetchThreads = 256;

// grid: (ceil(k / rows_per_block), BHq); rows_per_block = 16 rows per pass x passes
template <int ROW16>  // 16-byte units per row: 16 (bf16) or 32 (fp32)
__global__ __launch_bounds__(kFetchThreads) void fetch_direct_kernel(
    const uint4* __restrict__ K_host, const uint4* __restrict__ V_host,
    const int32_t* __restrict__ miss_tok, const int32_t* __restrict__ miss_slot,
    const int32_t* __restrict__ n_miss, uint4* __restrict__ cacheK, uint4* __restrict__ cacheV,
    int Hq, int Hkv, int l, int lrows, int C, int k, int rows_per_block) {
  const int bh = blockIdx.y;
  const int b = bh / Hq, h = bh - b * Hq;
  const int kvh = h / (Hq / Hkv);
  const int nm = min(n_miss[bh], k);
  const int row_begin = blockIdx.x * rows_per_block;
  const int row_end = min(nm, row_begin + rows_per_block);
  const int t = threadIdx.x, sub = t & 15, rgrp = t >> 4;  // 16 row groups per workgroup
  const uint4* __restrict__ Ks = K_host + ((size_t)b * Hkv + kvh) * (size_t)lrows * ROW16;
  const uint4* __restrict__ Vs = V_host + ((size_t)b * Hkv + kvh) * (size_t)lrows * ROW16;
  uint4* __restrict__ Kc = cacheK + (size_t)bh * C * ROW16;
  uint4* __restrict__ Vc = cacheV + (size_t)bh * C * ROW16;
  for (int j = row_begin + rgrp; j < row_end; j += 16) {
    const int32_t tok = miss_tok[(size_t)bh * k + j];
    const int32_t s = miss_slot[(size_t)bh * k + j];
    if (tok < 0 || tok >= l || s < 0 || s >= C) continue;
#pragma unroll
    for (int c = sub; c < ROW16; c += 16) {
      const uint4 kx = Ks[(size_t)tok * ROW16 + c];
      const uint4 vx = Vs[(size_t)tok * ROW16 + c];
      Kc[(size_t)s * ROW16 + c] = kx;
      Vc[(size_t)s * ROW16 + c] = vx;
    }
  }
}

// staging: n_rows x [K row | V row]; row_dst[i] = bh * C + slot
template <int ROW16>
__global__ __launch_bounds__(kFetchThreads) void scatter_staged_kernel(
    const uint4* __restrict__ staging, const int64_t* __restrict__ row_dst, int64_t n_rows,
    uint4* __restrict__ cacheK, uint4* __restrict__ cacheV) {
  const int t = threadIdx.x, sub = t & 15, rgrp = t >> 4;
  for (int64_t i = (int64_t)blockIdx.x * 16 + rgrp; i < n_rows; i += (int64_t)gridDim.x * 16) {
    const int64_t dst = row_dst[i];
    if (dst < 0) continue;
#pragma unroll
    for (int c = sub; c < ROW16; c += 16) {
      cacheK[(size_t)dst * ROW16 + c] = staging[(size_t)i * 2 * ROW16 + c];
      cacheV[(size_t)dst * ROW16 + c] = staging[(size_t)i * 2 * ROW16 + ROW16 + c];
    }
  }
}

}  // namespace

hipError_t launch_fetch_direct(const lrqk_shape& s, const void* K_host, const void* V_host,
                               const int32_t* miss_tok, const int32_t* miss_slot,
                               const int32_t* n_miss, void* cacheK, void* cacheV, hipStream_t st) {
  const int rows_per_block = 64;
  const dim3 grid(ceil_div(s.k, rows_per_block), s.B * s.Hq);
  if (s.kv_dtype == LRQK_KV_BF16)
    LRQK_LAUNCH((fetch_direct_kernel<16>), grid, dim3(kFetchThreads), 0, st,
                       (const uint4*)K_host, (const uint4*)V_host, miss_tok, miss_slot, n_miss,
                       (uint4*)cacheK, (uint4*)cacheV, s.Hq, s.Hkv, s.l, row_cap(s), s.C, s.k,
                       rows_per_block);
  else
    LRQK_LAUNCH((fetch_direct_kernel<32>), grid, dim3(kFetchThreads), 0, st,
                       (const uint4*)K_host, (const uint4*)V_host, miss_tok, miss_slot, n_miss,
                       (uint4*)cacheK, (uint4*)cacheV, s.Hq, s.Hkv, s.l, row_cap(s), s.C, s.k,
                       rows_per_block);
  return hipGetLastError();
}

hipError_t launch_scatter_staged(const lrqk_shape& s, const void* staging, const int64_t* row_dst,
                                 int64_t n_rows, void* cacheK, void* cacheV, hipStream_t st) {
  if (n_rows <= 0) return hipSuccess;
  int64_t nb = (n_rows + 15) / 16;
  if (nb > 4096) nb = 4096;
  if (s.kv_dtype == LRQK_KV_BF16)
    LRQK_LAUNCH((scatter_staged_kernel<16>), dim3((unsigned)nb), dim3(kFetchThreads), 0, st,
                       (const uint4*)staging, row_dst, n_rows, (uint4*)cacheK, (uint4*)cacheV);
  else
    LRQK_LAUNCH((scatter_staged_kernel<32>), dim3((unsigned)nb), dim3(kFetchThreads), 0, st,
                       (const uint4*)staging, row_dst, n_rows, (uint4*)cacheK, (uint4*)cacheV);
  return hipGetLastError();
}

}  // namespace lrqk
