// Pieces shared by the one-workgroup-per-head selection kernels (1024 threads): score
// loading, the proxy score of a single row, and the exact selection of a head from its
// materialised scores (the route taken when a candidate estimate turns out unusable).
#pragma once

#include "lrqk_device.h"
#include "lrqk_internal.h"

namespace lrqk {
namespace {

using namespace dev;

constexpr int kT = 1024;  // threads per workgroup
constexpr int kWaves = kT / 64;
constexpr int kIter = kT * 4;  // scores per workgroup iteration (one float4 per lane)
constexpr int kBatch = 8;      // iterations whose loads are issued together
constexpr int kAgeBins = 2048;
constexpr int kSampleStride = 8;

struct Keys4 {
  uint32_t k[4];
  bool ok[4];
};
struct Raw4 {
  float v[4];
};
// Four consecutive scores starting at element e (e % 4 == 0); 0 beyond n.  Rows are
// 16-byte aligned only if l % 4 == 0 (vec_ok).
__device__ __forceinline__ Raw4 load_raw4(const float* __restrict__ s, int e, int n, bool vec_ok) {
  Raw4 r;
  if (vec_ok && e + 3 < n) {
    const float4 x = *reinterpret_cast<const float4*>(s + e);
    r.v[0] = x.x; r.v[1] = x.y; r.v[2] = x.z; r.v[3] = x.w;
  } else {
#pragma unroll
    for (int c = 0; c < 4; ++c) r.v[c] = (e + c < n) ? s[e + c] : 0.0f;
  }
  return r;
}
__device__ __forceinline__ Keys4 keys_of(const Raw4& r, int e, int n) {
  Keys4 q;
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    q.ok[c] = e + c < n;
    q.k[c] = q.ok[c] ? order_key(r.v[c]) : 0u;
  }
  return q;
}

// Proxy score of one row of a head's key factor: the same fused-multiply-add chain (j
// ascending from 0.0f) as the proxy-score kernels, so the bits agree with theirs.
__device__ __forceinline__ float proxy_score_of_row(const float* __restrict__ Arow,
                                                    const float* __restrict__ qh, int r, int row) {
  const float4* __restrict__ a4 = reinterpret_cast<const float4*>(Arow + (size_t)row * r);
  float acc = 0.0f;
  for (int c = 0; c < r / 4; ++c) {
    const float4 a = a4[c];
    acc = __builtin_fmaf(a.x, qh[4 * c + 0], acc);
    acc = __builtin_fmaf(a.y, qh[4 * c + 1], acc);
    acc = __builtin_fmaf(a.z, qh[4 * c + 2], acc);
    acc = __builtin_fmaf(a.w, qh[4 * c + 3], acc);
  }
  return acc;
}

// Exact selection of one head from its n materialised scores s: the k positions with the
// largest keys, equal keys by lower position, written to sel[0..k) in ascending position.
// A complete histogram of the top 12 key bits, two 10-bit refinements of the threshold over
// the scores, one pass that sets a bitmap of the selection (positions with the threshold
// key counted in position order) and a prefix count over the bitmap.
// LDS: hist [kBins], bitmap [(n + 31) / 32], sel [k], wave_tot [kWaves], res [4].
// *bin_of_rank receives the 12-bit key prefix of the bin that holds the `rank`-th largest
// score (0 if the head has fewer scores than that).
// With MAKE_LIST false the function stops at the bitmap of the selection (bit e % 32 of word
// e / 32 for position e; complete for every thread on return) and sel is not touched.
template <bool MAKE_LIST>
__device__ __forceinline__ void exact_select_from_scores(const float* s, int n, int k, bool vec_ok,
                                                         uint32_t rank, uint32_t* hist,
                                                         uint32_t* bitmap, int32_t* sel,
                                                         uint32_t* wave_tot, uint32_t* res,
                                                         uint32_t* bin_of_rank) {
  const int t = threadIdx.x, lane = t & 63;
  const int n_iter = (n + kIter - 1) / kIter;
  const int words = (n + 31) / 32;
  const int wpt = (words + kT - 1) / kT;
  uint32_t bin, above;
  for (int i = t; i < kBins; i += kT) hist[i] = 0u;
  __syncthreads();
  for (int it0 = 0; it0 < n_iter; it0 += kBatch) {
    Raw4 raw[kBatch];
#pragma unroll
    for (int u = 0; u < kBatch; ++u) raw[u] = load_raw4(s, (it0 + u) * kIter + 4 * t, n, vec_ok);
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      const Keys4 q = keys_of(raw[u], (it0 + u) * kIter + 4 * t, n);
#pragma unroll
      for (int c = 0; c < 4; ++c)
        if (q.ok[c]) atomicAdd(&hist[q.k[c] >> kBinShift], 1u);
    }
  }
  __syncthreads();
  {
    uint32_t above_unused;
    find_from_top_4096(hist, rank, wave_tot, res, bin_of_rank, &above_unused);
  }
  find_from_top_4096(hist, (uint32_t)k, wave_tot, res, &bin, &above);
  // refine the threshold inside the bin: two 10-bit levels over the low 20 key bits
  uint32_t prefix = bin, remaining = (uint32_t)k - above;
  int shift = kBinShift;
  for (int level = 0; level < 2; ++level) {
    for (int i = t; i < 2048; i += kT) hist[i] = 0u;
    __syncthreads();
    const int nshift = shift - 10;
    for (int it0 = 0; it0 < n_iter; it0 += kBatch) {
      Raw4 raw[kBatch];
#pragma unroll
      for (int u = 0; u < kBatch; ++u) raw[u] = load_raw4(s, (it0 + u) * kIter + 4 * t, n, vec_ok);
#pragma unroll
      for (int u = 0; u < kBatch; ++u) {
        const Keys4 q = keys_of(raw[u], (it0 + u) * kIter + 4 * t, n);
#pragma unroll
        for (int c = 0; c < 4; ++c)
          if (q.ok[c] && (q.k[c] >> shift) == prefix)
            atomicAdd(&hist[(q.k[c] >> nshift) & 1023u], 1u);
      }
    }
    __syncthreads();
    find_from_top(hist, remaining, wave_tot, res);
    prefix = (prefix << 10) | res[0];
    remaining -= res[1];
    shift = nshift;
    __syncthreads();
  }
  const uint32_t tau = prefix, need_eq = remaining;
  // bitmap of the selection; positions with key == tau are counted in position order
  uint32_t taken = 0;
  for (int it = 0; it < n_iter; ++it) {
    const int e = it * kIter + 4 * t;
    const Keys4 q = keys_of(load_raw4(s, e, n, vec_ok), e, n);
    uint32_t cnt = 0;
#pragma unroll
    for (int c = 0; c < 4; ++c) cnt += (q.ok[c] && q.k[c] == tau) ? 1u : 0u;
    uint32_t tot;
    uint32_t rk = taken + block_exclusive_scan(cnt, wave_tot, &tot);
    uint32_t nib = 0;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      if (!q.ok[c]) continue;
      if (q.k[c] > tau) nib |= 1u << c;
      if (q.k[c] == tau) {
        if (rk < need_eq) nib |= 1u << c;
        ++rk;
      }
    }
    taken += tot;
    const uint32_t word = or_reduce8(nib << (4 * (lane & 7)));
    const int wi = e >> 5;
    if ((lane & 7) == 0 && wi < words) bitmap[wi] = word;
  }
  __syncthreads();
  if (!MAKE_LIST) return;
  uint32_t cnt = 0;
  for (int j = 0; j < wpt; ++j)
    if (t * wpt + j < words) cnt += (uint32_t)__popc(bitmap[t * wpt + j]);
  uint32_t tot;
  uint32_t off = block_exclusive_scan(cnt, wave_tot, &tot);
  for (int j = 0; j < wpt; ++j) {
    if (t * wpt + j >= words) break;
    uint32_t wbits = bitmap[t * wpt + j];
    while (wbits) {
      const int bpos = __ffs((int)wbits) - 1;
      wbits &= wbits - 1;
      if (off < (uint32_t)k) sel[off] = (t * wpt + j) * 32 + bpos;
      ++off;
    }
  }
}

}  // namespace
}  // namespace lrqk
