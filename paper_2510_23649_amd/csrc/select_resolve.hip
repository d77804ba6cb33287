// a2 + a3 in one workgroup per (batch, query head): exact top-k selection over the
// proxy scores followed, optionally, by hit/miss resolution against the cache state
// (Alg. 2, top(., k); Sec. 4.1 active / lite tokens and the hit-and-miss cache).
//
// Everything a head needs fits in the LDS of one CU, so a head is handled without
// any traffic between workgroups.  Selection works on an order-preserving 32-bit
// key of the score (larger score <=> larger key; equal scores: lower position first).
//
//  Selection, usual route (two reads of the head's scores, no sorting):
//   1. a histogram of the top 12 key bits over a 1-in-8 sample of the positions
//      (all positions when the head is small) gives a bin b_lo at or below the bin
//      of the k-th largest score, with a safety margin;
//   2. one pass over all scores marks every position whose bin is >= b_lo in an LDS
//      bitmap (4 positions per lane, 8 lanes OR-ed into one word: no atomics);
//   3. a prefix count over the bitmap turns it into an ascending list of m candidate
//      positions; if k <= m <= capacity the estimate was good (this is checked, not
//      assumed), the candidates' keys are read back and an exact 3-level radix
//      select in LDS finds the key of the k-th largest; candidates above it, and the
//      first ones equal to it in position order, are the selection — already in
//      ascending position.
//  Selection, safe route (taken by a head whose check in step 3 fails: a bad sample
//  or massive ties): full histogram, two 10-bit refinements of the threshold over the
//  scores, one pass that sets the bitmap (positions with the threshold key counted
//  in position order), then the same prefix count.  Slower, same result.
//
//  Resolution: each selected position looks up slot_of (hit: refresh; miss: ranked in
//  position order).  Victims are the least recently selected slots: a histogram of
//  the slots' ages finds the age class that completes the n_miss oldest, the class
//  is cut in slot order, and the victims are ranked among themselves on
//  (last_used, slot) by direct comparison.
//
// All decisions are integer comparisons: the result is exact and independent of
// scheduling.
#include "lrqk_internal.h"

#ifdef LRQK_KPROF
__device__ unsigned long long g_kprof[16];
#define KPROF(i)                                                          \
  do {                                                                    \
    if (blockIdx.x == 0 && threadIdx.x == 0) g_kprof[i] = wall_clock64(); \
  } while (0)
extern "C" __attribute__((visibility("default"))) int lrqk_kprof_read(unsigned long long* out) {
  return (int)hipMemcpyFromSymbol(out, HIP_SYMBOL(g_kprof), sizeof(g_kprof));
}
#else
#define KPROF(i) \
  do {           \
  } while (0)
#endif

namespace lrqk {
namespace {

constexpr int kT = 1024;  // threads per workgroup
constexpr int kWaves = kT / 64;
constexpr int kIter = kT * 4;  // scores per workgroup iteration (one float4 per lane)
constexpr int kBatch = 8;      // iterations whose loads are issued together
constexpr int kAgeBins = 2048;
constexpr int kSampleStride = 8;

__device__ __forceinline__ uint32_t order_key(float s) {
  uint32_t u = __float_as_uint(s);
  if (u == 0x80000000u) u = 0u;  // -0.0f ranks with +0.0f
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xf, 0xf, false);
}
// OR over aligned groups of 8 lanes; every lane of the group gets the result
__device__ __forceinline__ uint32_t or_reduce8(uint32_t v) {
  v |= dpp_u32<0xB1>(v);   // quad_perm [1,0,3,2]
  v |= dpp_u32<0x4E>(v);   // quad_perm [2,3,0,1]
  v |= dpp_u32<0x141>(v);  // row_half_mirror: lane i <-> 7-i within 8 lanes
  return v;
}

__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t v) {
  const int lane = threadIdx.x & 63;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const uint32_t n = __shfl_up(v, d);
    if (lane >= d) v += n;
  }
  return v;
}

// Exclusive prefix sum of v over the kT threads (thread order) and the block total.
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t* wave_tot,
                                                         uint32_t* total) {
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const uint32_t incl = wave_inclusive_scan(v);
  __syncthreads();  // wave_tot may still be read from an earlier call
  if (lane == 63) wave_tot[wv] = incl;
  __syncthreads();
  uint32_t before = 0, tot = 0;
#pragma unroll
  for (int i = 0; i < kWaves; ++i) {
    const uint32_t c = wave_tot[i];
    before += i < wv ? c : 0u;
    tot += c;
  }
  *total = tot;
  return before + incl - v;
}

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

template <typename T>
__device__ __forceinline__ void bitonic_sort_lds(T* a, int n) {
  for (int size = 2; size <= n; size <<= 1) {
    for (int stride = size >> 1; stride > 0; stride >>= 1) {
      __syncthreads();
      for (int i = threadIdx.x; i < (n >> 1); i += kT) {
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

// Scan a histogram of nbins = 2 * kT bins from the top: the bin d with
// (count in bins above d) < want <= (count in bins >= d).  Thread t owns bins 2t, 2t+1.
// Results through res[0] = d, res[1] = count above d, res[2] = total.  If the total is
// smaller than `want`, res[0] stays 0xffffffff.
__device__ __forceinline__ void find_from_top(const uint32_t* hist, uint32_t want,
                                              uint32_t* wave_tot, uint32_t* res) {
  const int t = threadIdx.x;
  const uint32_t c0 = hist[2 * t], c1 = hist[2 * t + 1];
  uint32_t total;
  const uint32_t below = block_exclusive_scan(c0 + c1, wave_tot, &total);
  if (t == 0) {
    res[0] = 0xffffffffu;
    res[2] = total;
  }
  __syncthreads();
  const uint32_t above1 = total - below - c0 - c1;  // above bin 2t+1
  const uint32_t above0 = above1 + c1;              // above bin 2t
  if (above1 < want && want <= above1 + c1) {
    res[0] = 2 * t + 1;
    res[1] = above1;
  } else if (above0 < want && want <= above0 + c0) {
    res[0] = 2 * t;
    res[1] = above0;
  }
  __syncthreads();
}

__host__ __device__ inline int cand_capacity(int k) {
  int c = 2 * k + 2048;
  if (c < 4096) c = 4096;
  if (c > 8192) c = 8192;
  return c;
}

struct ArenaSizes {
  size_t sel_b, words_b, u_bytes, total;
};
__host__ __device__ inline ArenaSizes arena_sizes(int k, int n, int C, bool resolve) {
  ArenaSizes a;
  a.sel_b = ((size_t)k * 4 + 255) / 256 * 256;
  a.words_b = (((size_t)n + 31) / 32 * 4 + 255) / 256 * 256;
  const size_t fast = (size_t)kBins * 4 + a.words_b + (size_t)cand_capacity(k) * 8;
  size_t res = 0;
  if (resolve) {
    int Cpad = 2;
    while (Cpad < C) Cpad <<= 1;
    int kpad = 2;
    while (kpad < k) kpad <<= 1;
    const size_t tail = (size_t)kpad * 12 > (size_t)Cpad * 8 ? (size_t)kpad * 12 : (size_t)Cpad * 8;
    res = ((size_t)C * 4 + 255) / 256 * 256 + (size_t)kAgeBins * 4 + tail;
  }
  a.u_bytes = fast > res ? fast : res;
  a.total = a.sel_b + a.u_bytes;
  return a;
}

template <bool RESOLVE>
__global__ __launch_bounds__(kT) void select_resolve_kernel(
    const float* __restrict__ scores, int l, int n, int k, int32_t* __restrict__ sel_idx,
    // resolution (unused when !RESOLVE)
    int32_t step, int C, int32_t* __restrict__ slot_of, int32_t* __restrict__ token_of,
    int32_t* __restrict__ last_used, int32_t* __restrict__ sel_slot, uint8_t* __restrict__ hit,
    int32_t* __restrict__ miss_tok, int32_t* __restrict__ miss_slot,
    int32_t* __restrict__ n_miss) {
  extern __shared__ __align__(16) unsigned char lds_raw[];
  __shared__ uint32_t wave_tot[kWaves];
  __shared__ uint32_t res[4];
  __shared__ uint32_t sh_nmiss, sh_bad;

  const int bh = blockIdx.x, t = threadIdx.x;
  const int lane = t & 63, wv = t >> 6;
  const ArenaSizes az = arena_sizes(k, n, C, RESOLVE);
  int32_t* const sel = reinterpret_cast<int32_t*>(lds_raw);
  unsigned char* const U = lds_raw + az.sel_b;
  uint32_t* const hist = reinterpret_cast<uint32_t*>(U);
  uint32_t* const bitmap = reinterpret_cast<uint32_t*>(U + (size_t)kBins * 4);
  const int cap = cand_capacity(k);
  int32_t* const clist = reinterpret_cast<int32_t*>(U + (size_t)kBins * 4 + az.words_b);
  uint32_t* const ckey = reinterpret_cast<uint32_t*>(clist + cap);

  const float* __restrict__ s = scores + (size_t)bh * l;
  const bool vec_ok = (l & 3) == 0;
  const int n_iter = (n + kIter - 1) / kIter;
  const int words = (n + 31) / 32;
  const int wpt = (words + kT - 1) / kT;  // bitmap words per thread in the prefix counts

  KPROF(0);
  // ---- 1. sampled histogram -> b_lo ------------------------------------------------------
  const int stride = (n >= 65536 && k >= 512) ? kSampleStride : 1;
  for (int i = t; i < kBins; i += kT) hist[i] = 0u;
  if (t == 0) {
    sh_nmiss = 0u;
    sh_bad = 0u;
  }
  __syncthreads();
  if (stride == 1) {
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
  } else {
    // wavefront wv samples its 256-position chunk of iterations it = (wv & 7) + 8 j
    for (int it0 = (wv & 7); it0 < n_iter; it0 += kSampleStride * kBatch) {
      Raw4 raw[kBatch];
#pragma unroll
      for (int u = 0; u < kBatch; ++u)
        raw[u] = load_raw4(s, (it0 + u * kSampleStride) * kIter + 4 * t, n, vec_ok);
#pragma unroll
      for (int u = 0; u < kBatch; ++u) {
        const Keys4 q = keys_of(raw[u], (it0 + u * kSampleStride) * kIter + 4 * t, n);
#pragma unroll
        for (int c = 0; c < 4; ++c)
          if (q.ok[c]) atomicAdd(&hist[q.k[c] >> kBinShift], 1u);
      }
    }
  }
  __syncthreads();
  uint32_t b_lo;
  {
    const uint32_t ks = (uint32_t)(k + stride - 1) / stride;
    const uint32_t want = stride == 1 ? (uint32_t)k : ks + (ks * 3) / 8 + 16;
    // 4096 bins = 2 halves of 2048: scan the upper half first, then the lower one
    find_from_top(hist + 2048, want, wave_tot, res);
    uint32_t d = res[0];
    const uint32_t upper_total = res[2];
    __syncthreads();
    if (d != 0xffffffffu) {
      b_lo = 2048 + d;
    } else {
      find_from_top(hist, want - upper_total, wave_tot, res);
      d = res[0];
      b_lo = d == 0xffffffffu ? 0u : d;
      __syncthreads();
    }
  }

  KPROF(1);
  // ---- 2. bitmap of the positions with bin >= b_lo ----------------------------------------
  for (int it0 = 0; it0 < n_iter; it0 += kBatch) {
    Raw4 raw[kBatch];
#pragma unroll
    for (int u = 0; u < kBatch; ++u) raw[u] = load_raw4(s, (it0 + u) * kIter + 4 * t, n, vec_ok);
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      const int e = (it0 + u) * kIter + 4 * t;
      const Keys4 q = keys_of(raw[u], e, n);
      uint32_t nib = 0;
#pragma unroll
      for (int c = 0; c < 4; ++c)
        if (q.ok[c] && (q.k[c] >> kBinShift) >= b_lo) nib |= 1u << c;
      const uint32_t word = or_reduce8(nib << (4 * (lane & 7)));
      const int wi = e >> 5;
      if ((lane & 7) == 0 && wi < words) bitmap[wi] = word;
    }
  }
  __syncthreads();

  KPROF(2);
  // ---- 3. candidates -> exact selection -----------------------------------------------------
  uint32_t m;
  {
    uint32_t cnt = 0;
    for (int j = 0; j < wpt; ++j)
      if (t * wpt + j < words) cnt += (uint32_t)__popc(bitmap[t * wpt + j]);
    uint32_t off = block_exclusive_scan(cnt, wave_tot, &m);
    if (m >= (uint32_t)k && m <= (uint32_t)cap) {
      for (int j = 0; j < wpt; ++j) {
        if (t * wpt + j >= words) break;
        uint32_t wbits = bitmap[t * wpt + j];
        while (wbits) {
          const int bpos = __ffs((int)wbits) - 1;
          wbits &= wbits - 1;
          clist[off++] = (t * wpt + j) * 32 + bpos;
        }
      }
    }
  }
  __syncthreads();
  if (m >= (uint32_t)k && m <= (uint32_t)cap) {
    for (uint32_t i = t; i < m; i += kT) ckey[i] = order_key(s[clist[i]]);
    // exact key of the k-th largest candidate: digits [31:21], [20:10], [9:0]
    uint32_t prefix = 0, remaining = (uint32_t)k;
#pragma unroll
    for (int level = 0; level < 3; ++level) {
      const int shift = level == 0 ? 21 : (level == 1 ? 10 : 0);
      const int bits = level == 2 ? 10 : 11;
      const int known = shift + bits;  // key >> known must equal prefix
      for (int i = t; i < 2048; i += kT) hist[i] = 0u;
      __syncthreads();
      for (uint32_t i = t; i < m; i += kT) {
        const uint32_t key = ckey[i];
        if (level == 0 || (key >> known) == prefix)
          atomicAdd(&hist[(key >> shift) & ((1u << bits) - 1u)], 1u);
      }
      __syncthreads();
      find_from_top(hist, remaining, wave_tot, res);
      prefix = (prefix << bits) | res[0];
      remaining -= res[1];
      __syncthreads();
    }
    const uint32_t tau = prefix, need_eq = remaining;
    // candidates are in ascending position: take key > tau, and the first need_eq with key == tau
    const uint32_t per = (m + kT - 1) / kT;
    const uint32_t i0 = min(m, (uint32_t)t * per), i1 = min(m, i0 + per);
    uint32_t neq = 0;
    for (uint32_t i = i0; i < i1; ++i) neq += ckey[i] == tau ? 1u : 0u;
    uint32_t tot;
    uint32_t eq_rank = block_exclusive_scan(neq, wave_tot, &tot);
    uint32_t nsel = 0;
    uint32_t flags = 0;  // per <= 8
    for (uint32_t i = i0; i < i1; ++i) {
      const uint32_t key = ckey[i];
      bool take = key > tau;
      if (key == tau) {
        take = eq_rank < need_eq;
        ++eq_rank;
      }
      if (take) {
        flags |= 1u << (i - i0);
        ++nsel;
      }
    }
    uint32_t pos = block_exclusive_scan(nsel, wave_tot, &tot);
    for (uint32_t i = i0; i < i1; ++i)
      if (flags & (1u << (i - i0))) {
        if (pos < (uint32_t)k) sel[pos] = clist[i];
        ++pos;
      }
  } else {
    // ---- safe route --------------------------------------------------------------------------
    uint32_t bin, above;
    // complete histogram
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
    find_from_top(hist + 2048, (uint32_t)k, wave_tot, res);
    {
      const uint32_t d = res[0], a = res[1], upper_total = res[2];
      __syncthreads();
      if (d != 0xffffffffu) {
        bin = 2048 + d;
        above = a;
      } else {
        find_from_top(hist, (uint32_t)k - upper_total, wave_tot, res);
        bin = res[0];
        above = upper_total + res[1];
        __syncthreads();
      }
    }
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
        for (int u = 0; u < kBatch; ++u)
          raw[u] = load_raw4(s, (it0 + u) * kIter + 4 * t, n, vec_ok);
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
      uint32_t rank = taken + block_exclusive_scan(cnt, wave_tot, &tot);
      uint32_t nib = 0;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        if (!q.ok[c]) continue;
        if (q.k[c] > tau) nib |= 1u << c;
        if (q.k[c] == tau) {
          if (rank < need_eq) nib |= 1u << c;
          ++rank;
        }
      }
      taken += tot;
      const uint32_t word = or_reduce8(nib << (4 * (lane & 7)));
      const int wi = e >> 5;
      if ((lane & 7) == 0 && wi < words) bitmap[wi] = word;
    }
    __syncthreads();
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
  __syncthreads();
  KPROF(3);
  for (int i = t; i < k; i += kT) sel_idx[(size_t)bh * k + i] = sel[i];
  if (!RESOLVE) return;

  // ---- resolution ------------------------------------------------------------------------------
  int32_t* __restrict__ so = slot_of + (size_t)bh * l;
  int32_t* __restrict__ to = token_of + (size_t)bh * C;
  int32_t* __restrict__ lu = last_used + (size_t)bh * C;
  int32_t* __restrict__ ss = sel_slot + (size_t)bh * k;
  uint8_t* __restrict__ ht = hit + (size_t)bh * k;
  int32_t* __restrict__ mt = miss_tok + (size_t)bh * k;
  int32_t* __restrict__ ms = miss_slot + (size_t)bh * k;
  int32_t* const lu_s = reinterpret_cast<int32_t*>(U);  // [C] last_used, then `step` where used now
  const size_t lu_b = ((size_t)C * 4 + 255) / 256 * 256;
  uint32_t* const ahist = reinterpret_cast<uint32_t*>(U + lu_b);                 // [kAgeBins]
  uint64_t* const vlist = reinterpret_cast<uint64_t*>(U + lu_b + kAgeBins * 4);  // victims' keys
  int kpad = 2;
  while (kpad < k) kpad <<= 1;
  int32_t* const vsorted = reinterpret_cast<int32_t*>(vlist + kpad);  // [k] victims in rank order

  __syncthreads();  // the selection buffers are dead from here on
  for (int i = t; i < C; i += kT) lu_s[i] = lu[i];
  for (int i = t; i < kAgeBins; i += kT) ahist[i] = 0u;
  __syncthreads();
  for (int j0 = 0; j0 < k; j0 += kT) {
    const int j = j0 + t;
    int32_t tok = -1, slot = -1;
    bool miss = false;
    if (j < k) {
      tok = sel[j];
      slot = so[tok];
      if (slot >= C) slot = -1;  // corrupt map entry: treat as absent
      miss = slot < 0;
      if (!miss) {
        ss[j] = slot;
        ht[j] = 1;
        lu[slot] = step;
        lu_s[slot] = step;  // used in this step: never a victim
      } else {
        ht[j] = 0;
      }
    }
    uint32_t tot;
    const uint32_t rank = sh_nmiss + block_exclusive_scan(miss ? 1u : 0u, wave_tot, &tot);
    if (miss) {
      mt[rank] = tok;
      sel[j] = -(int32_t)rank - 2;  // remember the rank; the slot is filled in below
    }
    __syncthreads();
    if (t == 0) sh_nmiss += tot;
    __syncthreads();
  }
  const int nm = (int)sh_nmiss;
  KPROF(4);
  if (nm > 0) {
    // ages of the slots not used in this step; thread t owns slots [t*spt, (t+1)*spt)
    const int spt = (C + kT - 1) / kT;
    const int s0 = min(C, t * spt), s1 = min(C, s0 + spt);
    for (int v = s0; v < s1; ++v) {
      const int32_t u = lu_s[v];
      if (u != step) atomicAdd(&ahist[min((uint32_t)(step - 1 - u), (uint32_t)(kAgeBins - 1))], 1u);
    }
    __syncthreads();
    find_from_top(ahist, (uint32_t)nm, wave_tot, res);
    const uint32_t Ta = res[0], c_older = res[1], n_elig = res[2];
    __syncthreads();
    const bool clipped = (Ta == (uint32_t)(kAgeBins - 1)) && step > kAgeBins - 1;
    int nv;  // number of victims found (< nm only if the caller reused `step`)
    const uint64_t* sorted64 = nullptr;
    if (Ta != 0xffffffffu && !clipped) {
      const uint32_t need_cls = (uint32_t)nm - c_older;
      uint32_t ncls = 0;
      for (int v = s0; v < s1; ++v) {
        const int32_t u = lu_s[v];
        if (u != step && min((uint32_t)(step - 1 - u), (uint32_t)(kAgeBins - 1)) == Ta) ++ncls;
      }
      uint32_t tot;
      uint32_t cls_rank = block_exclusive_scan(ncls, wave_tot, &tot);
      uint32_t ntake = 0, flags = 0;  // spt <= 8
      for (int v = s0; v < s1; ++v) {
        const int32_t u = lu_s[v];
        if (u == step) continue;
        const uint32_t a = min((uint32_t)(step - 1 - u), (uint32_t)(kAgeBins - 1));
        bool take = a > Ta;
        if (a == Ta) {
          take = cls_rank < need_cls;
          ++cls_rank;
        }
        if (take) {
          flags |= 1u << (v - s0);
          ++ntake;
        }
      }
      uint32_t pos = block_exclusive_scan(ntake, wave_tot, &tot);
      nv = (int)tot;
      for (int v = s0; v < s1; ++v)
        if (flags & (1u << (v - s0)))
          vlist[pos++] = (((uint64_t)(uint32_t)(lu_s[v] + 1)) << 32) | (uint32_t)v;
      __syncthreads();
      if (nv <= kT) {
        // rank every victim among the victims by direct comparison
        if (t < nv) {
          const uint64_t mine = vlist[t];
          int r = 0;
          for (int u = 0; u < nv; ++u) r += vlist[u] < mine ? 1 : 0;
          vsorted[r] = (int32_t)(uint32_t)mine;
        }
        __syncthreads();
      } else {
        int vpad = 2;
        while (vpad < nv) vpad <<= 1;
        for (int i = nv + t; i < vpad; i += kT) vlist[i] = ~0ull;
        bitonic_sort_lds(vlist, vpad);
        sorted64 = vlist;
      }
    } else {
      // out of victims, or ages beyond the histogram's range: sort every slot's key
      int Cpad = 2;
      while (Cpad < C) Cpad <<= 1;
      for (int v = t; v < Cpad; v += kT) {
        uint64_t key = ~0ull;
        if (v < C && lu_s[v] != step) key = (((uint64_t)(uint32_t)(lu_s[v] + 1)) << 32) | (uint32_t)v;
        vlist[v] = key;
      }
      bitonic_sort_lds(vlist, Cpad);
      nv = (int)min((uint32_t)nm, n_elig);
      sorted64 = vlist;
    }
    for (int j = t; j < nm; j += kT) {
      if (j >= nv) {  // ran out of victims (the caller reused `step`)
        atomicOr(&sh_bad, 1u);
        ms[j] = -1;
        continue;
      }
      const int32_t v = sorted64 ? (int32_t)(uint32_t)sorted64[j] : vsorted[j];
      const int32_t tok = mt[j];
      const int32_t old = to[v];
      if (old >= 0 && old < l) so[old] = -1;
      to[v] = tok;
      so[tok] = v;
      lu[v] = step;
      ms[j] = v;
    }
    __syncthreads();
    for (int j = t; j < k; j += kT) {
      const int32_t v = sel[j];
      if (v <= -2) ss[j] = ms[-(v + 2)];
    }
  }
  __syncthreads();
  KPROF(5);
  if (t == 0) n_miss[bh] = sh_bad ? -1 : nm;
}

constexpr size_t kLdsLimit = 150 * 1024;

template <bool RESOLVE>
hipError_t raise_lds_limit() {
  static bool done = false;
  if (done) return hipSuccess;
  const hipError_t e = hipFuncSetAttribute(
      reinterpret_cast<const void*>(select_resolve_kernel<RESOLVE>),
      hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsLimit);
  if (e == hipSuccess) done = true;
  return e;
}

}  // namespace

bool select_resolve_fits(const lrqk_shape& s, bool resolve) {
  // per-thread bit flags in the kernel hold up to 8 candidates / 8 slots per thread
  if (cand_capacity(s.k) > 8 * kT || s.C > 8 * kT) return false;
  return arena_sizes(s.k, s.l - s.w, s.C, resolve).total <= kLdsLimit;
}

hipError_t launch_select_only(const lrqk_shape& s, const float* scores, int32_t* sel_idx,
                              hipStream_t st) {
  const int n = s.l - s.w;
  const size_t lds = arena_sizes(s.k, n, s.C, false).total;
  hipError_t e = raise_lds_limit<false>();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((select_resolve_kernel<false>), dim3(s.B * s.Hq), dim3(kT), lds, st, scores,
                     s.l, n, s.k, sel_idx, 0, s.C, nullptr, nullptr, nullptr, nullptr, nullptr,
                     nullptr, nullptr, nullptr);
  return hipGetLastError();
}

hipError_t launch_select_resolve(const lrqk_shape& s, const float* scores, int32_t* sel_idx,
                                 int32_t step, int32_t* slot_of, int32_t* token_of,
                                 int32_t* last_used, int32_t* sel_slot, uint8_t* hit,
                                 int32_t* miss_tok, int32_t* miss_slot, int32_t* n_miss,
                                 hipStream_t st) {
  const int n = s.l - s.w;
  const size_t lds = arena_sizes(s.k, n, s.C, true).total;
  hipError_t e = raise_lds_limit<true>();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((select_resolve_kernel<true>), dim3(s.B * s.Hq), dim3(kT), lds, st, scores,
                     s.l, n, s.k, sel_idx, step, s.C, slot_of, token_of, last_used, sel_slot, hit,
                     miss_tok, miss_slot, n_miss);
  return hipGetLastError();
}

}  // namespace lrqk
