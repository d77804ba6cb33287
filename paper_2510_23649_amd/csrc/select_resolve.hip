// a2 + a3 in one workgroup per (batch, query head): exact top-k selection over the
// proxy scores followed, optionally, by hit/miss resolution against the cache state
// (Alg. 2, top(., k); Sec. 4.1 active / lite tokens and the hit-and-miss cache).
//
// Everything a head needs fits in the 160 KB of LDS of one CU, so the whole
// selection runs without any traffic between workgroups:
//   1. one pass over the head's scores builds a 4096-bin histogram of the top 12
//      bits of an order-preserving key in LDS; a scan from the top finds the bin
//      that holds the k-th largest score;
//   2. a second pass (the scores are L2-resident by now) marks every position of a
//      higher bin in an LDS bitmap of l bits and collects the positions of the
//      threshold bin as (key, position) candidates;
//   3. the candidates are sorted (key descending, position ascending) and the ones
//      still needed get their bits set; if there are more candidates than the
//      buffer holds (massive ties) the threshold is refined over the remaining 20
//      key bits from the scores instead;
//   4. a prefix count over the bitmap emits the k positions in ascending order;
//   5. (resolution) each selected position looks up slot_of; misses are ranked in
//      position order, the slots not used in this step are sorted by
//      (last_used, slot) and handed out in that order.
// All decisions are integer comparisons on keys: the result is exact and does not
// depend on scheduling.
#include "lrqk_internal.h"

#ifdef LRQK_KPROF
__device__ unsigned long long g_kprof[16];
#define KPROF(i)                                                     \
  do {                                                               \
    if (blockIdx.x == 0 && threadIdx.x == 0) g_kprof[i] = wall_clock64(); \
  } while (0)
extern "C" __attribute__((visibility("default"))) int lrqk_kprof_read(unsigned long long* out) {
  return (int)hipMemcpyFromSymbol(out, HIP_SYMBOL(g_kprof), sizeof(g_kprof));
}
#else
#define KPROF(i) do {} while (0)
#endif

namespace lrqk {
namespace {

constexpr int kT = 1024;           // threads per workgroup
constexpr int kWaves = kT / 64;
constexpr int kIter = kT * 4;      // scores per workgroup iteration (one float4 per lane)

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

// Four consecutive scores starting at element e (e % 4 == 0) as order keys; elements
// at or beyond n get valid = false.  Rows are 16-byte aligned only if l % 4 == 0.
struct Keys4 {
  uint32_t k[4];
  bool ok[4];
};
__device__ __forceinline__ Keys4 load_keys4(const float* __restrict__ s, int e, int n,
                                            bool vec_ok) {
  Keys4 r;
  if (vec_ok && e + 3 < n) {
    const float4 v = *reinterpret_cast<const float4*>(s + e);
    r.k[0] = order_key(v.x); r.k[1] = order_key(v.y);
    r.k[2] = order_key(v.z); r.k[3] = order_key(v.w);
    r.ok[0] = r.ok[1] = r.ok[2] = r.ok[3] = true;
  } else {
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      r.ok[c] = e + c < n;
      r.k[c] = r.ok[c] ? order_key(s[e + c]) : 0u;
    }
  }
  return r;
}

// Raw scores of kBatch consecutive workgroup iterations, all loads issued before any use,
// so one workgroup keeps kBatch * 16 KB in flight.
constexpr int kBatch = 8;
struct Raw4 {
  float v[4];
};
__device__ __forceinline__ void load_batch(const float* __restrict__ s, int it0, int n_iter,
                                           int t, int n, bool vec_ok, Raw4 (&raw)[kBatch]) {
#pragma unroll
  for (int u = 0; u < kBatch; ++u) {
    const int e = (it0 + u) * kIter + 4 * t;
    if (it0 + u < n_iter && vec_ok && e + 3 < n) {
      const float4 x = *reinterpret_cast<const float4*>(s + e);
      raw[u].v[0] = x.x; raw[u].v[1] = x.y; raw[u].v[2] = x.z; raw[u].v[3] = x.w;
    } else {
#pragma unroll
      for (int c = 0; c < 4; ++c)
        raw[u].v[c] = (it0 + u < n_iter && e + c < n) ? s[e + c] : 0.0f;
    }
  }
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

struct Arena {
  int32_t* sel;       // [k]           selected positions, ascending (lives through both phases)
  uint32_t* hist;     // [kBins]       phase a2
  uint64_t* cand;     // [kCandCap]    phase a2
  uint32_t* bitmap;   // [words]       phase a2
  uint64_t* vkeys;    // [Cpad]        phase a3 (aliases hist/cand/bitmap)
};

__host__ __device__ inline size_t arena_bytes(int k, int n, int Cpad, bool resolve) {
  const size_t sel = ((size_t)k * 4 + 255) / 256 * 256;
  const size_t words = ((size_t)n + 31) / 32;
  const size_t a = (size_t)kBins * 4 + (size_t)kCandCap * 8 + (words * 4 + 255) / 256 * 256;
  const size_t b = resolve ? (size_t)Cpad * 8 : 0;
  return sel + (a > b ? a : b);
}

template <bool RESOLVE>
__global__ __launch_bounds__(kT) void select_resolve_kernel(
    const float* __restrict__ scores, int l, int n, int k, int32_t* __restrict__ sel_idx,
    // resolution (unused when !RESOLVE)
    int32_t step, int C, int Cpad, int32_t* __restrict__ slot_of, int32_t* __restrict__ token_of,
    int32_t* __restrict__ last_used, int32_t* __restrict__ sel_slot, uint8_t* __restrict__ hit,
    int32_t* __restrict__ miss_tok, int32_t* __restrict__ miss_slot,
    int32_t* __restrict__ n_miss) {
  extern __shared__ __align__(16) unsigned char lds_raw[];
  __shared__ uint32_t wave_tot[kWaves];
  __shared__ uint32_t sh_bin, sh_above, sh_ncand, sh_a, sh_b, sh_nmiss, sh_bad;

  const int bh = blockIdx.x, t = threadIdx.x;
  const int lane = t & 63;
  Arena A;
  {
    const size_t sel_b = ((size_t)k * 4 + 255) / 256 * 256;
    A.sel = reinterpret_cast<int32_t*>(lds_raw);
    A.hist = reinterpret_cast<uint32_t*>(lds_raw + sel_b);
    A.cand = reinterpret_cast<uint64_t*>(lds_raw + sel_b + (size_t)kBins * 4);
    A.bitmap = reinterpret_cast<uint32_t*>(lds_raw + sel_b + (size_t)kBins * 4 +
                                           (size_t)kCandCap * 8);
    A.vkeys = reinterpret_cast<uint64_t*>(lds_raw + sel_b);
  }
  const float* __restrict__ s = scores + (size_t)bh * l;
  const bool vec_ok = (l & 3) == 0;
  const int n_iter = (n + kIter - 1) / kIter;
  const int words = (n + 31) / 32;

  KPROF(0);
  // ---- 1. histogram of the top 12 key bits -------------------------------------------
  for (int i = t; i < kBins; i += kT) A.hist[i] = 0u;
  if (t == 0) {
    sh_ncand = 0u;
    sh_nmiss = 0u;
    sh_bad = 0u;
  }
  __syncthreads();
  for (int it0 = 0; it0 < n_iter; it0 += kBatch) {
    Raw4 raw[kBatch];
    load_batch(s, it0, n_iter, t, n, vec_ok, raw);
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      const Keys4 q = keys_of(raw[u], (it0 + u) * kIter + 4 * t, n);
#pragma unroll
      for (int c = 0; c < 4; ++c)
        if (q.ok[c]) atomicAdd(&A.hist[q.k[c] >> kBinShift], 1u);
    }
  }
  __syncthreads();
  KPROF(1);
  {
    // thread t owns bins [4t, 4t+4); count of scores in bins above them, then walk down
    uint32_t loc[4], sum = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      loc[j] = A.hist[4 * t + j];
      sum += loc[j];
    }
    uint32_t total;
    const uint32_t below = block_exclusive_scan(sum, wave_tot, &total);
    uint32_t running = total - below - sum;
#pragma unroll
    for (int j = 3; j >= 0; --j) {
      const uint32_t before = running;
      running += loc[j];
      if (running >= (uint32_t)k && before < (uint32_t)k) {
        sh_bin = (uint32_t)(4 * t + j);
        sh_above = before;
      }
    }
  }
  __syncthreads();
  const uint32_t bin = sh_bin;
  const int need = k - (int)sh_above;  // taken from the threshold bin, >= 1

  KPROF(2);
  // ---- 2. bitmap of the certain members, candidates of the threshold bin --------------
  for (int it0 = 0; it0 < n_iter; it0 += kBatch) {
    Raw4 raw[kBatch];
    load_batch(s, it0, n_iter, t, n, vec_ok, raw);
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      const int e = (it0 + u) * kIter + 4 * t;
      const Keys4 q = keys_of(raw[u], e, n);
      uint32_t nib = 0;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        if (!q.ok[c]) continue;
        const uint32_t b = q.k[c] >> kBinShift;
        if (b > bin) {
          nib |= 1u << c;
        } else if (b == bin) {
          const uint32_t p = atomicAdd(&sh_ncand, 1u);
          if (p < (uint32_t)kCandCap)
            A.cand[p] = ((uint64_t)(~q.k[c]) << 32) | (uint32_t)(e + c);
        }
      }
      const uint32_t word = or_reduce8(nib << (4 * (lane & 7)));
      const int wi = (e >> 5);
      if ((lane & 7) == 0 && wi < words) A.bitmap[wi] = word;
    }
  }
  __syncthreads();
  const int n_cand = (int)sh_ncand;

  KPROF(3);
  // ---- 3. the members that come from the threshold bin --------------------------------
  if (n_cand <= kCandCap) {
    int cpad = 2;
    while (cpad < n_cand) cpad <<= 1;
    for (int i = n_cand + t; i < cpad; i += kT) A.cand[i] = ~0ull;
    bitonic_sort_lds(A.cand, cpad);
    for (int i = t; i < need; i += kT) {
      const uint32_t pos = (uint32_t)A.cand[i];
      atomicOr(&A.bitmap[pos >> 5], 1u << (pos & 31));
    }
  } else {
    // refine the threshold inside the bin: two 10-bit levels over the low 20 key bits
    uint32_t prefix = bin;
    int shift = kBinShift;
    uint32_t remaining = (uint32_t)need;
    for (int level = 0; level < 2; ++level) {
      for (int i = t; i < 1024; i += kT) A.hist[i] = 0u;
      __syncthreads();
      const int nshift = shift - 10;
      for (int it = 0; it < n_iter; ++it) {
        const Keys4 q = load_keys4(s, it * kIter + 4 * t, n, vec_ok);
#pragma unroll
        for (int c = 0; c < 4; ++c)
          if (q.ok[c] && (q.k[c] >> shift) == prefix)
            atomicAdd(&A.hist[(q.k[c] >> nshift) & 1023u], 1u);
      }
      __syncthreads();
      {
        const uint32_t mine = A.hist[t];  // kT == 1024 bins
        uint32_t total;
        const uint32_t below = block_exclusive_scan(mine, wave_tot, &total);
        const uint32_t above = total - below - mine;
        if (above + mine >= remaining && above < remaining) {
          sh_a = (uint32_t)t;
          sh_b = remaining - above;
        }
      }
      __syncthreads();
      prefix = (prefix << 10) | sh_a;
      remaining = sh_b;
      shift = nshift;
      __syncthreads();
    }
    const uint32_t tau = prefix;          // exact key of the k-th largest score
    const uint32_t need_eq = remaining;   // positions with key == tau taken, lowest first
    uint32_t taken = 0;
    for (int it = 0; it < n_iter; ++it) {
      const int e = it * kIter + 4 * t;
      const Keys4 q = load_keys4(s, e, n, vec_ok);
      uint32_t eqmask = 0, cnt = 0;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        if (!q.ok[c] || (q.k[c] >> kBinShift) != bin) continue;
        if (q.k[c] > tau) atomicOr(&A.bitmap[(e + c) >> 5], 1u << ((e + c) & 31));
        if (q.k[c] == tau) {
          eqmask |= 1u << c;
          ++cnt;
        }
      }
      uint32_t total;
      uint32_t rank = taken + block_exclusive_scan(cnt, wave_tot, &total);
#pragma unroll
      for (int c = 0; c < 4; ++c)
        if (eqmask & (1u << c)) {
          if (rank < need_eq) atomicOr(&A.bitmap[(e + c) >> 5], 1u << ((e + c) & 31));
          ++rank;
        }
      taken += total;  // uniform over the workgroup
    }
  }
  __syncthreads();

  KPROF(4);
  // ---- 4. emit the k set bits in ascending position -----------------------------------
  {
    const int wpt = (words + kT - 1) / kT;
    const int w0 = t * wpt;
    uint32_t cnt = 0;
    for (int j = 0; j < wpt; ++j)
      if (w0 + j < words) cnt += (uint32_t)__popc(A.bitmap[w0 + j]);
    uint32_t total;
    uint32_t off = block_exclusive_scan(cnt, wave_tot, &total);
    for (int j = 0; j < wpt; ++j) {
      if (w0 + j >= words) break;
      uint32_t wbits = A.bitmap[w0 + j];
      while (wbits) {
        const int bpos = __ffs((int)wbits) - 1;
        wbits &= wbits - 1;
        if (off < (uint32_t)k) A.sel[off] = (w0 + j) * 32 + bpos;
        ++off;
      }
    }
  }
  __syncthreads();
  for (int i = t; i < k; i += kT) sel_idx[(size_t)bh * k + i] = A.sel[i];
  KPROF(5);
  if (!RESOLVE) return;

  // ---- 5. hit/miss resolution -----------------------------------------------------------
  int32_t* __restrict__ so = slot_of + (size_t)bh * l;
  int32_t* __restrict__ to = token_of + (size_t)bh * C;
  int32_t* __restrict__ lu = last_used + (size_t)bh * C;
  int32_t* __restrict__ ss = sel_slot + (size_t)bh * k;
  uint8_t* __restrict__ ht = hit + (size_t)bh * k;
  int32_t* __restrict__ mt = miss_tok + (size_t)bh * k;
  int32_t* __restrict__ ms = miss_slot + (size_t)bh * k;
  __syncthreads();  // phase-a2 buffers are dead; vkeys may overwrite them
  for (int sidx = t; sidx < Cpad; sidx += kT) {
    uint64_t key = ~0ull;
    if (sidx < C) {
      const int32_t u = lu[sidx];
      if (u != step) key = (((uint64_t)(uint32_t)(u + 1)) << 32) | (uint32_t)sidx;
    }
    A.vkeys[sidx] = key;
  }
  __syncthreads();
  for (int j0 = 0; j0 < k; j0 += kT) {
    const int j = j0 + t;
    int32_t tok = -1, slot = -1;
    bool miss = false;
    if (j < k) {
      tok = A.sel[j];
      slot = so[tok];
      if (slot >= C) slot = -1;  // corrupt map entry: treat as absent
      miss = slot < 0;
      if (!miss) {
        ss[j] = slot;
        ht[j] = 1;
        lu[slot] = step;
        A.vkeys[slot] = ~0ull;  // used in this step: never a victim
      } else {
        ht[j] = 0;
      }
    }
    uint32_t tot;
    const uint32_t rank = sh_nmiss + block_exclusive_scan(miss ? 1u : 0u, wave_tot, &tot);
    if (miss) {
      mt[rank] = tok;
      A.sel[j] = -(int32_t)rank - 2;  // remember the rank; the slot is filled in below
    }
    __syncthreads();
    if (t == 0) sh_nmiss += tot;
    __syncthreads();
  }
  const int nm = (int)sh_nmiss;
  KPROF(6);
  if (nm > 0) {
    bitonic_sort_lds(A.vkeys, Cpad);
    KPROF(7);
    for (int j = t; j < nm; j += kT) {
      const uint64_t key = A.vkeys[j];
      if (key == ~0ull) {  // ran out of victims (the caller reused `step`)
        atomicOr(&sh_bad, 1u);
        ms[j] = -1;
        continue;
      }
      const int32_t tok = mt[j];
      const int32_t v = (int32_t)(uint32_t)key;
      const int32_t old = to[v];
      if (old >= 0 && old < l) so[old] = -1;
      to[v] = tok;
      so[tok] = v;
      lu[v] = step;
      ms[j] = v;
    }
    __syncthreads();
    for (int j = t; j < k; j += kT) {
      const int32_t v = A.sel[j];
      if (v <= -2) ss[j] = ms[-(v + 2)];
    }
  }
  __syncthreads();
  KPROF(8);
  if (t == 0) n_miss[bh] = sh_bad ? -1 : nm;
}

template <bool RESOLVE>
hipError_t raise_lds_limit() {
  static bool done = false;
  if (done) return hipSuccess;
  const hipError_t e = hipFuncSetAttribute(
      reinterpret_cast<const void*>(select_resolve_kernel<RESOLVE>),
      hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024);
  if (e == hipSuccess) done = true;
  return e;
}

}  // namespace

bool select_resolve_fits(const lrqk_shape& s, bool resolve) {
  const int Cpad = next_pow2(s.C < 2 ? 2 : s.C);
  return arena_bytes(s.k, s.l - s.w, Cpad, resolve) <= 150 * 1024;
}

hipError_t launch_select_only(const lrqk_shape& s, const float* scores, int32_t* sel_idx,
                              hipStream_t st) {
  const int n = s.l - s.w;
  const size_t lds = arena_bytes(s.k, n, 0, false);
  hipError_t e = raise_lds_limit<false>();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((select_resolve_kernel<false>), dim3(s.B * s.Hq), dim3(kT), lds, st, scores,
                     s.l, n, s.k, sel_idx, 0, 0, 0, nullptr, nullptr, nullptr, nullptr, nullptr,
                     nullptr, nullptr, nullptr);
  return hipGetLastError();
}

hipError_t launch_select_resolve(const lrqk_shape& s, const float* scores, int32_t* sel_idx,
                                 int32_t step, int32_t* slot_of, int32_t* token_of,
                                 int32_t* last_used, int32_t* sel_slot, uint8_t* hit,
                                 int32_t* miss_tok, int32_t* miss_slot, int32_t* n_miss,
                                 hipStream_t st) {
  const int n = s.l - s.w;
  const int Cpad = next_pow2(s.C < 2 ? 2 : s.C);
  const size_t lds = arena_bytes(s.k, n, Cpad, true);
  hipError_t e = raise_lds_limit<true>();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((select_resolve_kernel<true>), dim3(s.B * s.Hq), dim3(kT), lds, st, scores,
                     s.l, n, s.k, sel_idx, step, s.C, Cpad, slot_of, token_of, last_used,
                     sel_slot, hit, miss_tok, miss_slot, n_miss);
  return hipGetLastError();
}

}  // namespace lrqk
