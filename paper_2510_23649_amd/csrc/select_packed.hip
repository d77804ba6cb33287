// a2 + a3 of the fused step, one workgroup of 1024 threads per (batch, query head), working
// straight from what the proxy-score pass left behind: the candidate bitmap (one 64-bit word
// per group of 64 positions) and the candidates' scores packed 8 per group
// (Alg. 2, top(., k); Sec. 4.1 active / lite tokens and the hit-and-miss cache).
//
// Thread t owns GPT consecutive groups, i.e. a contiguous run of positions, and keeps its
// candidates in registers from the first load to the last store: "thread order" is
// "position order", so nothing is ever listed or sorted, and every prefix count over the
// threads is a count in position order.
//   * one round of coalesced loads brings the thread's bitmap words and packed scores in
//     (with what the resolution will need from the cache state: last_used and token_of go
//     to LDS).  The first 8 (or 4) candidates of a group stay in registers, further ones are
//     parked in LDS; a group with more than the 8 packed candidates computes the others
//     again from A_K and q_hat with the proxy pass's fma chain;
//   * ONE histogram over (key - threshold key) >> s, 2048 bins (the candidates are the tail
//     of the score distribution above the threshold, so they spread over the bins instead
//     of piling into the two or three bins that fixed key bits would give), is scanned from
//     the top: it gives the bin that holds the k-th largest.  The few candidates of that bin
//     are ranked on (key, position) -- every wavefront does it for itself -- and the one
//     with the right rank is the cut: the selection is every candidate at or above it.  A
//     bin with many candidates (ties) goes through further 11-bit histogram levels and an
//     ordered cut instead;
//   * each thread then looks up slot_of for its own selected positions, and one prefix count
//     over (selected, missing) gives it its place in the outputs;
//   * the same histogram yields the key at rank 1.5 k, which (divided by |q_hat|) is handed
//     to the next step of the layer as its candidate threshold, so that steps after the
//     first need no threshold estimate of their own.
// A head whose candidates are unusable (fewer than k, or too many beyond the packed 8 per
// group) recomputes all its scores into the workspace and selects exactly from them
// (exact_select_from_scores): slower, same result.
//
// Resolution (Sec. 4.1; least recently selected victims in (last_used, slot) order): a
// histogram of the ages of the slots not used in this step is scanned from the oldest; the
// age classes that hold the n_miss oldest slots are numbered, and a victim's rank is the
// number of slots in older classes plus its index inside its class in slot order -- one
// more prefix count, whatever the number of victims.  Cache state is read from LDS: the
// slot_of look-ups are the only dependent global round trip of the kernel.
//
// All decisions are integer comparisons: the result is exact and independent of scheduling.
#include "lrqk_device.h"
#include "lrqk_internal.h"
#include "select_common.h"

namespace lrqk {
namespace {

constexpr int kOvCap = 2048;  // candidate keys beyond the packed 8 per group that a head may park
constexpr int kSmall = 64;    // candidates of the threshold bin that one wavefront ranks directly
constexpr int kMaxSpt = 8;    // cache slots per thread (C <= 8192)
constexpr size_t kPackedLdsLimit = 150 * 1024;

__host__ __device__ inline size_t up256(size_t x) { return (x + 255) / 256 * 256; }

constexpr int kMaxCls = 16;   // victim age classes numbered by the fast resolution

struct PackedArena {
  size_t st_b, k_b, fixed, x_b, total;
};
__host__ __device__ inline PackedArena packed_arena(int k, int n, int C) {
  PackedArena a;
  a.st_b = up256((size_t)C * 4);  // last_used; token_of has the same size
  a.k_b = up256((size_t)k * 4);   // miss positions; their output indices; victims in rank order
  // hist0 + ahist + parked keys + the threshold bin's (key, position) pairs
  a.fixed = 2 * a.st_b + 3 * a.k_b + 2 * 2048 * 4 + (size_t)kOvCap * 4 + up256((kSmall + 1) * 8);
  // shared: exact route (histogram + selection bitmap) | further histogram levels | the
  // all-slots sort of the rare resolution cases
  const size_t exact = (size_t)kBins * 4 + up256(((size_t)n + 31) / 32 * 4);
  int Cpad = 2;
  while (Cpad < C) Cpad <<= 1;
  const size_t sort_b = (size_t)Cpad * 8;
  a.x_b = exact > sort_b ? exact : sort_b;
  a.total = a.fixed + a.x_b;
  return a;
}

// Workgroup barrier that orders LDS traffic only: the wavefront's LDS operations have
// completed before it arrives, its global loads and stores stay in flight (a __syncthreads
// would wait for those too, i.e. expose a memory round trip at every barrier).  Used where
// the threads exchange data through LDS alone.
__device__ __forceinline__ void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Prefix sum over the 16 wave totals held in wt[0..16): returns the sum of the totals of the
// wavefronts before this one, and the grand total.  Lanes 0..15 of every wavefront read one
// total each and scan them with DPP row shifts (one LDS read instead of sixteen per thread).
__device__ __forceinline__ uint32_t waves_before(const uint32_t* wt, uint32_t* total) {
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  uint32_t v = wt[lane & 15];
  uint32_t incl = v;
  incl += dpp_zero_fill<0x111, 0xf>(incl);  // row_shr:1
  incl += dpp_zero_fill<0x112, 0xf>(incl);  // row_shr:2
  incl += dpp_zero_fill<0x114, 0xf>(incl);  // row_shr:4
  incl += dpp_zero_fill<0x118, 0xf>(incl);  // row_shr:8
  *total = (uint32_t)__builtin_amdgcn_readlane((int)incl, 15);
  return (uint32_t)__builtin_amdgcn_readlane((int)(incl - v), wv);
}

// Exclusive prefix sum over the 1024 threads and the total, with ONE LDS-only barrier.
// wt: 16 words of LDS that no thread may still be reading from an earlier scan: consecutive
// scans take different areas (scan_area), and an area comes round again only after two
// other barriers.
__device__ __forceinline__ uint32_t scan1(uint32_t v, uint32_t* wt, uint32_t* total) {
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const uint32_t incl = wave_inclusive_scan(v);
  if (lane == 63) wt[wv] = incl;
  lds_barrier();
  return waves_before(wt, total) + incl - v;
}
// The same for two values at once.  wt: 32 words of LDS, as above.
__device__ __forceinline__ void scan2(uint32_t v0, uint32_t v1, uint32_t* wt, uint32_t* ex0,
                                      uint32_t* ex1, uint32_t* tot0, uint32_t* tot1) {
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const uint32_t i0 = wave_inclusive_scan(v0), i1 = wave_inclusive_scan(v1);
  if (lane == 63) {
    wt[wv] = i0;
    wt[16 + wv] = i1;
  }
  lds_barrier();
  *ex0 = waves_before(wt, tot0) + i0 - v0;
  *ex1 = waves_before(wt + 16, tot1) + i1 - v1;
}

// Scan of a 2048-bin histogram from the top (thread t owns bins 2t, 2t+1) for two ranks at
// once: res[0] = the bin d that holds the want_a-th entry from the top, res[1] = the entries
// above d, res[3] = the bin that holds the want_b-th entry (0xffffffff where there are fewer
// entries than that).  Returns the number of entries.  LDS-only barriers.
__device__ __forceinline__ uint32_t find_two_from_top(const uint32_t* hist, uint32_t want_a,
                                                      uint32_t want_b, uint32_t* wt,
                                                      uint32_t* res) {
  const int t = threadIdx.x;
  const uint32_t c0 = hist[2 * t], c1 = hist[2 * t + 1];
  if (t == 0) {
    res[0] = 0xffffffffu;
    res[3] = 0xffffffffu;
  }
  uint32_t total;
  const uint32_t below = scan1(c0 + c1, wt, &total);  // its barriers order the writes of res
  const uint32_t above1 = total - below - c0 - c1;
  const uint32_t above0 = above1 + c1;
  if (above1 < want_a && want_a <= above1 + c1) {
    res[0] = 2 * t + 1;
    res[1] = above1;
  } else if (above0 < want_a && want_a <= above0 + c0) {
    res[0] = 2 * t;
    res[1] = above0;
  }
  if (above1 < want_b && want_b <= above1 + c1) {
    res[3] = 2 * t + 1;
  } else if (above0 < want_b && want_b <= above0 + c0) {
    res[3] = 2 * t;
  }
  lds_barrier();
  return total;
}

// Victim slots for the nm missing positions of a head (Sec. 4.1 hit-and-miss cache; replacement
// by least recent selection: victims in (last_used, slot) order, the j-th miss taking the j-th
// victim), then eviction and installation in the maps.  Called by all 1024 threads.
struct VictimWork {
  // LDS
  int32_t* lu_s;          // [C] last_used, already `step` where used in this step
  const int32_t* to_s;    // [C] token_of before the step
  const int32_t* mt_s;    // [nm] missing positions, ascending
  const int32_t* mj_s;    // [nm] their indices in the outputs
  int32_t* vsorted;       // [nm] receives the victims in rank order
  uint32_t* ahist;        // [kAgeBins], zero
  uint32_t* cls_age;      // [kMaxCls]
  uint32_t* cls_base;     // [kMaxCls]
  uint32_t* sh_ncls;      // zero
  uint32_t* sh_clip;      // zero
  uint32_t* sh_bad;
  uint32_t* scan_areas;   // four areas of 32 words for the prefix counts
  unsigned char* sort_area;  // 8 bytes per slot (C rounded up to a power of two): rare cases only
  // this head's maps and outputs (global)
  int32_t* so;
  int32_t* to;
  int32_t* lu;
  int32_t* ms;
  int32_t* ss;
  int32_t step;
  int C, l, spt;
};
template <int SPT>
__device__ __forceinline__ void assign_victims(const VictimWork& v, int nm) {
  const int t = threadIdx.x;
  const int C = v.C, l = v.l, spt = v.spt;
  const int32_t step = v.step;
  auto scan_area = [&](int i) { return v.scan_areas + (i & 3) * 2 * kWaves; };
  // ages of the slots not used in this step; thread t owns slots [s0, s1)
  const int s0 = min(C, t * spt), s1 = min(C, s0 + spt);
  uint32_t age[SPT];
#pragma unroll
  for (int u = 0; u < SPT; ++u) {
    age[u] = 0xffffffffu;  // not eligible
    if (u < spt && s0 + u < s1) {
      const int32_t lv = v.lu_s[s0 + u];
      if (lv != step) {
        age[u] = min((uint32_t)(step - 1 - lv), (uint32_t)(kAgeBins - 1));
        atomicAdd(&v.ahist[age[u]], 1u);
      }
    }
  }
  lds_barrier();
  // scan the age classes from the oldest: eligible slots above each class, and the number of
  // non-empty classes above it.  A non-empty class with fewer than nm slots above it holds
  // victims; its number among those classes is its index in cls_age / cls_base.
  uint32_t n_elig;
  {
    const uint32_t c0b = v.ahist[2 * t], c1b = v.ahist[2 * t + 1];
    const uint32_t e0 = c0b ? 1u : 0u, e1 = c1b ? 1u : 0u;
    uint32_t bc, be, ne;
    scan2(c0b + c1b, e0 + e1, scan_area(3), &bc, &be, &n_elig, &ne);
    const uint32_t above1 = n_elig - bc - c0b - c1b, ne_above1 = ne - be - e0 - e1;
    const uint32_t above0 = above1 + c1b, ne_above0 = ne_above1 + e1;
    if (c1b && above1 < (uint32_t)nm) {
      if (ne_above1 < (uint32_t)kMaxCls) {
        v.cls_age[ne_above1] = 2 * t + 1;
        v.cls_base[ne_above1] = above1;
      }
      atomicMax(v.sh_ncls, ne_above1 + 1);
      if (2 * t + 1 == kAgeBins - 1) *v.sh_clip = 1u;
    }
    if (c0b && above0 < (uint32_t)nm) {
      if (ne_above0 < (uint32_t)kMaxCls) {
        v.cls_age[ne_above0] = 2 * t;
        v.cls_base[ne_above0] = above0;
      }
      atomicMax(v.sh_ncls, ne_above0 + 1);
    }
    lds_barrier();
  }
  const int ncls = (int)*v.sh_ncls;
  // ages beyond the histogram's range share its last class, which then does not order them
  const bool clipped = *v.sh_clip != 0u && step > kAgeBins - 1;
  int nv = nm;  // number of victims found (< nm only if the caller reused `step`)
  if (n_elig >= (uint32_t)nm && ncls <= kMaxCls && !clipped) {
    // rank of a victim = slots in older classes + its index in its class, in slot order:
    // four classes per prefix count (16-bit fields)
    for (int c4 = 0; c4 < ncls; c4 += 4) {
      uint32_t ca[4], cb[4];
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        ca[c] = c4 + c < ncls ? v.cls_age[c4 + c] : 0xfffffffeu;
        cb[c] = c4 + c < ncls ? v.cls_base[c4 + c] : 0u;
      }
      uint32_t lo = 0, hi = 0;
#pragma unroll
      for (int u = 0; u < SPT; ++u)
        if (u < spt) {
          lo += (age[u] == ca[0] ? 1u : 0u) + (age[u] == ca[1] ? 1u << 16 : 0u);
          hi += (age[u] == ca[2] ? 1u : 0u) + (age[u] == ca[3] ? 1u << 16 : 0u);
        }
      uint32_t exlo, exhi, tl, th;
      scan2(lo, hi, scan_area(c4 >> 2), &exlo, &exhi, &tl, &th);
      uint32_t before[4] = {cb[0] + (exlo & 0xffffu), cb[1] + (exlo >> 16),
                            cb[2] + (exhi & 0xffffu), cb[3] + (exhi >> 16)};
#pragma unroll
      for (int u = 0; u < SPT; ++u)
        if (u < spt) {
#pragma unroll
          for (int c = 0; c < 4; ++c)
            if (age[u] == ca[c]) {
              const uint32_t rk = before[c]++;
              if (rk < (uint32_t)nm) v.vsorted[rk] = s0 + u;
            }
        }
    }
    lds_barrier();
  } else {
    // out of victims, too many classes, or ages beyond the histogram's range: sort every
    // slot's (last_used, slot) key
    uint64_t* const vlist = reinterpret_cast<uint64_t*>(v.sort_area);
    int Cpad = 2;
    while (Cpad < C) Cpad <<= 1;
    for (int i = t; i < Cpad; i += kT) {
      uint64_t key64 = ~0ull;
      if (i < C && v.lu_s[i] != step)
        key64 = (((uint64_t)(uint32_t)(v.lu_s[i] + 1)) << 32) | (uint32_t)i;
      vlist[i] = key64;
    }
    bitonic_sort_lds(vlist, Cpad);
    nv = (int)min((uint32_t)nm, n_elig);
    for (int jj = t; jj < nv; jj += kT) v.vsorted[jj] = (int32_t)(uint32_t)vlist[jj];
    __syncthreads();
  }
  for (int jj = t; jj < nm; jj += kT) {
    if (jj >= nv) {  // ran out of victims (the caller reused `step`)
      atomicOr(v.sh_bad, 1u);
      v.ms[jj] = -1;
      v.ss[v.mj_s[jj]] = -1;
      continue;
    }
    const int32_t slot = v.vsorted[jj];
    const int32_t tok = v.mt_s[jj];
    const int32_t old = v.to_s[slot];
    if (old >= 0 && old < l) v.so[old] = -1;
    v.to[slot] = tok;
    v.so[tok] = slot;
    v.lu[slot] = step;
    v.ms[jj] = slot;
    v.ss[v.mj_s[jj]] = slot;
  }
}

struct PackedArgs {
  const unsigned long long* bitmap;  // [BHq][words64]
  const float* cand_scores;          // [BHq][words64][kCandPerGroup]
  const uint32_t* thr_used;          // [BHq] key the proxy pass filtered with
  const float* A_K;
  const float* q_hat;
  float* scores_w;  // [BHq][l] scratch of a head that takes the exact route
  float* sel_thr;   // [BHq] threshold / |q_hat| handed to the layer's next step (may be null)
  int words64, r, Hq, Hkv, l, lrows, n, k, C;
  int32_t step;
  int32_t* sel_idx;
  int32_t* slot_of;
  int32_t* token_of;
  int32_t* last_used;
  int32_t* sel_slot;
  uint8_t* hit;
  int32_t* miss_tok;
  int32_t* miss_slot;
  int32_t* n_miss;
};

template <int GPT, int SPT, int SLOTS>
__global__ __launch_bounds__(kT) void select_packed_kernel(const PackedArgs a) {
  extern __shared__ __align__(16) unsigned char lds_raw[];
  __shared__ uint32_t wave_tot[4 * 2 * kWaves];  // four areas of 32 words, used in rotation
  auto scan_area = [&](int i) { return wave_tot + (i & 3) * 2 * kWaves; };
  __shared__ uint32_t res[4];
  __shared__ uint32_t sh_ov, sh_small_n, sh_bad, sh_ncls, sh_clip;
  __shared__ uint64_t sh_cut;
  __shared__ uint32_t cls_age[kMaxCls], cls_base[kMaxCls];

  const int bh = blockIdx.x, t = threadIdx.x;
  const int lane = t & 63, wv = t >> 6;
  const int n = a.n, k = a.k, C = a.C, l = a.l, r = a.r;
  const PackedArena az = packed_arena(k, n, C);
  int32_t* const lu_s = reinterpret_cast<int32_t*>(lds_raw);
  int32_t* const to_s = reinterpret_cast<int32_t*>(lds_raw + az.st_b);
  int32_t* const mt_s = reinterpret_cast<int32_t*>(lds_raw + 2 * az.st_b);  // [k] miss positions
  int32_t* const mj_s = reinterpret_cast<int32_t*>(lds_raw + 2 * az.st_b + az.k_b);  // their j
  int32_t* const vsorted = reinterpret_cast<int32_t*>(lds_raw + 2 * az.st_b + 2 * az.k_b);
  uint32_t* const ahist = reinterpret_cast<uint32_t*>(lds_raw + 2 * az.st_b + 3 * az.k_b);
  uint32_t* const hist0 = ahist + kAgeBins;
  uint32_t* const ov_key = hist0 + 2048;
  uint64_t* const small = reinterpret_cast<uint64_t*>(ov_key + kOvCap);
  unsigned char* const X = lds_raw + az.fixed;
  // staging of the outputs in output order, over memory the selection no longer needs
  int32_t* const sel_o = reinterpret_cast<int32_t*>(hist0);  // [k] <= hist0 + ov_key
  int32_t* const slot_o = reinterpret_cast<int32_t*>(X);     // [k] slot, or -1 - miss rank

  const int b = bh / a.Hq, h = bh - b * a.Hq, kvh = h / (a.Hq / a.Hkv);
  const float* __restrict__ Arow = a.A_K + ((size_t)b * a.Hkv + kvh) * (size_t)a.lrows * r;
  const float* __restrict__ qh = a.q_hat + (size_t)bh * r;
  int32_t* __restrict__ so = a.slot_of + (size_t)bh * a.lrows;
  int32_t* __restrict__ to = a.token_of + (size_t)bh * C;
  int32_t* __restrict__ lu = a.last_used + (size_t)bh * C;
  const int32_t step = a.step;
  // ---- 0. every load that does not depend on the selection -----------------------------------
  const int ngroups = (n + 63) >> 6;
  const unsigned long long* __restrict__ bm = a.bitmap + (size_t)bh * a.words64;
  const float4* __restrict__ cs4 =
      reinterpret_cast<const float4*>(a.cand_scores + (size_t)bh * a.words64 * kCandPerGroup);
  unsigned long long mask[GPT];
  float4 sc[GPT][2];
#pragma unroll
  for (int g = 0; g < GPT; ++g) {
    const int gi = t * GPT + g;
    const bool on = gi < ngroups;
    mask[g] = on ? bm[gi] : 0ull;
    // a group without candidates holds stale scores; they are never interpreted
    sc[g][0] = on ? cs4[2 * gi] : make_float4(0.f, 0.f, 0.f, 0.f);
    sc[g][1] = on ? cs4[2 * gi + 1] : make_float4(0.f, 0.f, 0.f, 0.f);
  }
  // cache state: coalesced loads (slot i by thread i mod 1024), handed over through LDS to
  // the threads that own contiguous runs of slots below
  const int spt = (C + kT - 1) / kT;  // cache slots per thread, <= SPT
  int32_t lu_r[SPT], to_r[SPT];
#pragma unroll
  for (int u = 0; u < SPT; ++u) {
    lu_r[u] = 0;
    to_r[u] = -1;
    if (u < spt && u * kT + t < C) {
      lu_r[u] = lu[u * kT + t];
      to_r[u] = to[u * kT + t];
    }
  }
  const uint32_t thr_key = a.thr_used[bh];
  float qq = 0.0f;  // |q_hat|^2, summed by the last wavefront
  if (wv == kWaves - 1)
    for (int j = lane; j < r; j += 64) qq = __builtin_fmaf(qh[j], qh[j], qq);

  for (int i = t; i < 2048 + kAgeBins; i += kT) ahist[i] = 0u;  // ahist and hist0
  if (t == 0) {
    sh_ov = 0u;
    sh_small_n = 0u;
    sh_bad = 0u;
    sh_ncls = 0u;
    sh_clip = 0u;
  }
  lds_barrier();

  // ---- 1. the thread's candidates: key and position of each, histogram of the keys ---------------
  // Every candidate's key is >= thr_key.  Bin of a key: (key - thr_key) >> s, the top bin
  // taking everything beyond.  For a positive threshold s = 12 spreads the scores between the
  // threshold and twice the threshold over the 2048 bins.
  int s = (thr_key > 0x80800000u && thr_key < 0xff800000u) ? 12 : 21;
  auto bin_of = [&](uint32_t kk) { return min((kk - thr_key) >> s, 2047u); };
  // (key, position) as one number: larger = better (higher key, or equal key and lower position)
  auto value_of = [&](uint32_t kk, int g, int bpos) {
    return ((uint64_t)kk << 32) | (uint32_t) ~(uint32_t)((t * GPT + g) * 64 + bpos);
  };
  // The first SLOTS candidates of a group stay in registers; the others (packed entries beyond
  // SLOTS, and candidates beyond the 8 packed ones, whose scores are computed again from A_K)
  // are parked in LDS, in position order, in a run the thread reserves.
  uint32_t key[GPT][SLOTS];
  unsigned long long bpos6[GPT];  // bit positions of the candidates in registers, 6 bits each
  auto bpos_of = [&](int g, int i) { return (int)((bpos6[g] >> (6 * i)) & 63ull); };
  int cnt[GPT];
  int extra = 0;
#pragma unroll
  for (int g = 0; g < GPT; ++g) {
    cnt[g] = __popcll(mask[g]);
    extra += max(cnt[g] - SLOTS, 0);
  }
  int ov_base = 0;
  bool ov_ok = true;
  if (extra > 0) {
    ov_base = (int)atomicAdd(&sh_ov, (uint32_t)extra);
    ov_ok = ov_base + extra <= kOvCap;
  }
  {
    int idx = ov_base;
#pragma unroll
    for (int g = 0; g < GPT; ++g) {
      const float v[kCandPerGroup] = {sc[g][0].x, sc[g][0].y, sc[g][0].z, sc[g][0].w,
                                      sc[g][1].x, sc[g][1].y, sc[g][1].z, sc[g][1].w};
      unsigned long long mb = mask[g];
      bpos6[g] = 0ull;
#pragma unroll
      for (int i = 0; i < kCandPerGroup; ++i) {
        if (i < SLOTS) key[g][i] = 0u;
        if (i < cnt[g]) {
          const uint32_t kk = order_key(v[i]);
          if (i < SLOTS) {
            key[g][i] = kk;
            bpos6[g] |= (unsigned long long)__builtin_ctzll(mb) << (6 * (i < SLOTS ? i : 0));
            atomicAdd(&hist0[bin_of(kk)], 1u);
          } else if (ov_ok) {
            ov_key[idx++] = kk;
            atomicAdd(&hist0[bin_of(kk)], 1u);
          }
          mb &= mb - 1ull;
        }
      }
      if (cnt[g] > kCandPerGroup && ov_ok) {
        while (mb) {  // more candidates than the proxy pass packed
          const int bp = __builtin_ctzll(mb);
          mb &= mb - 1ull;
          const uint32_t kk = order_key(proxy_score_of_row(Arow, qh, r, (t * GPT + g) * 64 + bp));
          ov_key[idx++] = kk;
          atomicAdd(&hist0[bin_of(kk)], 1u);
        }
      }
    }
  }
  // Calls f(key, group, bit) for each of the thread's candidates beyond those in registers.
  auto for_each_extra = [&](auto&& f) {
    if (extra == 0) return;
    int idx = ov_base;
#pragma unroll
    for (int g = 0; g < GPT; ++g) {
      if (cnt[g] <= SLOTS) continue;
      unsigned long long mb = mask[g];
#pragma unroll
      for (int i = 0; i < SLOTS; ++i) mb &= mb - 1ull;
      while (mb) {
        const int bp = __builtin_ctzll(mb);
        mb &= mb - 1ull;
        f(ov_key[idx++], g, bp);
      }
    }
  };
  // ... and for all of them, those in registers first (any order will do for the callers)
  auto for_each_candidate = [&](auto&& f) {
#pragma unroll
    for (int g = 0; g < GPT; ++g)
#pragma unroll
      for (int i = 0; i < SLOTS; ++i)
        if (i < cnt[g]) f(key[g][i], g, bpos_of(g, i));
    for_each_extra(f);
  };
  // the cache state goes to LDS while the histogram settles
#pragma unroll
  for (int u = 0; u < SPT; ++u)
    if (u < spt && u * kT + t < C) {
      lu_s[u * kT + t] = lu_r[u];
      to_s[u * kT + t] = to_r[u];
    }

  const uint32_t rank_next = (uint32_t)k + (uint32_t)(k >> 1);  // candidates wanted next step
  uint32_t selm[GPT];                                           // selected packed candidates
  unsigned long long take_x[GPT];                               // selected ones beyond them
#pragma unroll
  for (int g = 0; g < GPT; ++g) {
    selm[g] = 0u;
    take_x[g] = 0ull;
  }
  float thr_next;

  lds_barrier();
  uint32_t m = find_two_from_top(hist0, (uint32_t)k, rank_next, scan_area(0), res);
  uint32_t d0 = res[0], above0 = res[1], d_next = res[3];
  const bool fast = m >= (uint32_t)k && sh_ov <= (uint32_t)kOvCap;

  if (fast) {
    if (d0 == 2047u && s != 21) {
      // the k-th largest lies beyond twice the threshold: bin the whole key range instead
      s = 21;
      lds_barrier();  // res has been read
      for (int i = t; i < 2048; i += kT) hist0[i] = 0u;
      lds_barrier();
      for_each_candidate([&](uint32_t kk, int, int) { atomicAdd(&hist0[bin_of(kk)], 1u); });
      lds_barrier();
      m = find_two_from_top(hist0, (uint32_t)k, rank_next, scan_area(1), res);
      d0 = res[0];
      above0 = res[1];
      d_next = res[3];
    }
    const uint32_t c0 = hist0[d0];
    const uint32_t want1 = (uint32_t)k - above0;  // how many of bin d0 are selected
    uint64_t cut;
    if (c0 <= (uint32_t)kSmall) {
      // the few candidates of bin d0 are ranked on (key, position); the want1-th of them is
      // the cut
      for_each_candidate([&](uint32_t kk, int g, int bp) {
        if (bin_of(kk) == d0) small[atomicAdd(&sh_small_n, 1u)] = value_of(kk, g, bp);
      });
      lds_barrier();
      {
        // every wavefront ranks the bin for itself (no second barrier to hand the cut over)
        const uint64_t mine = lane < (int)c0 ? small[lane] : 0ull;
        uint32_t larger = 0;
#pragma unroll 8
        for (uint32_t jj = 0; jj < c0; ++jj) larger += small[jj] > mine ? 1u : 0u;
        const unsigned long long is_cut = __ballot(lane < (int)c0 && larger == want1 - 1u);
        const int src = __builtin_ctzll(is_cut);  // exactly one entry has that rank
        const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(mine >> 32), src);
        const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)mine, src);
        cut = ((uint64_t)hi << 32) | lo;
      }
    } else {
      // many candidates in the bin (ties): further histogram levels over the low s bits give
      // the exact key tau of the k-th largest; of the candidates with that key the first
      // need_eq in position order are selected, so the cut is the need_eq-th of them
      uint32_t* const hist1 = reinterpret_cast<uint32_t*>(X);
      uint32_t known = d0, want = want1;
      int rem = s;
      while (rem > 0) {
        const int bits = rem < 11 ? rem : 11;
        const int nsh = rem - bits;
        __syncthreads();  // res and hist1 of the previous level have been read
        for (int i = t; i < 2048; i += kT) hist1[i] = 0u;
        __syncthreads();
        for_each_candidate([&](uint32_t kk, int, int) {
          const uint32_t rel = kk - thr_key;
          if ((rel >> rem) == known) atomicAdd(&hist1[(rel >> nsh) & ((1u << bits) - 1u)], 1u);
        });
        __syncthreads();
        find_from_top(hist1, want, wave_tot, res);
        const uint32_t dd = res[0], ab = res[1];
        known = (known << bits) | dd;
        want -= ab;
        rem = nsh;
      }
      // (bin d0 is never the catch-all top bin here, so rel >> s == d0 identifies it)
      const uint32_t tau = thr_key + known, need_eq = want;
      // the thread's candidates with key tau, in position order
      uint32_t neq = 0;
#pragma unroll
      for (int g = 0; g < GPT; ++g) {
#pragma unroll
        for (int i = 0; i < SLOTS; ++i) neq += (i < cnt[g] && key[g][i] == tau) ? 1u : 0u;
      }
      for_each_extra([&](uint32_t kk, int, int) { neq += kk == tau ? 1u : 0u; });
      uint32_t tot;
      uint32_t eq_rank = block_exclusive_scan(neq, wave_tot, &tot);
      if (eq_rank < need_eq && need_eq <= eq_rank + neq) {  // the need_eq-th is one of mine
        int idx = ov_base;
#pragma unroll
        for (int g = 0; g < GPT; ++g) {
          unsigned long long mb = mask[g];
          int i = 0;
          while (mb) {  // position order: packed ones, then the others
            const int bp = __builtin_ctzll(mb);
            mb &= mb - 1ull;
            uint32_t kk = 0u;
#pragma unroll
            for (int ii = 0; ii < SLOTS; ++ii)
              if (ii == i) kk = key[g][ii];
            if (i >= SLOTS) kk = ov_key[idx++];
            ++i;
            if (kk == tau && ++eq_rank == need_eq) sh_cut = value_of(kk, g, bp);
          }
        }
      }
      __syncthreads();
      cut = sh_cut;
    }
    // ---- 2. the selection = candidates at or above the cut; their slot_of look-ups ---------------
#pragma unroll
    for (int g = 0; g < GPT; ++g) {
#pragma unroll
      for (int i = 0; i < SLOTS; ++i)
        if (i < cnt[g] && value_of(key[g][i], g, bpos_of(g, i)) >= cut) selm[g] |= 1u << i;
    }
    for_each_extra([&](uint32_t kk, int g, int bp) {
      if (value_of(kk, g, bp) >= cut) take_x[g] |= 1ull << bp;
    });
    // threshold for the layer's next step: the lower edge of the bin that holds rank 1.5 k, or,
    // with fewer candidates than that, an extrapolation along an exponential tail through
    // (threshold used, m) and (the k-th largest, k)
    if (d_next != 0xffffffffu) {
      thr_next = key_to_float(thr_key + (d_next << s));
    } else {
      const float tau_f = key_to_float((uint32_t)(cut >> 32)), used_f = key_to_float(thr_key);
      float ratio = 8.0f;
      if (m > (uint32_t)k) {
        ratio = __logf(1.5f) / __logf((float)m / (float)k);
        ratio = fminf(fmaxf(ratio, 1.0f), 8.0f);
      }
      thr_next = tau_f - fmaxf(tau_f - used_f, 0.0f) * ratio;
    }
  } else {
    // ---- exact route: all scores of this head, then selection from them ------------------------------
    float* sw = a.scores_w + (size_t)bh * l;
    for (int row = t; row < n; row += kT) sw[row] = proxy_score_of_row(Arow, qh, r, row);
    __threadfence_block();
    __syncthreads();
    uint32_t* const hist = reinterpret_cast<uint32_t*>(X);
    uint32_t* const bitmap_l = hist + kBins;
    uint32_t bin_next;
    exact_select_from_scores<false>(sw, n, k, (l & 3) == 0, rank_next, hist, bitmap_l, nullptr,
                                    wave_tot, res, &bin_next);
    // the selection as bits of the thread's groups; none of it is a candidate in registers
#pragma unroll
    for (int g = 0; g < GPT; ++g) {
      const int gi = t * GPT + g;
      cnt[g] = 0;
      if (gi < ngroups) {
        const uint32_t lo = bitmap_l[2 * gi];
        const uint32_t hi = (2 * gi + 1) * 32 < n ? bitmap_l[2 * gi + 1] : 0u;
        take_x[g] = ((unsigned long long)hi << 32) | lo;
      }
    }
    thr_next = key_to_float(bin_next << kBinShift);  // lower edge of that 12-bit bin
  }
  if (wv == kWaves - 1) {
    // |q_hat|: the next step multiplies by its own
    float q2 = qq;
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) q2 += __shfl_xor(q2, d);
    if (lane == 0 && a.sel_thr) {
      const float nrm = sqrtf(q2);
      const float v = thr_next / nrm;
      a.sel_thr[bh] = (nrm > 0.0f && isfinite(v)) ? v : __uint_as_float(0x7fc00000u);
    }
  }

  // slot_of of the thread's selected positions (selected packed candidates: in registers)
  int32_t slot[GPT][SLOTS];
  uint32_t nsel = 0, nmiss = 0;
#pragma unroll
  for (int g = 0; g < GPT; ++g) {
    const int base = (t * GPT + g) * 64;
#pragma unroll
    for (int i = 0; i < SLOTS; ++i) {
      slot[g][i] = 0;
      if (selm[g] & (1u << i)) slot[g][i] = so[base + bpos_of(g, i)];
    }
  }
#pragma unroll
  for (int g = 0; g < GPT; ++g) {
    nsel += (uint32_t)__popc(selm[g]) + (uint32_t)__popcll(take_x[g]);
#pragma unroll
    for (int i = 0; i < SLOTS; ++i)
      if (selm[g] & (1u << i)) {
        if (slot[g][i] >= C) slot[g][i] = -1;  // corrupt map entry: treat as absent
        nmiss += slot[g][i] < 0 ? 1u : 0u;
      }
    unsigned long long tb = take_x[g];
    while (tb) {
      const int32_t sl = so[(t * GPT + g) * 64 + __builtin_ctzll(tb)];
      nmiss += (sl < 0 || sl >= C) ? 1u : 0u;
      tb &= tb - 1ull;
    }
  }
  // ---- 3. places in the outputs: one prefix count over (selected, missing) ---------------------------
  uint32_t j, mrank, tot_sel, tot_miss;
  scan2(nsel, nmiss, scan_area(2), &j, &mrank, &tot_sel, &tot_miss);
  const int nm = (int)tot_miss;
  int32_t* __restrict__ out = a.sel_idx + (size_t)bh * k;
  int32_t* __restrict__ ss = a.sel_slot + (size_t)bh * k;
  uint8_t* __restrict__ ht = a.hit + (size_t)bh * k;
  int32_t* __restrict__ mt = a.miss_tok + (size_t)bh * k;
  int32_t* __restrict__ ms = a.miss_slot + (size_t)bh * k;
  {
    // staged in LDS in output order (the thread's own entries are scattered lanes of many
    // predicated stores); the global stores follow, coalesced.  (Every thread has made its
    // decisions before the barrier of the prefix count above: the selection's LDS is free.)
    auto emit = [&](int p, int32_t sl) {
      if (j >= (uint32_t)k) return;  // cannot happen: exactly k positions are selected
      sel_o[j] = p;
      if (sl >= 0) {
        slot_o[j] = sl;
      } else {
        slot_o[j] = -1 - (int32_t)mrank;
        mt_s[mrank] = p;
        mj_s[mrank] = (int32_t)j;
        ++mrank;
      }
      ++j;
    };
#pragma unroll
    for (int g = 0; g < GPT; ++g) {
      const int base = (t * GPT + g) * 64;
      // position order inside the group: the candidates in registers come first, in position
      // order; the ones beyond them lie at higher positions
#pragma unroll
      for (int i = 0; i < SLOTS; ++i)
        if (selm[g] & (1u << i)) emit(base + bpos_of(g, i), slot[g][i]);
      unsigned long long tb = take_x[g];
      while (tb) {
        const int p = base + __builtin_ctzll(tb);
        int32_t sl = so[p];
        if (sl >= C) sl = -1;
        emit(p, sl);
        tb &= tb - 1ull;
      }
    }
    lds_barrier();
    for (int jj = t; jj < k; jj += kT) {
      const int p = sel_o[jj];
      const int32_t sl = slot_o[jj];
      out[jj] = p;
      ht[jj] = sl >= 0 ? 1 : 0;
      if (sl >= 0) {
        ss[jj] = sl;
        lu[sl] = step;
        lu_s[sl] = step;  // used in this step: never a victim
      } else {
        mt[-1 - sl] = p;
      }
    }
  }
  lds_barrier();

  // ---- 4. victims ------------------------------------------------------------------------------------
  if (nm > 0) {
    VictimWork v;
    v.lu_s = lu_s;
    v.to_s = to_s;
    v.mt_s = mt_s;
    v.mj_s = mj_s;
    v.vsorted = vsorted;
    v.ahist = ahist;
    v.cls_age = cls_age;
    v.cls_base = cls_base;
    v.sh_ncls = &sh_ncls;
    v.sh_clip = &sh_clip;
    v.sh_bad = &sh_bad;
    v.scan_areas = wave_tot;
    v.sort_area = X;
    v.so = so;
    v.to = to;
    v.lu = lu;
    v.ms = ms;
    v.ss = ss;
    v.step = step;
    v.C = C;
    v.l = l;
    v.spt = spt;
    assign_victims<SPT>(v, nm);
  }
  lds_barrier();
  if (t == 0) a.n_miss[bh] = sh_bad ? -1 : nm;
}

// Candidates of a group kept in registers: all 8 packed ones where a thread owns one or two
// groups, 4 where it owns three or four (the registers would not hold more; at one or two
// groups per thread 4, 6 or 8 measure the same).
template <int GPT>
constexpr int slots_in_registers() {
  return GPT <= 2 ? kCandPerGroup : 4;
}

template <int GPT, int SPT>
hipError_t launch_inst(const PackedArgs& a, int BHq, size_t lds, hipStream_t st) {
  static std::atomic<uint64_t> raised{0};  // devices on which this instantiation's ceiling is up
  const hipError_t e =
      raise_dynamic_lds_once(select_packed_kernel<GPT, SPT, slots_in_registers<GPT>()>,
                             kPackedLdsLimit, raised);
  if (e != hipSuccess) return e;
  LRQK_LAUNCH((select_packed_kernel<GPT, SPT, slots_in_registers<GPT>()>), dim3(BHq), dim3(kT), lds,
              st, a);
  return hipGetLastError();
}
template <int GPT>
hipError_t launch_gpt(const PackedArgs& a, int BHq, size_t lds, hipStream_t st) {
  if (a.C <= 2 * kT) return launch_inst<GPT, 2>(a, BHq, lds, st);
  if (a.C <= 4 * kT) return launch_inst<GPT, 4>(a, BHq, lds, st);
  return launch_inst<GPT, 8>(a, BHq, lds, st);
}

}  // namespace

bool select_packed_fits(const lrqk_shape& s) {
  const int n = s.l - s.w;
  if (((n + 63) >> 6) > 4 * kT) return false;  // at most 4 groups of 64 positions per thread
  if (s.C > kMaxSpt * kT) return false;
  // Dense selections (k a sizeable fraction of the context) put more than 8 candidates into
  // most groups: the 1.5 k candidates the threshold aims at, less the 8 per group that the proxy
  // pass packs, must leave room in the area for the others
  if ((long)s.k + s.k / 2 - (long)kCandPerGroup * ((n + 63) >> 6) > kOvCap / 2) return false;
  return packed_arena(s.k, n, s.C).total <= kPackedLdsLimit;
}

hipError_t launch_select_packed(const lrqk_shape& s, const unsigned long long* bitmap,
                                const float* cand_scores, const uint32_t* thr_used,
                                const float* A_K, const float* q_hat, float* scores_w,
                                float* sel_thr, int32_t* sel_idx, int32_t step, int32_t* slot_of,
                                int32_t* token_of, int32_t* last_used, int32_t* sel_slot,
                                uint8_t* hit, int32_t* miss_tok, int32_t* miss_slot,
                                int32_t* n_miss, hipStream_t st) {
  const int n = s.l - s.w;
  PackedArgs a;
  a.bitmap = bitmap;
  a.cand_scores = cand_scores;
  a.thr_used = thr_used;
  a.A_K = A_K;
  a.q_hat = q_hat;
  a.scores_w = scores_w;
  a.sel_thr = sel_thr;
  a.words64 = filter_words64(n);
  a.r = s.r;
  a.Hq = s.Hq;
  a.Hkv = s.Hkv;
  a.l = s.l;
  a.lrows = row_cap(s);
  a.n = n;
  a.k = s.k;
  a.C = s.C;
  a.step = step;
  a.sel_idx = sel_idx;
  a.slot_of = slot_of;
  a.token_of = token_of;
  a.last_used = last_used;
  a.sel_slot = sel_slot;
  a.hit = hit;
  a.miss_tok = miss_tok;
  a.miss_slot = miss_slot;
  a.n_miss = n_miss;
  const size_t lds = packed_arena(s.k, n, s.C).total;
  const int groups = (n + 63) >> 6;
  const int BHq = s.B * s.Hq;
  if (groups <= kT) return launch_gpt<1>(a, BHq, lds, st);
  if (groups <= 2 * kT) return launch_gpt<2>(a, BHq, lds, st);
  if (groups <= 3 * kT) return launch_gpt<3>(a, BHq, lds, st);
  return launch_gpt<4>(a, BHq, lds, st);
}

}  // namespace lrqk
