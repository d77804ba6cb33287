// a2 + a3 in one workgroup per (batch, query head): exact top-k selection over the
// proxy scores followed, optionally, by hit/miss resolution against the cache state
// (Alg. 2, top(., k); Sec. 4.1 active / lite tokens and the hit-and-miss cache).
//
// Everything a head needs fits in the LDS of one CU, so a head is handled without
// any traffic between workgroups.  Selection works on an order-preserving 32-bit
// key of the score (larger score <=> larger key; equal scores: lower position first).
//
//  Selection, usual route (no sorting, the l scores of the head are never read here):
//   1. a candidate bitmap of the positions whose key is at or above an estimated threshold.
//      In the fused step it comes from the proxy-score pass (one 64-bit ballot per 64
//      positions, with the candidates' scores packed 8 per 64-position group beside it)
//      and is copied into LDS.  Working from a materialised score array (the stand-alone
//      entry point) the kernel builds it itself: a histogram of the top 12 key bits over a
//      1-in-8 sample of the positions gives a bin at or below the bin of the k-th largest
//      score, with a safety margin, and one pass over the scores marks every position at
//      or above that bin (4 positions per lane, 8 lanes OR-ed into one word: no atomics);
//   2. a prefix count over the bitmap turns it into an ascending list of m candidate
//      positions; if k <= m <= capacity the estimate was good (this is checked, not
//      assumed).  The candidates' keys are taken from the packed scores (a group with more
//      than 8 candidates recomputes the others from A_K and q_hat with the same fma chain)
//      or read back from the score array, and an exact 3-level radix select in LDS finds
//      the key of the k-th largest; candidates above it, and the first ones equal to it
//      in position order, are the selection -- already in ascending position.
//  Selection, safe route (taken by a head whose check in step 2 fails: a bad estimate or
//  massive ties): the head's scores are needed in full -- in the fused step they are first
//  recomputed from A_K into the workspace -- then a full histogram, two 10-bit refinements
//  of the threshold over the scores, one pass that sets the bitmap (positions with the
//  threshold key counted in position order), and the same prefix count.  Slower, same
//  result.
//
//  Resolution: each selected position looks up slot_of (hit: refresh; miss: ranked in
//  position order).  Victims are the least recently selected slots: a histogram of
//  the slots' ages finds the age class that completes the n_miss oldest, the class
//  is cut in slot order, and the victims are ranked among themselves on
//  (last_used, slot) by direct comparison.
//
// All decisions are integer comparisons: the result is exact and independent of
// scheduling.
#include "lrqk_device.h"
#include "lrqk_internal.h"
#include "select_common.h"

namespace lrqk {
namespace {

using namespace dev;

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
    const float* scores, const uint32_t* __restrict__ ext_bitmap, int ext_words,
    // with an external bitmap the scores are not materialised: they are recomputed from A_K
    // (scores_w: this head's slice is filled in only if the safe route needs every score)
    const float* __restrict__ cand_scores, const float* __restrict__ A_K,
    const float* __restrict__ q_hat, float* scores_w, int r,
    int Hq, int Hkv, int l, int lrows, int n, int k, int32_t* __restrict__ sel_idx,
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

  const float* s = scores + (size_t)bh * l;
  const bool vec_ok = (l & 3) == 0;
  const bool recompute = ext_bitmap != nullptr && A_K != nullptr;
  const float* __restrict__ Arow = nullptr;  // this head's A_K and q_hat (recompute only)
  const float* __restrict__ qh = nullptr;
  if (recompute) {
    const int b = bh / Hq, h = bh - b * Hq, kvh = h / (Hq / Hkv);
    Arow = A_K + ((size_t)b * Hkv + kvh) * (size_t)lrows * r;
    qh = q_hat + (size_t)bh * r;
  }
  const int n_iter = (n + kIter - 1) / kIter;
  const int words = (n + 31) / 32;
  const int wpt = (words + kT - 1) / kT;  // bitmap words per thread in the prefix counts

  if (t == 0) {
    sh_nmiss = 0u;
    sh_bad = 0u;
  }
  if (ext_bitmap != nullptr) {
    // the proxy-score pass already marked the candidates of this head
    const uint32_t* __restrict__ eb = ext_bitmap + (size_t)bh * ext_words;
    for (int i = t; i < words; i += kT) bitmap[i] = eb[i];
    __syncthreads();
  } else {
  // ---- 1. sampled histogram -> b_lo ------------------------------------------------------
  const int stride = (n >= 65536 && k >= 512) ? kSampleStride : 1;
  for (int i = t; i < kBins; i += kT) hist[i] = 0u;
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
    uint32_t above_unused;
    find_from_top_4096(hist, want, wave_tot, res, &b_lo, &above_unused);
  }
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

  }
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
        const int wi = t * wpt + j;
        uint32_t wbits = bitmap[wi];
        // rank of a bit inside its 64-position group (two words): where the proxy-score
        // pass left that candidate's score
        int grank = (wi & 1) ? __popc(bitmap[wi - 1]) : 0;
        while (wbits) {
          const int bpos = __ffs((int)wbits) - 1;
          wbits &= wbits - 1;
          clist[off] = wi * 32 + bpos;
          ckey[off] = grank < kCandPerGroup ? (uint32_t)((wi >> 1) * kCandPerGroup + grank)
                                            : 0xffffffffu;
          ++grank;
          ++off;
        }
      }
    }
  }
  __syncthreads();
  if (m >= (uint32_t)k && m <= (uint32_t)cap) {
    for (int i = t; i < kBins; i += kT) hist[i] = 0u;
    if (recompute) {
      const float* __restrict__ cs =
          cand_scores + (size_t)bh * (size_t)(ext_words >> 1) * kCandPerGroup;
      for (uint32_t i = t; i < m; i += kT) {
        const uint32_t slot = ckey[i];
        ckey[i] = order_key(slot != 0xffffffffu ? cs[slot] : proxy_score_of_row(Arow, qh, r, clist[i]));
      }
    } else {
      for (uint32_t i = t; i < m; i += kT) ckey[i] = order_key(s[clist[i]]);
    }
    __syncthreads();
    // exact key of the k-th largest candidate: digits [31:21], [20:10], [9:0]
    uint32_t prefix = 0, remaining = (uint32_t)k;
    uint32_t n_eq_total = 0;
#pragma unroll
    for (int level = 0; level < 3; ++level) {
      const int shift = level == 0 ? 21 : (level == 1 ? 10 : 0);
      const int bits = level == 2 ? 10 : 11;
      const int known = shift + bits;  // key >> known must equal prefix
      uint32_t* const lh = hist + (level & 1) * 2048;  // the other half was cleared meanwhile
      for (uint32_t i = t; i < m; i += kT) {
        const uint32_t key = ckey[i];
        if (level == 0 || (key >> known) == prefix)
          atomicAdd(&lh[(key >> shift) & ((1u << bits) - 1u)], 1u);
      }
      for (int i = t; i < 2048; i += kT) hist[((level + 1) & 1) * 2048 + i] = 0u;
      __syncthreads();
      find_from_top(lh, remaining, wave_tot, res);
      prefix = (prefix << bits) | res[0];
      remaining -= res[1];
      n_eq_total = lh[res[0]];
      __syncthreads();
    }
    const uint32_t tau = prefix, need_eq = remaining;
    // candidates are in ascending position: take key > tau, and the first need_eq with key == tau
    const uint32_t per = (m + kT - 1) / kT;
    const uint32_t i0 = min(m, (uint32_t)t * per), i1 = min(m, i0 + per);
    uint32_t tot;
    uint32_t eq_rank = 0;
    if (need_eq < n_eq_total) {  // ties at the threshold are cut: rank them in position order
      uint32_t neq = 0;
      for (uint32_t i = i0; i < i1; ++i) neq += ckey[i] == tau ? 1u : 0u;
      eq_rank = block_exclusive_scan(neq, wave_tot, &tot);
    }
    uint32_t nsel = 0;
    uint32_t flags = 0;  // per <= 8
    for (uint32_t i = i0; i < i1; ++i) {
      const uint32_t key = ckey[i];
      bool take = key > tau;
      if (key == tau) {
        take = need_eq >= n_eq_total || eq_rank < need_eq;
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
    if (recompute) {
      // every score of this head is needed now: compute them into the score array
      float* sw = scores_w + (size_t)bh * l;
      for (int row = t; row < n; row += kT) sw[row] = proxy_score_of_row(Arow, qh, r, row);
      __threadfence_block();
      __syncthreads();
    }
    uint32_t bin_unused;
    exact_select_from_scores<true>(s, n, k, vec_ok, (uint32_t)k, hist, bitmap, sel, wave_tot, res,
                             &bin_unused);
  }
  __syncthreads();
  for (int i = t; i < k; i += kT) sel_idx[(size_t)bh * k + i] = sel[i];
  if (!RESOLVE) return;

  // ---- resolution ------------------------------------------------------------------------------
  int32_t* __restrict__ so = slot_of + (size_t)bh * lrows;
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
  {
    // thread t owns the selected positions [t*jp, (t+1)*jp) (jp <= 4): one prefix count
    // ranks all misses in position order
    const int jp = (k + kT - 1) / kT;
    const int j0 = min(k, t * jp), j1 = min(k, j0 + jp);
    int32_t toks[4], slots[4];
    uint32_t nmine = 0;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int j = j0 + u;
      toks[u] = -1;
      slots[u] = 0;
      if (j < j1) {
        toks[u] = sel[j];
        int32_t slot = so[toks[u]];
        if (slot >= C) slot = -1;  // corrupt map entry: treat as absent
        slots[u] = slot;
        nmine += slot < 0 ? 1u : 0u;
      }
    }
    uint32_t tot;
    uint32_t rank = block_exclusive_scan(nmine, wave_tot, &tot);
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int j = j0 + u;
      if (j >= j1) continue;
      if (slots[u] >= 0) {
        ss[j] = slots[u];
        ht[j] = 1;
        lu[slots[u]] = step;
        lu_s[slots[u]] = step;  // used in this step: never a victim
      } else {
        ht[j] = 0;
        mt[rank] = toks[u];
        sel[j] = -(int32_t)rank - 2;  // remember the rank; the slot is filled in below
        ++rank;
      }
    }
    if (t == 0) sh_nmiss = tot;
    __syncthreads();
  }
  const int nm = (int)sh_nmiss;
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
  if (t == 0) n_miss[bh] = sh_bad ? -1 : nm;
}

constexpr size_t kLdsLimit = 150 * 1024;

template <bool RESOLVE>
hipError_t raise_lds_limit() {
  static std::atomic<uint64_t> done{0};
  return raise_dynamic_lds_once(select_resolve_kernel<RESOLVE>, kLdsLimit, done);
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
  LRQK_LAUNCH((select_resolve_kernel<false>), dim3(s.B * s.Hq), dim3(kT), lds, st, scores,
                     nullptr, 0, nullptr, nullptr, nullptr, nullptr, s.r, s.Hq, s.Hkv, s.l,
                     row_cap(s), n, s.k, sel_idx, 0, s.C, nullptr, nullptr, nullptr, nullptr,
                     nullptr, nullptr, nullptr, nullptr);
  return hipGetLastError();
}

hipError_t launch_select_resolve(const lrqk_shape& s, float* scores,
                                 const unsigned long long* ext_bitmap, const float* cand_scores,
                                 const float* A_K, const float* q_hat, int32_t* sel_idx,
                                 int32_t step, int32_t* slot_of, int32_t* token_of,
                                 int32_t* last_used, int32_t* sel_slot, uint8_t* hit,
                                 int32_t* miss_tok, int32_t* miss_slot, int32_t* n_miss,
                                 hipStream_t st) {
  const int n = s.l - s.w;
  const size_t lds = arena_sizes(s.k, n, s.C, true).total;
  hipError_t e = raise_lds_limit<true>();
  if (e != hipSuccess) return e;
  LRQK_LAUNCH((select_resolve_kernel<true>), dim3(s.B * s.Hq), dim3(kT), lds, st, scores,
                     reinterpret_cast<const uint32_t*>(ext_bitmap), 2 * filter_words64(n),
                     cand_scores, ext_bitmap ? A_K : nullptr, q_hat, scores, s.r, s.Hq, s.Hkv, s.l,
                     row_cap(s), n, s.k, sel_idx, step, s.C, slot_of, token_of, last_used,
                     sel_slot, hit, miss_tok, miss_slot, n_miss);
  return hipGetLastError();
}

}  // namespace lrqk
