// a3 — hit/miss resolution against the GPU-resident KV cache (Sec. 4.1: a token
// already in the GPU cache is a hit, only missing tokens are fetched; Sec. 5.3:
// miss rate = fetched rows / selected rows).
//
// The paper does this indexing on the CPU and names it as its bottleneck
// (Limitations); here it is one workgroup per (batch, query head), entirely in
// LDS.  Replacement rule for C >= k slots: least recently selected, ties by lower
// slot; the j-th miss in ascending position takes the j-th victim.
//   1. every selected token looks up slot_of: hits refresh last_used, misses get
//      their rank by a prefix count in position order;
//   2. the slots not used in this step are the victim candidates; their keys
//      (last_used + 1) << 32 | slot are sorted in LDS (all other slots sort last);
//   3. miss j takes sorted[j]: evict its token, install the new one.
// All of it is integer work with a fixed order, so the result is deterministic.
#include "lrqk_device.h"
#include "lrqk_internal.h"

namespace lrqk {
namespace {

using dev::bitonic_sort_lds;

constexpr int kResThreads = 1024;

__global__ __launch_bounds__(256) void fill_i32_kernel(int32_t* p, size_t n, int32_t v) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = v;
}

// dynamic LDS: uint64 keys[Cpad]
__global__ __launch_bounds__(kResThreads) void cache_resolve_kernel(
    const int32_t* __restrict__ sel_idx, int32_t step, int l, int lrows, int C, int Cpad, int k,
    int32_t* __restrict__ slot_of, int32_t* __restrict__ token_of,
    int32_t* __restrict__ last_used, int32_t* __restrict__ sel_slot, uint8_t* __restrict__ hit,
    int32_t* __restrict__ miss_tok, int32_t* __restrict__ miss_slot,
    int32_t* __restrict__ n_miss) {
  extern __shared__ uint64_t keys[];
  __shared__ uint32_t wave_counts[kResThreads / 64];
  __shared__ uint32_t sh_nmiss, sh_bad;
  const int bh = blockIdx.x, t = threadIdx.x;
  const int lane = t & 63, wv = t >> 6;
  const int32_t* __restrict__ sel = sel_idx + (size_t)bh * k;
  int32_t* __restrict__ so = slot_of + (size_t)bh * lrows;
  int32_t* __restrict__ to = token_of + (size_t)bh * C;
  int32_t* __restrict__ lu = last_used + (size_t)bh * C;
  int32_t* __restrict__ ss = sel_slot + (size_t)bh * k;
  uint8_t* __restrict__ ht = hit + (size_t)bh * k;
  int32_t* __restrict__ mt = miss_tok + (size_t)bh * k;
  int32_t* __restrict__ ms = miss_slot + (size_t)bh * k;

  if (t == 0) {
    sh_nmiss = 0u;
    sh_bad = 0u;
  }
  // victim keys from the state before this step; slots hit below are taken out afterwards
  for (int s = t; s < Cpad; s += kResThreads)
    keys[s] = s < C ? (((uint64_t)(uint32_t)(lu[s] + 1)) << 32) | (uint32_t)s : ~0ull;
  __syncthreads();

  // pass over the selected tokens in position order, kResThreads at a time
  for (int j0 = 0; j0 < k; j0 += kResThreads) {
    const int j = j0 + t;
    int32_t tok = -1, slot = -1;
    bool valid = false, miss = false;
    if (j < k) {
      tok = sel[j];
      valid = tok >= 0 && tok < l;
      if (valid) slot = so[tok];
      if (valid && slot >= C) slot = -1;  // corrupt map entry: treat as absent
      miss = valid && slot < 0;
      if (!valid) {
        atomicOr(&sh_bad, 1u);
        ss[j] = -1;
        ht[j] = 0;
      } else if (!miss) {
        ss[j] = slot;
        ht[j] = 1;
        lu[slot] = step;
        keys[slot] = ~0ull;  // used in this step: never a victim
      } else {
        ht[j] = 0;
      }
    }
    // rank of this miss among all misses, in position order
    const unsigned long long m = __ballot(miss);
    if (lane == 0) wave_counts[wv] = (uint32_t)__popcll(m);
    __syncthreads();
    uint32_t before = sh_nmiss, tot = 0;
    for (int i = 0; i < kResThreads / 64; ++i) {
      const uint32_t c = wave_counts[i];
      before += i < wv ? c : 0u;
      tot += c;
    }
    const uint32_t rank = before + (uint32_t)__popcll(m & ((1ull << lane) - 1ull));
    if (miss) {
      mt[rank] = tok;
      ss[j] = -(int32_t)rank - 2;  // remember the rank; replaced by the slot below
    }
    __syncthreads();
    if (t == 0) sh_nmiss += tot;
    __syncthreads();
  }
  const int nm = (int)sh_nmiss;
  if (nm > 0) {
    // a slot whose last_used already equals `step` (step reused by the caller) is protected too
    for (int s = t; s < C; s += kResThreads)
      if (keys[s] != ~0ull && (int32_t)(keys[s] >> 32) - 1 == step) keys[s] = ~0ull;
    bitonic_sort_lds(keys, Cpad);
    for (int j = t; j < nm; j += kResThreads) {
      const uint64_t key = keys[j];
      const int32_t tok = mt[j];
      if (key == ~0ull) {  // ran out of victims
        atomicOr(&sh_bad, 1u);
        ms[j] = -1;
        continue;
      }
      const int32_t s = (int32_t)(uint32_t)key;
      const int32_t old = to[s];
      if (old >= 0 && old < l) so[old] = -1;
      to[s] = tok;
      so[tok] = s;
      lu[s] = step;
      ms[j] = s;
    }
    __syncthreads();
    // translate remembered ranks into slots
    for (int j = t; j < k; j += kResThreads) {
      const int32_t v = ss[j];
      if (v <= -2) ss[j] = ms[-(v + 2)];
    }
  }
  __syncthreads();
  if (t == 0) n_miss[bh] = sh_bad ? -1 : nm;
}

}  // namespace

hipError_t launch_fill_i32(int32_t* p, size_t n, int32_t v, hipStream_t st) {
  if (n == 0) return hipSuccess;
  LRQK_LAUNCH(fill_i32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, p, n, v);
  return hipGetLastError();
}

hipError_t launch_cache_init(const lrqk_shape& s, int32_t* slot_of, int32_t* token_of,
                             int32_t* last_used, hipStream_t st) {
  const size_t BHq = (size_t)s.B * s.Hq;
  const size_t n1 = BHq * row_cap(s), n2 = BHq * s.C;
  LRQK_LAUNCH(fill_i32_kernel, dim3((unsigned)((n1 + 255) / 256)), dim3(256), 0, st,
                     slot_of, n1, -1);
  LRQK_LAUNCH(fill_i32_kernel, dim3((unsigned)((n2 + 255) / 256)), dim3(256), 0, st,
                     token_of, n2, -1);
  LRQK_LAUNCH(fill_i32_kernel, dim3((unsigned)((n2 + 255) / 256)), dim3(256), 0, st,
                     last_used, n2, -1);
  return hipGetLastError();
}

hipError_t launch_cache_resolve(const lrqk_shape& s, const int32_t* sel_idx, int32_t step,
                                int32_t* slot_of, int32_t* token_of, int32_t* last_used,
                                int32_t* sel_slot, uint8_t* hit, int32_t* miss_tok,
                                int32_t* miss_slot, int32_t* n_miss, hipStream_t st) {
  const int Cpad = next_pow2(s.C < 2 ? 2 : s.C);
  const size_t lds = (size_t)Cpad * sizeof(uint64_t);
  if (lds > 48 * 1024) {  // large caches need the dynamic-LDS ceiling raised once
    static std::atomic<uint64_t> raised{0};
    const hipError_t e = raise_dynamic_lds_once(cache_resolve_kernel, 64 * 1024, raised);
    if (e != hipSuccess) return e;
  }
  LRQK_LAUNCH(cache_resolve_kernel, dim3(s.B * s.Hq), dim3(kResThreads), lds, st, sel_idx,
                     step, s.l, row_cap(s), s.C, Cpad, s.k, slot_of, token_of, last_used, sel_slot, hit,
                     miss_tok, miss_slot, n_miss);
  return hipGetLastError();
}

}  // namespace lrqk
