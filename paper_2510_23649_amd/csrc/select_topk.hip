// a2 — active-token selection: the k largest proxy scores over positions [0, l-w),
// equal scores ordered by lower position, listed in ascending position
// (Alg. 2, top(., k); Sec. 4.1 active tokens; the lite window is implicit).
//
// Exact radix selection on an order-preserving 32-bit key, spread over many
// workgroups per head so that a batch-1 step still fills the chip:
//   1. histogram of the top 12 key bits (LDS atomics per workgroup, merged with
//      global atomics); the last workgroup of a head to finish scans the 4096
//      bins from the top and records the bin holding the k-th largest score;
//   2. one more pass over the scores: positions in higher bins are certain
//      members (appended unordered), positions in the threshold bin become
//      candidates (key, position);
//   3. one workgroup per head sorts the candidates by (key descending, position
//      ascending), takes what is still needed, and sorts the k positions.
// If a head has more candidates than the buffer holds (massive ties), step 3
// refines the threshold over the remaining 20 key bits from the scores
// themselves; the result is the same, only slower.
// Everything is integer work on keys, so the result does not depend on the
// order in which workgroups or atomics run.
#include "lrqk_device.h"
#include "lrqk_internal.h"

namespace lrqk {
namespace {

constexpr int kSelThreads = 256;
constexpr int kSelChunk = 4096;      // scores per workgroup in passes 1 and 2
constexpr int kFinThreads = 1024;

using dev::bitonic_sort_lds;
using dev::order_key;

__device__ __forceinline__ uint32_t load_u32_coherent(const uint32_t* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__global__ __launch_bounds__(256) void select_zero_kernel(uint32_t* hist, uint32_t* counters,
                                                          int n_hist, int n_counters) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n_hist) hist[i] = 0u;
  if (i < n_counters) counters[i] = 0u;
}

__global__ __launch_bounds__(kSelThreads) void select_hist_kernel(
    const float* __restrict__ scores, int l, int n, int k, uint32_t* __restrict__ hist,
    uint32_t* __restrict__ counters) {
  __shared__ uint32_t h[kBins];
  __shared__ uint32_t scan_buf[256];
  __shared__ int is_last;
  const int bh = blockIdx.y, t = threadIdx.x;
  const float* __restrict__ s = scores + (size_t)bh * l;
  for (int i = t; i < kBins; i += kSelThreads) h[i] = 0u;
  __syncthreads();
  const int c0 = blockIdx.x * kSelChunk;
  const int c1 = min(n, c0 + kSelChunk);
  for (int i = c0 + t; i < c1; i += kSelThreads) atomicAdd(&h[order_key(s[i]) >> kBinShift], 1u);
  __syncthreads();
  uint32_t* __restrict__ gh = hist + (size_t)bh * kBins;
  for (int i = t; i < kBins; i += kSelThreads) {
    const uint32_t c = h[i];
    if (c) atomicAdd(&gh[i], c);
  }
  __threadfence();
  __syncthreads();
  if (t == 0) {
    const uint32_t ticket = atomicAdd(&counters[bh * 8 + 0], 1u);
    is_last = (ticket == gridDim.x - 1);
  }
  __syncthreads();
  if (!is_last) return;
  __threadfence();
  // bins of thread t: [16t, 16t+16); suffix sums from the top bin down
  uint32_t loc[16];
  uint32_t sum = 0;
#pragma unroll
  for (int j = 0; j < 16; ++j) {
    loc[j] = load_u32_coherent(&gh[t * 16 + j]);
    sum += loc[j];
  }
  // inclusive scan over reversed thread order gives sum over threads >= t
  const int rt = 255 - t;
  scan_buf[rt] = sum;
  __syncthreads();
  for (int off = 1; off < 256; off <<= 1) {
    const uint32_t add = rt >= off ? scan_buf[rt - off] : 0u;
    __syncthreads();
    scan_buf[rt] += add;
    __syncthreads();
  }
  uint32_t running = scan_buf[rt] - sum;  // count in bins above this thread's bins
#pragma unroll
  for (int j = 15; j >= 0; --j) {
    const uint32_t before = running;
    running += loc[j];
    if (running >= (uint32_t)k && before < (uint32_t)k) {
      counters[bh * 8 + 4] = (uint32_t)(t * 16 + j);
      counters[bh * 8 + 5] = before;
    }
  }
}

__global__ __launch_bounds__(kSelThreads) void select_collect_kernel(
    const float* __restrict__ scores, int l, int n, int k, uint32_t* __restrict__ counters,
    int32_t* __restrict__ out_list, uint64_t* __restrict__ cand) {
  __shared__ uint32_t blk_above, blk_cand, base_above, base_cand;
  const int bh = blockIdx.y, t = threadIdx.x;
  const float* __restrict__ s = scores + (size_t)bh * l;
  const uint32_t bin = counters[bh * 8 + 4];
  if (t == 0) {
    blk_above = 0u;
    blk_cand = 0u;
  }
  __syncthreads();
  constexpr int PER = kSelChunk / kSelThreads;  // 16
  const int c0 = blockIdx.x * kSelChunk;
  uint32_t key[PER];
  uint32_t na = 0, nc = 0;
#pragma unroll
  for (int j = 0; j < PER; ++j) {
    const int i = c0 + j * kSelThreads + t;
    key[j] = i < n ? order_key(s[i]) : 0u;  // key 0 is below every real key's bin unless bin == 0
    const uint32_t b = key[j] >> kBinShift;
    const bool valid = i < n;
    na += (valid && b > bin) ? 1u : 0u;
    nc += (valid && b == bin) ? 1u : 0u;
  }
  const uint32_t off_a = na ? atomicAdd(&blk_above, na) : 0u;
  const uint32_t off_c = nc ? atomicAdd(&blk_cand, nc) : 0u;
  __syncthreads();
  if (t == 0) {
    base_above = blk_above ? atomicAdd(&counters[bh * 8 + 2], blk_above) : 0u;
    base_cand = blk_cand ? atomicAdd(&counters[bh * 8 + 3], blk_cand) : 0u;
  }
  __syncthreads();
  uint32_t pa = base_above + off_a, pc = base_cand + off_c;
  int32_t* __restrict__ ol = out_list + (size_t)bh * k;
  uint64_t* __restrict__ cd = cand + (size_t)bh * kCandCap;
#pragma unroll
  for (int j = 0; j < PER; ++j) {
    const int i = c0 + j * kSelThreads + t;
    if (i >= n) continue;
    const uint32_t b = key[j] >> kBinShift;
    if (b > bin) {
      if (pa < (uint32_t)k) ol[pa] = i;
      ++pa;
    } else if (b == bin) {
      if (pc < (uint32_t)kCandCap) cd[pc] = ((uint64_t)(~key[j]) << 32) | (uint32_t)i;
      ++pc;
    }
  }
}

// Block-wide exclusive prefix of a 0/1 flag in thread order, plus the block total.
__device__ __forceinline__ uint32_t block_rank_of_flag(bool flag, uint32_t* wave_counts,
                                                       uint32_t* total) {
  const unsigned long long m = __ballot(flag);
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int nw = blockDim.x >> 6;
  if (lane == 0) wave_counts[wv] = (uint32_t)__popcll(m);
  __syncthreads();
  uint32_t before = 0, tot = 0;
  for (int i = 0; i < nw; ++i) {
    const uint32_t c = wave_counts[i];
    before += i < wv ? c : 0u;
    tot += c;
  }
  __syncthreads();
  *total = tot;
  return before + (uint32_t)__popcll(m & ((1ull << lane) - 1ull));
}

__global__ __launch_bounds__(kFinThreads) void select_finalize_kernel(
    const float* __restrict__ scores, int l, int n, int k, uint32_t* __restrict__ counters,
    const int32_t* __restrict__ out_list, const uint64_t* __restrict__ cand,
    int32_t* __restrict__ sel_idx) {
  __shared__ uint64_t cbuf[kCandCap];
  __shared__ int32_t obuf[kMaxK];
  __shared__ uint32_t sub_hist[1024];
  __shared__ uint32_t wave_counts[kFinThreads / 64];
  __shared__ uint32_t sh_a, sh_b, sh_c;
  const int bh = blockIdx.x, t = threadIdx.x;
  const float* __restrict__ s = scores + (size_t)bh * l;
  const uint32_t bin = counters[bh * 8 + 4];
  const int n_above = (int)counters[bh * 8 + 5];
  const int n_cand = (int)counters[bh * 8 + 3];
  const int need = k - n_above;  // >= 1, all taken from the threshold bin
  const int kpad = max(2, (int)(1u << (32 - __clz(k - 1))));

  for (int i = t; i < kpad; i += kFinThreads)
    obuf[i] = i < n_above ? out_list[(size_t)bh * k + i] : 0x7fffffff;

  if (n_cand <= kCandCap) {
    const int cpad = max(2, (int)(1u << (32 - __clz(max(n_cand, 2) - 1))));
    for (int i = t; i < cpad; i += kFinThreads)
      cbuf[i] = i < n_cand ? cand[(size_t)bh * kCandCap + i] : ~0ull;
    bitonic_sort_lds(cbuf, cpad);
    for (int i = t; i < need; i += kFinThreads) obuf[n_above + i] = (int32_t)(uint32_t)cbuf[i];
  } else {
    // Refine the threshold inside the threshold bin from the scores themselves:
    // two 10-bit levels over the low 20 key bits.
    uint32_t prefix = bin;       // known high bits of the threshold key
    int shift = kBinShift;       // number of low bits still unknown
    uint32_t remaining = (uint32_t)need;
    for (int level = 0; level < 2; ++level) {
      for (int i = t; i < 1024; i += kFinThreads) sub_hist[i] = 0u;
      __syncthreads();
      const int nshift = shift - 10;
      for (int i = t; i < n; i += kFinThreads) {
        const uint32_t key = order_key(s[i]);
        if ((key >> shift) == prefix) atomicAdd(&sub_hist[(key >> nshift) & 1023u], 1u);
      }
      __syncthreads();
      if (t == 0) {  // 1024 bins: a serial scan from the top is cheap enough for this rare path
        uint32_t run = 0;
        int b = 1023;
        for (; b > 0; --b) {
          if (run + sub_hist[b] >= remaining) break;
          run += sub_hist[b];
        }
        sh_a = (uint32_t)b;
        sh_b = remaining - run;
      }
      __syncthreads();
      prefix = (prefix << 10) | sh_a;
      remaining = sh_b;
      shift = nshift;
      __syncthreads();
    }
    const uint32_t tau = prefix;       // exact key of the k-th largest score
    const uint32_t need_eq = remaining;  // how many positions with key == tau are taken (lowest first)
    if (t == 0) {
      sh_a = (uint32_t)n_above;  // write cursor for keys strictly above tau inside the bin
      sh_c = 0u;                 // positions with key == tau taken so far
    }
    __syncthreads();
    const int gt_base = n_above;
    const int eq_base = k - (int)need_eq;
    (void)gt_base;
    for (int i0 = 0; i0 < n; i0 += kFinThreads) {
      const int i = i0 + t;
      uint32_t key = 0u;
      bool in_bin = false;
      if (i < n) {
        key = order_key(s[i]);
        in_bin = (key >> kBinShift) == bin;
      }
      if (in_bin && key > tau) obuf[atomicAdd(&sh_a, 1u)] = i;
      const bool eq = in_bin && key == tau;
      uint32_t tot;
      const uint32_t rank = block_rank_of_flag(eq, wave_counts, &tot);
      const uint32_t taken = sh_c;
      if (eq && taken + rank < need_eq) obuf[eq_base + (int)(taken + rank)] = i;
      __syncthreads();
      if (t == 0) sh_c = taken + tot;
      __syncthreads();
    }
  }
  bitonic_sort_lds(obuf, kpad);
  for (int i = t; i < k; i += kFinThreads) sel_idx[(size_t)bh * k + i] = obuf[i];
}

}  // namespace

SelectWs carve_select_ws(void* base, int BHq, int k) {
  SelectWs ws;
  char* p = static_cast<char*>(base);
  size_t off = 0;
  ws.hist = reinterpret_cast<uint32_t*>(p + off);
  off += round_up((size_t)BHq * kBins * sizeof(uint32_t), 256);
  ws.counters = reinterpret_cast<uint32_t*>(p + off);
  off += round_up((size_t)BHq * 8 * sizeof(uint32_t), 256);
  ws.out_list = reinterpret_cast<int32_t*>(p + off);
  off += round_up((size_t)BHq * k * sizeof(int32_t), 256);
  ws.cand = reinterpret_cast<uint64_t*>(p + off);
  off += round_up((size_t)BHq * kCandCap * sizeof(uint64_t), 256);
  ws.bytes = off;
  return ws;
}

hipError_t launch_select_topk(const lrqk_shape& s, const float* scores, int32_t* sel_idx,
                              const SelectWs& ws, hipStream_t st) {
  const int BHq = s.B * s.Hq;
  const int n = s.l - s.w;
  const int n_hist = BHq * kBins, n_cnt = BHq * 8;
  LRQK_LAUNCH(select_zero_kernel, dim3(ceil_div(n_hist, 256)), dim3(256), 0, st, ws.hist,
                     ws.counters, n_hist, n_cnt);
  const dim3 grid(ceil_div(n, kSelChunk), BHq);
  LRQK_LAUNCH(select_hist_kernel, grid, dim3(kSelThreads), 0, st, scores, s.l, n, s.k,
                     ws.hist, ws.counters);
  LRQK_LAUNCH(select_collect_kernel, grid, dim3(kSelThreads), 0, st, scores, s.l, n, s.k,
                     ws.counters, ws.out_list, ws.cand);
  LRQK_LAUNCH(select_finalize_kernel, dim3(BHq), dim3(kFinThreads), 0, st, scores, s.l, n,
                     s.k, ws.counters, ws.out_list, ws.cand, sel_idx);
  return hipGetLastError();
}

}  // namespace lrqk
