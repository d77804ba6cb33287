// a1 — proxy attention scores s = A_K q_hat^T (Alg. 2, "compute proxy attention").
//
// The only work of a decode step that grows with the context length l: a
// stream over the l x r key factor of every KV head.  It is bound by HBM reads
// (r*4 bytes per row against 2*G*r flops), so the kernel is organised around
// memory traffic:
//   * a workgroup owns one tile of 256 consecutive rows (256*r floats, one
//     contiguous span) and reads it with fully coalesced 16-byte loads; A_K is
//     touched once per step, so the loads are non-temporal;
//   * the tile goes through LDS (row stride r+4 floats, so that 16-byte row
//     reads by neighbouring lanes fall on different banks) to turn "lane =
//     16-byte chunk" into "lane = row";
//   * each lane then owns one row and runs, for each of the G query heads that
//     share the KV head, one fp32 fused-multiply-add chain over j = 0..r-1.
//     A_K is read once for the whole group; q_hat is wave-uniform;
//   * scores leave as 256-byte coalesced stores, one per head.
// Many small workgroups (l/256 per KV head, several resident per CU) hide the
// load -> LDS -> compute chain of each other; measured on MI355X this beats fewer
// workgroups that loop over tiles with a register prefetch.
// The chain order (j ascending from 0.0f) makes the scores bit-reproducible.
#include <hip/hip_runtime.h>

#include "lrqk_device.h"
#include "lrqk_internal.h"

namespace lrqk {
namespace {

constexpr int kTileRows = 256;

typedef float v4f __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 load_streaming(const float4* p) {
  const v4f x = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(p));
  return make_float4(x.x, x.y, x.z, x.w);
}

// FILTER: emit, INSTEAD of the scores, a bitmap per head of the positions in [0, n) whose
// order key is >= thr[head] (one 64-bit ballot per wavefront and head, no atomics) and
// the scores of those candidates, packed in position order into a slot of
// kCandPerGroup floats per 64-row group (the i-th set bit of the group's ballot goes to
// entry i; a group with more candidates than the slot holds keeps the first ones and
// the selection kernel recomputes the others from A_K).  The fused step therefore never
// writes the l-sized score array: about 5 MB leave this kernel instead of 16.8 MB at
// l = 131072.
// The threshold key of a head comes either from thr (keys estimated from a sample for this
// very q_hat) or, when thr_norm is given, from the value the selection of the layer's previous
// step left behind: thr_norm[head] * |q_hat[head]| (a NaN there gives a key above every score:
// no candidates, and the selection falls back to its exact route).  The keys used are written
// to thr_out by the first workgroup of each KV head.
template <int R, int G, bool FILTER>
__global__ __launch_bounds__(kTileRows) void proxy_scores_kernel(
    const float* __restrict__ A_K, const float* __restrict__ q_hat, float* __restrict__ scores,
    int l, int lrows, int Hq, int Hkv, int n, const uint32_t* __restrict__ thr,
    const float* __restrict__ thr_norm, uint32_t* __restrict__ thr_out,
    unsigned long long* __restrict__ bitmap, float* __restrict__ cand_scores, int words64) {
  // The tile goes through LDS in column phases of CH floats; the fma chain simply continues
  // from one phase to the next, in the same order.  Every supported rank takes one phase: at
  // r = 64 two phases of 32 columns (half the LDS, twice the resident workgroups, one more pair
  // of barriers) measured 2.5 % slower, four phases of 16 columns 50 % slower.
  constexpr int CH = R;                // columns per phase
  constexpr int NPH = R / CH;          // phases
  constexpr int V4 = CH / 4;           // 16-byte chunks per row and phase
  constexpr int ROW4 = V4 + 1;         // padded LDS row stride in 16-byte units
  static_assert(R % CH == 0, "rank must be a multiple of the phase width");
  __shared__ float4 tile[kTileRows * ROW4];
  // threshold key of head g: kept in the padding chunk of tile row 255 - g, which neither the
  // tile stores nor the staging of the packed scores below touch (no LDS of its own: the
  // number of resident workgroups is set by the tile)
  auto thr_slot = [&](int g) {
    return reinterpret_cast<uint32_t*>(&tile[(kTileRows - 1 - g) * ROW4 + V4]);
  };

  const int bkv = blockIdx.y;
  const int b = bkv / Hkv, kv = bkv - b * Hkv;
  const float* __restrict__ A = A_K + (size_t)bkv * (size_t)lrows * R;
  const float* __restrict__ qh = q_hat + ((size_t)b * Hq + (size_t)kv * G) * R;
  float* __restrict__ sc = scores + ((size_t)b * Hq + (size_t)kv * G) * (size_t)l;
  const int t = threadIdx.x;
  const int row0 = blockIdx.x * kTileRows;
  const float4* __restrict__ src = reinterpret_cast<const float4*>(A + (size_t)row0 * R);
  const int rows_valid = min(kTileRows, l - row0);

  const size_t bh0 = (size_t)b * Hq + (size_t)kv * G;  // first head of the group
  // all phases' loads are issued up front: chunk idx of phase p is row idx / V4,
  // 16-byte column p * V4 + idx % V4 (8 lanes read 128 contiguous bytes of a row)
  float4 pre[NPH][V4];
#pragma unroll
  for (int p = 0; p < NPH; ++p)
#pragma unroll
    for (int i = 0; i < V4; ++i) {
      const int idx = i * kTileRows + t;
      const int rr = idx / V4, cc = idx % V4;
      pre[p][i] = rr < rows_valid ? load_streaming(src + (size_t)rr * (R / 4) + p * V4 + cc)
                                  : make_float4(0.f, 0.f, 0.f, 0.f);
    }

  // (the tile's loads stay ahead of what follows: it is meant to run in their shadow)
  __builtin_amdgcn_sched_barrier(0);
  // Threshold key of each head of the group.  With carried thresholds |q_hat| is needed:
  // q_hat is wave-uniform (scalar loads, the same ones the products below use), so the squares
  // are summed with no memory instruction of their own while the tile's loads are in flight --
  // the heads dealt out over the four wavefronts, which keeps this off the workgroup's
  // critical path -- and the keys are handed to everyone through LDS (published by the
  // barrier that follows the tile store).
  if (FILTER) {
    const int wv = t >> 6;
#pragma unroll
    for (int g = 0; g < G; ++g) {
      if ((g & 3) != wv) continue;  // wave-uniform
      uint32_t key;
      if (thr_norm != nullptr) {
        float q2 = 0.0f;
#pragma unroll
        for (int j = 0; j < R; ++j) q2 = __builtin_fmaf(qh[g * R + j], qh[g * R + j], q2);
        const float tf = thr_norm[bh0 + g] * __builtin_sqrtf(q2);
        key = (tf != tf) ? 0xffffffffu : dev::order_key(tf);
      } else {
        key = thr[bh0 + g];
      }
      if ((t & 63) == 0) *thr_slot(g) = key;
    }
  }

  float acc[G];
#pragma unroll
  for (int g = 0; g < G; ++g) acc[g] = 0.0f;
#pragma unroll
  for (int p = 0; p < NPH; ++p) {
    if (p > 0) __syncthreads();  // the previous phase has been consumed
#pragma unroll
    for (int i = 0; i < V4; ++i) {
      const int idx = i * kTileRows + t;
      tile[(idx / V4) * ROW4 + (idx % V4)] = pre[p][i];
    }
    __syncthreads();
#pragma unroll
    for (int c = 0; c < V4; ++c) {
      const float4 a = tile[t * ROW4 + c];
      const int j = p * CH + 4 * c;
#pragma unroll
      for (int g = 0; g < G; ++g) {
        acc[g] = __builtin_fmaf(a.x, qh[g * R + j + 0], acc[g]);
        acc[g] = __builtin_fmaf(a.y, qh[g * R + j + 1], acc[g]);
        acc[g] = __builtin_fmaf(a.z, qh[g * R + j + 2], acc[g]);
        acc[g] = __builtin_fmaf(a.w, qh[g * R + j + 3], acc[g]);
      }
    }
  }
  const int row = row0 + t;
  if (!FILTER) {
    if (row < l) {
#pragma unroll
      for (int g = 0; g < G; ++g) sc[(size_t)g * l + row] = acc[g];
    }
  } else {
    const int wrow = row0 + (t & ~63);  // first row of this wavefront
    const int lane = t & 63;
    // The 64 rows of the tile that this wavefront owns are read by no other wavefront, so
    // their LDS space can stage the packed candidate scores without a workgroup barrier.
    float* stage = reinterpret_cast<float*>(&tile[(t & ~63) * ROW4]);
    // The packed scores of all G heads are staged together and leave with one store
    // instruction (lane = head * 8 + entry), the G ballots with another (lane = head): the
    // per-head part is the compare, the ballot and one LDS write.
    static_assert(G * kCandPerGroup <= 64, "one lane per packed entry");
    if (lane < G * kCandPerGroup) stage[lane] = 0.0f;
    __builtin_amdgcn_wave_barrier();
    const unsigned long long below = (1ull << lane) - 1ull;
    const int my_head = lane >> 3;       // head of this lane in the two stores below
    unsigned long long mask_of_my_head = 0ull, mask_of_lane_head = 0ull;
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const uint32_t thr_g = *thr_slot(g);
      if (blockIdx.x == 0 && t == 0) thr_out[bh0 + g] = thr_g;
      const bool in = row < n && dev::order_key(acc[g]) >= thr_g;
      const unsigned long long mask = __ballot(in);
      const int rank = __popcll(mask & below);
      if (in && rank < kCandPerGroup) stage[g * kCandPerGroup + rank] = acc[g];
      if (my_head == g) mask_of_my_head = mask;
      if (lane == g) mask_of_lane_head = mask;
    }
    __builtin_amdgcn_wave_barrier();
    if (wrow < n) {
      const size_t grp = (size_t)(wrow >> 6);
      if (lane < G) bitmap[(bh0 + lane) * words64 + grp] = mask_of_lane_head;
      // a head without candidates in this group leaves its entries alone (they are not read)
      if (lane < G * kCandPerGroup && mask_of_my_head != 0ull)
        cand_scores[((bh0 + my_head) * words64 + grp) * kCandPerGroup + (lane & 7)] = stage[lane];
    }
  }
}

// Sampled estimate of the selection threshold of every head, before the scores exist.
// Kernel 1: the proxy score of every SS-th row, kThrParts workgroups per (batch, query
// head): 8 lanes share a row (one 16-byte chunk each, partial sums added across the
// lanes -- the estimate does not need the exact rounding of the full pass), several rows'
// loads in flight per lane; the sample scores go to a small buffer.
// Kernel 2: one workgroup per head histograms the head's sample keys (top 12 bits, then
// 6 more inside the bin found) and writes the key below which a position is not expected
// among the k largest, with a margin of six standard deviations of the sample count
// (SS = 1 for short contexts: every row is sampled).
// The estimate only decides how many candidates the selection kernel gets; that kernel
// checks the count and derives everything exactly.  (Two launches rather than one with
// a "last workgroup" hand-over: the device-wide fences that hand-over needs cost far
// more on this chip than a launch.)
constexpr int kThrThreads = 1024;
constexpr int kThrParts = 8;
constexpr int kThrRowsPerIter = kThrThreads / 8;
constexpr int kThrBatch = 4;

__device__ __forceinline__ float sum8(float v) {
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xf, 0xf, false));
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xf, 0xf, false));
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x141, 0xf, 0xf, false));
  return v;
}

__global__ __launch_bounds__(kThrThreads) void proxy_sample_kernel(
    const float* __restrict__ A_K, const float* __restrict__ q_hat, int lrows, int r, int Hq,
    int Hkv, int SS, int ns, int parts, float* __restrict__ samples) {
  const int bh = blockIdx.y, part = blockIdx.x, t = threadIdx.x;
  const int b = bh / Hq, h = bh - b * Hq, kv = h / (Hq / Hkv);
  const float* __restrict__ A = A_K + ((size_t)b * Hkv + kv) * (size_t)lrows * r;
  const float* __restrict__ qh = q_hat + (size_t)bh * r;
  float* __restrict__ smp = samples + (size_t)bh * kThrMaxSamples;
  const int off = SS >> 1;
  const int V4 = r / 4;
  const int c = t & 7, rg = t >> 3;
  // this lane's chunks of q_hat: c, c+8, c+16, c+24 (r <= 128)
  float4 qv[4];
#pragma unroll
  for (int u = 0; u < 4; ++u)
    qv[u] = (c + 8 * u < V4) ? reinterpret_cast<const float4*>(qh)[c + 8 * u]
                             : make_float4(0.f, 0.f, 0.f, 0.f);
  const int per_part = (ns + parts - 1) / parts;
  const int j_begin = part * per_part, j_end = min(ns, j_begin + per_part);
  for (int j0 = j_begin; j0 < j_end; j0 += kThrRowsPerIter * kThrBatch) {
    float part_sum[kThrBatch];
#pragma unroll
    for (int u = 0; u < kThrBatch; ++u) {
      const int j = j0 + u * kThrRowsPerIter + rg;
      float acc = 0.0f;
      if (j < j_end) {
        const float4* __restrict__ row =
            reinterpret_cast<const float4*>(A + ((size_t)off + (size_t)j * SS) * r);
#pragma unroll
        for (int v = 0; v < 4; ++v)
          if (c + 8 * v < V4) {
            const float4 a = row[c + 8 * v];
            acc = __builtin_fmaf(a.x, qv[v].x, acc);
            acc = __builtin_fmaf(a.y, qv[v].y, acc);
            acc = __builtin_fmaf(a.z, qv[v].z, acc);
            acc = __builtin_fmaf(a.w, qv[v].w, acc);
          }
      }
      part_sum[u] = acc;
    }
#pragma unroll
    for (int u = 0; u < kThrBatch; ++u) {
      const float sc = sum8(part_sum[u]);
      const int j = j0 + u * kThrRowsPerIter + rg;
      if (c == 0 && j < j_end) smp[j] = sc;
    }
  }
}

__global__ __launch_bounds__(kThrThreads) void proxy_threshold_kernel(
    const float* __restrict__ samples, int n, int k, int SS, int ns, uint32_t* __restrict__ thr) {
  __shared__ uint32_t hist[kBins];
  __shared__ uint32_t wave_tot[16];
  __shared__ uint32_t res[4];
  const int bh = blockIdx.x, t = threadIdx.x;
  const float* __restrict__ smp = samples + (size_t)bh * kThrMaxSamples;
  for (int i = t; i < kBins; i += kThrThreads) hist[i] = 0u;
  __syncthreads();
  for (int j = t; j < ns; j += kThrThreads) {
    const float sc = smp[j];
    atomicAdd(&hist[dev::order_key(sc) >> kBinShift], 1u);
  }
  __syncthreads();
  uint32_t want = (uint32_t)k;
  if (SS > 1) {
    const uint32_t ks = (uint32_t)(((long long)k * ns + n - 1) / n);  // expected hits in the sample
    uint32_t sq = 1;
    while (sq * sq < ks) ++sq;
    want = ks + 6 * sq + 4;
  }
  uint32_t bin, above;
  dev::find_from_top_4096(hist, want, wave_tot, res, &bin, &above);
  // refine inside that bin with the next 6 key bits, so that the cut does not overshoot
  // by a whole 12-bit bin
  for (int i = t; i < 2048; i += kThrThreads) hist[i] = 0u;
  __syncthreads();
  for (int j = t; j < ns; j += kThrThreads) {
    const uint32_t key = dev::order_key(smp[j]);
    if ((key >> kBinShift) == bin) atomicAdd(&hist[(key >> 14) & 63u], 1u);
  }
  __syncthreads();
  dev::find_from_top(hist, want > above ? want - above : 1u, wave_tot, res);
  const uint32_t sub = res[0] == 0xffffffffu ? 0u : res[0];
  if (t == 0) thr[bh] = (bin << kBinShift) | (sub << 14);
}

// Any r (multiple of 4, <= 128) and any G <= 8: tiles of 64 rows; the four
// waves of a workgroup split the heads of the group between them.
constexpr int kGenRows = 64;
__global__ __launch_bounds__(256) void proxy_scores_generic_kernel(
    const float* __restrict__ A_K, const float* __restrict__ q_hat, float* __restrict__ scores,
    int l, int lrows, int r, int Hq, int Hkv, int G, int tiles_per_block) {
  extern __shared__ float4 gtile[];  // kGenRows * (r/4 + 1)
  const int V4 = r / 4, ROW4 = V4 + 1;
  const int bkv = blockIdx.y;
  const int b = bkv / Hkv, kv = bkv - b * Hkv;
  const float* __restrict__ A = A_K + (size_t)bkv * (size_t)lrows * r;
  const float* __restrict__ qh = q_hat + ((size_t)b * Hq + (size_t)kv * G) * r;
  float* __restrict__ sc = scores + ((size_t)b * Hq + (size_t)kv * G) * (size_t)l;
  const int t = threadIdx.x;
  const int lane_row = t & (kGenRows - 1);
  const int wave = t / kGenRows;  // 0..3
  const int n_tiles = (l + kGenRows - 1) / kGenRows;
  const int tile_begin = blockIdx.x * tiles_per_block;
  const int tile_end = min(n_tiles, tile_begin + tiles_per_block);
  for (int ti = tile_begin; ti < tile_end; ++ti) {
    const int row0 = ti * kGenRows;
    const float4* __restrict__ src = reinterpret_cast<const float4*>(A + (size_t)row0 * r);
    const int nvalid = min(kGenRows, l - row0) * V4;
    __syncthreads();
    for (int idx = t; idx < kGenRows * V4; idx += 256)
      gtile[(idx / V4) * ROW4 + (idx % V4)] =
          idx < nvalid ? src[idx] : make_float4(0.f, 0.f, 0.f, 0.f);
    __syncthreads();
    const int row = row0 + lane_row;
    for (int g = wave; g < G; g += 4) {
      float acc = 0.0f;
      for (int c = 0; c < V4; ++c) {
        const float4 a = gtile[lane_row * ROW4 + c];
        acc = __builtin_fmaf(a.x, qh[g * r + 4 * c + 0], acc);
        acc = __builtin_fmaf(a.y, qh[g * r + 4 * c + 1], acc);
        acc = __builtin_fmaf(a.z, qh[g * r + 4 * c + 2], acc);
        acc = __builtin_fmaf(a.w, qh[g * r + 4 * c + 3], acc);
      }
      if (row < l) sc[(size_t)g * l + row] = acc;
    }
  }
}

struct FilterOut {
  const uint32_t* thr;    // threshold keys (null: take them from thr_norm)
  const float* thr_norm;  // carried thresholds / |q_hat| (null: take the keys in thr)
  uint32_t* thr_out;      // keys used
  unsigned long long* bitmap;
  float* cand_scores;
};

template <int R, int G>
hipError_t launch_fast(const lrqk_shape& s, const float* A_K, const float* q_hat, float* scores,
                       const FilterOut* f, hipStream_t st) {
  dim3 grid(ceil_div(s.l, kTileRows), s.B * s.Hkv);
  const int n = s.l - s.w;
  if (f)
    LRQK_LAUNCH((proxy_scores_kernel<R, G, true>), grid, dim3(kTileRows), 0, st, A_K,
                       q_hat, scores, s.l, row_cap(s), s.Hq, s.Hkv, n, f->thr, f->thr_norm,
                       f->thr_out, f->bitmap, f->cand_scores, filter_words64(n));
  else
    LRQK_LAUNCH((proxy_scores_kernel<R, G, false>), grid, dim3(kTileRows), 0, st, A_K,
                       q_hat, scores, s.l, row_cap(s), s.Hq, s.Hkv, n, nullptr, nullptr, nullptr,
                       nullptr, nullptr, 0);
  return hipGetLastError();
}

template <int R>
hipError_t dispatch_G(const lrqk_shape& s, const float* A_K, const float* q_hat, float* scores,
                      const FilterOut* f, hipStream_t st, bool* handled) {
  *handled = true;
  switch (s.Hq / s.Hkv) {
    case 1: return launch_fast<R, 1>(s, A_K, q_hat, scores, f, st);
    case 2: return launch_fast<R, 2>(s, A_K, q_hat, scores, f, st);
    case 4: return launch_fast<R, 4>(s, A_K, q_hat, scores, f, st);
    case 7: return launch_fast<R, 7>(s, A_K, q_hat, scores, f, st);
    case 8: return launch_fast<R, 8>(s, A_K, q_hat, scores, f, st);
    default: *handled = false; return hipSuccess;
  }
}

}  // namespace

bool proxy_filter_supported(const lrqk_shape& s) {
  const int G = s.Hq / s.Hkv;
  return (s.r == 16 || s.r == 32 || s.r == 64) && (G == 1 || G == 2 || G == 4 || G == 7 || G == 8);
}

hipError_t launch_proxy_threshold(const lrqk_shape& s, const float* A_K, const float* q_hat,
                                  float* samples, uint32_t* thr, hipStream_t st) {
  const int n = s.l - s.w;
  // every SS-th row, 8192 .. 16384 samples per head once the context is long enough (with
  // fewer, the six-sigma margin of the estimate lets more than the selection's capacity through)
  int SS = 1;
  while (SS < 256 && n / (SS * 2) >= 8192) SS *= 2;
  if (n / SS >= kThrMaxSamples) SS *= 2;  // very long contexts: stay inside the sample buffer
  while (n / SS >= kThrMaxSamples) SS *= 2;
  const int off = SS >> 1;
  const int ns = n > off ? (n - off + SS - 1) / SS : 0;
  int parts = ceil_div(ns, 512);
  if (parts > kThrParts) parts = kThrParts;
  if (parts < 1) parts = 1;
  LRQK_LAUNCH(proxy_sample_kernel, dim3(parts, s.B * s.Hq), dim3(kThrThreads), 0, st, A_K,
                     q_hat, row_cap(s), s.r, s.Hq, s.Hkv, SS, ns, parts, samples);
  LRQK_LAUNCH(proxy_threshold_kernel, dim3(s.B * s.Hq), dim3(kThrThreads), 0, st, samples,
                     n, s.k, SS, ns, thr);
  return hipGetLastError();
}

hipError_t launch_proxy_scores_filter(const lrqk_shape& s, const float* A_K, const float* q_hat,
                                      float* scores, const uint32_t* thr, const float* thr_norm,
                                      uint32_t* thr_out, unsigned long long* bitmap,
                                      float* cand_scores, hipStream_t st) {
  if ((thr == nullptr) == (thr_norm == nullptr) || !thr_out) return hipErrorInvalidValue;
  const FilterOut f{thr, thr_norm, thr_out, bitmap, cand_scores};
  bool handled = false;
  hipError_t e = hipErrorInvalidValue;
  switch (s.r) {
    case 16: e = dispatch_G<16>(s, A_K, q_hat, scores, &f, st, &handled); break;
    case 32: e = dispatch_G<32>(s, A_K, q_hat, scores, &f, st, &handled); break;
    case 64: e = dispatch_G<64>(s, A_K, q_hat, scores, &f, st, &handled); break;
    default: break;
  }
  return handled ? e : hipErrorInvalidValue;
}

hipError_t launch_proxy_scores(const lrqk_shape& s, const float* A_K, const float* q_hat,
                               float* scores, hipStream_t st) {
  bool handled = false;
  hipError_t e = hipSuccess;
  switch (s.r) {
    case 16: e = dispatch_G<16>(s, A_K, q_hat, scores, nullptr, st, &handled); break;
    case 32: e = dispatch_G<32>(s, A_K, q_hat, scores, nullptr, st, &handled); break;
    case 64: e = dispatch_G<64>(s, A_K, q_hat, scores, nullptr, st, &handled); break;
    default: break;
  }
  if (handled) return e;
  const int n_tiles = ceil_div(s.l, kGenRows);
  const int bkv = s.B * s.Hkv;
  int tiles_per_block = 8;
  while (tiles_per_block > 1 && (long)ceil_div(n_tiles, tiles_per_block) * bkv < 2048)
    tiles_per_block >>= 1;
  dim3 grid(ceil_div(n_tiles, tiles_per_block), bkv);
  const size_t lds = (size_t)kGenRows * (s.r / 4 + 1) * sizeof(float4);
  LRQK_LAUNCH(proxy_scores_generic_kernel, grid, dim3(256), lds, st, A_K, q_hat, scores,
                     s.l, row_cap(s), s.r, s.Hq, s.Hkv, s.Hq / s.Hkv, tiles_per_block);
  return hipGetLastError();
}

}  // namespace lrqk
