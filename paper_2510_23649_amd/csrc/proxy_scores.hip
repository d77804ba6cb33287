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
#include "lrqk_internal.h"

namespace lrqk {
namespace {

constexpr int kTileRows = 256;

typedef float v4f __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 load_streaming(const float4* p) {
  const v4f x = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(p));
  return make_float4(x.x, x.y, x.z, x.w);
}

template <int R, int G>
__global__ __launch_bounds__(kTileRows) void proxy_scores_kernel(
    const float* __restrict__ A_K, const float* __restrict__ q_hat, float* __restrict__ scores,
    int l, int Hq, int Hkv) {
  constexpr int V4 = R / 4;       // 16-byte chunks per row
  constexpr int ROW4 = V4 + 1;    // padded LDS row stride in 16-byte units
  __shared__ float4 tile[kTileRows * ROW4];

  const int bkv = blockIdx.y;
  const int b = bkv / Hkv, kv = bkv - b * Hkv;
  const float* __restrict__ A = A_K + (size_t)bkv * (size_t)l * R;
  const float* __restrict__ qh = q_hat + ((size_t)b * Hq + (size_t)kv * G) * R;
  float* __restrict__ sc = scores + ((size_t)b * Hq + (size_t)kv * G) * (size_t)l;
  const int t = threadIdx.x;
  const int row0 = blockIdx.x * kTileRows;
  const float4* __restrict__ src = reinterpret_cast<const float4*>(A + (size_t)row0 * R);
  const int nvalid = min(kTileRows, l - row0) * V4;

  float4 pre[V4];
#pragma unroll
  for (int i = 0; i < V4; ++i) {
    const int idx = i * kTileRows + t;
    pre[i] = idx < nvalid ? load_streaming(src + idx) : make_float4(0.f, 0.f, 0.f, 0.f);
  }
#pragma unroll
  for (int i = 0; i < V4; ++i) {
    const int idx = i * kTileRows + t;
    tile[(idx / V4) * ROW4 + (idx % V4)] = pre[i];
  }
  __syncthreads();

  float acc[G];
#pragma unroll
  for (int g = 0; g < G; ++g) acc[g] = 0.0f;
#pragma unroll
  for (int c = 0; c < V4; ++c) {
    const float4 a = tile[t * ROW4 + c];
#pragma unroll
    for (int g = 0; g < G; ++g) {
      acc[g] = __builtin_fmaf(a.x, qh[g * R + 4 * c + 0], acc[g]);
      acc[g] = __builtin_fmaf(a.y, qh[g * R + 4 * c + 1], acc[g]);
      acc[g] = __builtin_fmaf(a.z, qh[g * R + 4 * c + 2], acc[g]);
      acc[g] = __builtin_fmaf(a.w, qh[g * R + 4 * c + 3], acc[g]);
    }
  }
  const int row = row0 + t;
  if (row < l) {
#pragma unroll
    for (int g = 0; g < G; ++g) sc[(size_t)g * l + row] = acc[g];
  }
}

// Any r (multiple of 4, <= 128) and any G <= 8: tiles of 64 rows; the four
// waves of a workgroup split the heads of the group between them.
constexpr int kGenRows = 64;
__global__ __launch_bounds__(256) void proxy_scores_generic_kernel(
    const float* __restrict__ A_K, const float* __restrict__ q_hat, float* __restrict__ scores,
    int l, int r, int Hq, int Hkv, int G, int tiles_per_block) {
  extern __shared__ float4 gtile[];  // kGenRows * (r/4 + 1)
  const int V4 = r / 4, ROW4 = V4 + 1;
  const int bkv = blockIdx.y;
  const int b = bkv / Hkv, kv = bkv - b * Hkv;
  const float* __restrict__ A = A_K + (size_t)bkv * (size_t)l * r;
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

template <int R, int G>
hipError_t launch_fast(const lrqk_shape& s, const float* A_K, const float* q_hat, float* scores,
                       hipStream_t st) {
  dim3 grid(ceil_div(s.l, kTileRows), s.B * s.Hkv);
  hipLaunchKernelGGL((proxy_scores_kernel<R, G>), grid, dim3(kTileRows), 0, st, A_K, q_hat,
                     scores, s.l, s.Hq, s.Hkv);
  return hipGetLastError();
}

template <int R>
hipError_t dispatch_G(const lrqk_shape& s, const float* A_K, const float* q_hat, float* scores,
                      hipStream_t st, bool* handled) {
  *handled = true;
  switch (s.Hq / s.Hkv) {
    case 1: return launch_fast<R, 1>(s, A_K, q_hat, scores, st);
    case 2: return launch_fast<R, 2>(s, A_K, q_hat, scores, st);
    case 4: return launch_fast<R, 4>(s, A_K, q_hat, scores, st);
    case 7: return launch_fast<R, 7>(s, A_K, q_hat, scores, st);
    case 8: return launch_fast<R, 8>(s, A_K, q_hat, scores, st);
    default: *handled = false; return hipSuccess;
  }
}

}  // namespace

hipError_t launch_proxy_scores(const lrqk_shape& s, const float* A_K, const float* q_hat,
                               float* scores, hipStream_t st) {
  bool handled = false;
  hipError_t e = hipSuccess;
  switch (s.r) {
    case 16: e = dispatch_G<16>(s, A_K, q_hat, scores, st, &handled); break;
    case 32: e = dispatch_G<32>(s, A_K, q_hat, scores, st, &handled); break;
    case 64: e = dispatch_G<64>(s, A_K, q_hat, scores, st, &handled); break;
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
  hipLaunchKernelGGL(proxy_scores_generic_kernel, grid, dim3(256), lds, st, A_K, q_hat, scores,
                     s.l, s.r, s.Hq, s.Hkv, s.Hq / s.Hkv, tiles_per_block);
  return hipGetLastError();
}

}  // namespace lrqk
