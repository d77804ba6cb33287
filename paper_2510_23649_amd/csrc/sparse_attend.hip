// a5 — exact softmax attention of one query over the k + w selected rows
// (Sec. 4.3: Attention(q_t, K_Omega, V_Omega) with the original q, K, V).
//
// One query row per head and 2*d flops per K/V element pair: the step is bound by
// the HBM reads of the selected rows (a random gather of d-element rows from the
// cache plus the contiguous lite rows).  Layout of the work:
//   * the k + w rows of a head are split over `nsplit` workgroups so that batch-1
//     steps still fill the chip; a workgroup of 4 wavefronts handles a contiguous
//     range of the row list;
//   * a row is read by 16 lanes, each taking one 16-byte (bf16) or 32-byte (fp32)
//     chunk of the K row and the same chunk of the V row, so a wavefront reads 4
//     rows per load instruction in full 256/512-byte segments; four such groups
//     of loads are issued before any is consumed;
//   * q.K is finished with a 16-lane rotate-and-add; every 16-lane group keeps its
//     own running (max, sum, acc[8 per lane]) so no cross-group traffic is needed
//     until the end, where the 4 groups and then the 4 wavefronts are merged;
//   * each workgroup writes one partial (m, s, acc[128]); a second small kernel
//     merges the partials of a head.
// Arithmetic is fp32 throughout; exp is exp2 on log2(e)-scaled logits.
#include "lrqk_internal.h"

namespace lrqk {
namespace {

constexpr int kAttThreads = 256;
constexpr int kRowsPerPass = 16;  // 4 wavefronts x 4 row groups
// passes whose loads are in flight together; with 16 rows a pass, a workgroup's minimal share is
// 32 rows (measured on rows that no cache holds: 32 rows a workgroup 11.7 us, 64 rows 13.2 us,
// 128 rows 16.4 us for the 33.8 MB of the 128K-context shape: many small workgroups win)
constexpr int kUnroll = 2;
constexpr float kLog2e = 1.4426950408889634f;

template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v) {
  return __int_as_float(
      __builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}
// sum over the 16 lanes of a DPP row; every lane of the row ends with the total
__device__ __forceinline__ float row16_allreduce_sum(float v) {
  v += dpp_f32<0x128>(v);  // row_ror:8
  v += dpp_f32<0x124>(v);  // row_ror:4
  v += dpp_f32<0x122>(v);  // row_ror:2
  v += dpp_f32<0x121>(v);  // row_ror:1
  return v;
}

struct Chunk8 {
  float v[8];
};

__device__ __forceinline__ Chunk8 unpack_bf16x8(const uint4 u) {
  Chunk8 c;
  c.v[0] = __uint_as_float(u.x << 16);
  c.v[1] = __uint_as_float(u.x & 0xffff0000u);
  c.v[2] = __uint_as_float(u.y << 16);
  c.v[3] = __uint_as_float(u.y & 0xffff0000u);
  c.v[4] = __uint_as_float(u.z << 16);
  c.v[5] = __uint_as_float(u.z & 0xffff0000u);
  c.v[6] = __uint_as_float(u.w << 16);
  c.v[7] = __uint_as_float(u.w & 0xffff0000u);
  return c;
}

typedef unsigned v4u __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));

// Loads the lane's 8-element chunk of a row.  BF16: 16 bytes; F32: 32 bytes.
template <bool BF16>
struct RowChunk;
template <>
struct RowChunk<true> {
  uint4 raw;
  __device__ __forceinline__ void load(const void* row, int c) {
    // a selected row is read once per step: streaming load
    const v4u x = __builtin_nontemporal_load(reinterpret_cast<const v4u*>(row) + c);
    raw = make_uint4(x.x, x.y, x.z, x.w);
  }
  __device__ __forceinline__ void store(void* row, int c) const {
    reinterpret_cast<uint4*>(row)[c] = raw;
  }
  __device__ __forceinline__ Chunk8 get() const { return unpack_bf16x8(raw); }
};
template <>
struct RowChunk<false> {
  float4 a, b;
  __device__ __forceinline__ void load(const void* row, int c) {
    const v4f x = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(row) + 2 * c);
    const v4f y = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(row) + 2 * c + 1);
    a = make_float4(x.x, x.y, x.z, x.w);
    b = make_float4(y.x, y.y, y.z, y.w);
  }
  __device__ __forceinline__ void store(void* row, int c) const {
    reinterpret_cast<float4*>(row)[2 * c] = a;
    reinterpret_cast<float4*>(row)[2 * c + 1] = b;
  }
  __device__ __forceinline__ Chunk8 get() const {
    Chunk8 o;
    o.v[0] = a.x; o.v[1] = a.y; o.v[2] = a.z; o.v[3] = a.w;
    o.v[4] = b.x; o.v[5] = b.y; o.v[6] = b.z; o.v[7] = b.w;
    return o;
  }
};

// kAttendAllFetch: rows that missed the cache are read straight from the pinned host store
// (device-visible host memory), used, and written into their cache slot on the way: the
// fetch leg and the attention become one kernel, so the host-link reads of the few missing
// rows overlap with the HBM reads of all the others.
struct FetchSrc {
  const char* K_host;       // [B,Hkv,lrows,d] rows
  const char* V_host;
  const int32_t* sel_idx;   // [B,Hq,k] position of each selected row
  int l;                    // context length
  int lrows;                // rows allocated per (batch, KV head)
};

struct AttendArgs {
  int mode;
  FetchSrc fs;
  const float* q;
  const void* cacheK;
  const void* cacheV;
  const int32_t* sel_slot;
  const uint8_t* hit;
  const int32_t* miss_slot;
  const int32_t* n_miss;
  const void* liteK;
  const void* liteV;
  float* partials;
  int Hq, Hkv, C, k, w, rows_per_block, parts_per_head, part_offset;
  float scale;
};

// One workgroup's share of a head's row list: block bx of head bh.
template <bool BF16>
__device__ __forceinline__ void attend_partial_body(const AttendArgs& a, int bx, int bh) {
  const int mode = a.mode;
  const FetchSrc fs = a.fs;
  const float* __restrict__ q = a.q;
  const void* cacheK = a.cacheK;
  const void* cacheV = a.cacheV;
  const int32_t* __restrict__ sel_slot = a.sel_slot;
  const uint8_t* __restrict__ hit = a.hit;
  const int32_t* __restrict__ miss_slot = a.miss_slot;
  const int32_t* __restrict__ n_miss = a.n_miss;
  const void* __restrict__ liteK = a.liteK;
  const void* __restrict__ liteV = a.liteV;
  float* __restrict__ partials = a.partials;
  const int Hq = a.Hq, Hkv = a.Hkv, C = a.C, k = a.k, w = a.w;
  const int rows_per_block = a.rows_per_block, parts_per_head = a.parts_per_head;
  const int part_offset = a.part_offset;
  const float scale = a.scale;
  constexpr size_t ROWB = kD * (BF16 ? 2 : 4);
  __shared__ float wm[4], wsum[4];
  __shared__ float wacc[4][kD];

  const int b = bh / Hq, h = bh - b * Hq;
  const int kvh = h / (Hq / Hkv);
  const int t = threadIdx.x, lane = t & 63, wv = t >> 6;
  const int grp = lane >> 4, c = lane & 15;

  const char* Kc = static_cast<const char*>(cacheK) + (size_t)bh * C * ROWB;
  const char* Vc = static_cast<const char*>(cacheV) + (size_t)bh * C * ROWB;
  const char* __restrict__ Kh = nullptr;
  const char* __restrict__ Vh = nullptr;
  const int32_t* __restrict__ toks = nullptr;
  if (mode == kAttendAllFetch) {
    Kh = fs.K_host + ((size_t)b * Hkv + kvh) * (size_t)fs.lrows * ROWB;
    Vh = fs.V_host + ((size_t)b * Hkv + kvh) * (size_t)fs.lrows * ROWB;
    toks = fs.sel_idx + (size_t)bh * k;
  }
  const char* __restrict__ Kl =
      static_cast<const char*>(liteK) + ((size_t)b * Hkv + kvh) * (size_t)w * ROWB;
  const char* __restrict__ Vl =
      static_cast<const char*>(liteV) + ((size_t)b * Hkv + kvh) * (size_t)w * ROWB;
  const int32_t* __restrict__ slots =
      (mode == kAttendMisses ? miss_slot : sel_slot) + (size_t)bh * k;
  const uint8_t* __restrict__ hits = hit ? hit + (size_t)bh * k : nullptr;

  int n_rows;  // length of this head's row list
  if (mode == kAttendMisses) {
    const int nm = n_miss[bh];
    n_rows = nm < 0 ? 0 : min(nm, k);
  } else {
    n_rows = k + w;
  }

  float qv[8];
  {
    const float4 q0 = reinterpret_cast<const float4*>(q + (size_t)bh * kD)[2 * c];
    const float4 q1 = reinterpret_cast<const float4*>(q + (size_t)bh * kD)[2 * c + 1];
    const float f = scale * kLog2e;  // logits are kept in log2 units
    qv[0] = q0.x * f; qv[1] = q0.y * f; qv[2] = q0.z * f; qv[3] = q0.w * f;
    qv[4] = q1.x * f; qv[5] = q1.y * f; qv[6] = q1.z * f; qv[7] = q1.w * f;
  }

  float m = -INFINITY, ssum = 0.0f;
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

  const int row_begin = bx * rows_per_block;
  const int row_end = min(n_rows, row_begin + rows_per_block);
  for (int base = row_begin; base < row_end; base += kRowsPerPass * kUnroll) {
    const void* kp[kUnroll];
    const void* vp[kUnroll];
    void* kdst[kUnroll];  // cache slot to fill when the row comes from the host store
    void* vdst[kUnroll];
    bool ok[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const int j = base + u * kRowsPerPass + wv * 4 + grp;
      ok[u] = j < row_end;
      kp[u] = nullptr;
      vp[u] = nullptr;
      kdst[u] = nullptr;
      vdst[u] = nullptr;
      if (ok[u]) {
        if (mode != kAttendMisses && j >= k) {
          kp[u] = Kl + (size_t)(j - k) * ROWB;
          vp[u] = Vl + (size_t)(j - k) * ROWB;
        } else {
          const int32_t s = slots[j];
          ok[u] = s >= 0 && s < C && !(mode == kAttendHitsAndLite && hits[j] == 0);
          kp[u] = Kc + (size_t)s * ROWB;
          vp[u] = Vc + (size_t)s * ROWB;
          if (mode == kAttendAllFetch && ok[u] && hits[j] == 0) {
            const int32_t tok = toks[j];
            if (tok >= 0 && tok < fs.l) {
              kdst[u] = const_cast<char*>(Kc) + (size_t)s * ROWB;
              vdst[u] = const_cast<char*>(Vc) + (size_t)s * ROWB;
              kp[u] = Kh + (size_t)tok * ROWB;
              vp[u] = Vh + (size_t)tok * ROWB;
            }
          }
        }
      }
    }
    RowChunk<BF16> kc[kUnroll], vc[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u)
      if (ok[u]) {
        kc[u].load(kp[u], c);
        vc[u].load(vp[u], c);
      }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u)
      if (kdst[u]) {
        kc[u].store(kdst[u], c);
        vc[u].store(vdst[u], c);
      }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      float part = 0.0f;
      Chunk8 kk = kc[u].get();
#pragma unroll
      for (int i = 0; i < 8; ++i) part = __builtin_fmaf(qv[i], ok[u] ? kk.v[i] : 0.0f, part);
      const float logit = row16_allreduce_sum(part);  // all lanes take part in the DPP ops
      if (ok[u]) {
        const float m_new = fmaxf(m, logit);
        const float corr = exp2f(m - m_new);  // m = -inf on the first row gives 0
        const float p = exp2f(logit - m_new);
        ssum = ssum * corr + p;
        Chunk8 vv = vc[u].get();
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = __builtin_fmaf(p, vv.v[i], acc[i] * corr);
        m = m_new;
      }
    }
  }

  // merge the 4 row groups of the wavefront (lanes c, c+16, c+32, c+48)
  float mw = fmaxf(m, __shfl_xor(m, 16));
  mw = fmaxf(mw, __shfl_xor(mw, 32));
  const float f = (m == -INFINITY) ? 0.0f : exp2f(m - mw);
  ssum *= f;
  ssum += __shfl_xor(ssum, 16);
  ssum += __shfl_xor(ssum, 32);
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    float a = acc[i] * f;
    a += __shfl_xor(a, 16);
    a += __shfl_xor(a, 32);
    acc[i] = a;
  }
  if (lane < 16) {
#pragma unroll
    for (int i = 0; i < 8; ++i) wacc[wv][8 * c + i] = acc[i];
    if (lane == 0) {
      wm[wv] = mw;
      wsum[wv] = ssum;
    }
  }
  __syncthreads();
  // merge the 4 wavefronts; thread j < 128 owns output dimension j
  if (t < kD) {
    const float M = fmaxf(fmaxf(wm[0], wm[1]), fmaxf(wm[2], wm[3]));
    float a = 0.0f, s = 0.0f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float g = (wm[i] == -INFINITY) ? 0.0f : exp2f(wm[i] - M);
      a += wacc[i][t] * g;
      s += wsum[i] * g;
    }
    float* __restrict__ P =
        partials + ((size_t)bh * parts_per_head + part_offset + bx) * kPartialStride;
    P[4 + t] = a;
    if (t == 0) {
      P[0] = M;
      P[1] = s;
    }
  }
}

template <bool BF16>
__global__ __launch_bounds__(kAttThreads) void attend_partial_kernel(const AttendArgs a) {
  attend_partial_body<BF16>(a, blockIdx.x, blockIdx.y);
}

// Fetch shared by the query heads of a KV group (K and V exist once per KV head, Sec. 4
// preliminaries; Alg. 2 "Fetch missing", "merge"): the missing rows of head bh, 16 lanes a row.
// A position that several heads of the group miss is read from the host store once, by the
// lowest of those heads, and written into the slot each of them gave it; the other heads skip
// it.  The heads' miss lists are ascending, so "does head g2 miss this position, and where" is
// a binary search, run by lane g2 of the 16-lane group for its head.
struct GroupFetchArgs {
  FetchSrc fs;          // sel_idx unused
  void* cacheK;
  void* cacheV;
  const int32_t* miss_tok;
  const int32_t* miss_slot;
  const int32_t* n_miss;
  int32_t* link_rows;   // [B,Hkv] rows read from the host store, or null (not counted)
  int Hq, Hkv, C, k;
};
template <bool BF16>
__device__ __forceinline__ void group_fetch_body(const GroupFetchArgs& a, int fx, int nfx, int bh) {
  constexpr size_t ROWB = kD * (BF16 ? 2 : 4);
  const int Hq = a.Hq, Hkv = a.Hkv, C = a.C, k = a.k;
  const int G = Hq / Hkv;
  const int b = bh / Hq, h = bh - b * Hq, kvh = h / G, g = h - kvh * G;
  const int bh0 = bh - g;  // first head of the group
  const int t = threadIdx.x, lane = t & 63, sub = t & 15, rgrp = t >> 4;
  const int nm = max(0, min(a.n_miss[bh], k));
  const int32_t* __restrict__ mt = a.miss_tok + (size_t)bh * k;
  const int32_t* __restrict__ ms = a.miss_slot + (size_t)bh * k;
  const char* __restrict__ Kh = a.fs.K_host + ((size_t)b * Hkv + kvh) * (size_t)a.fs.lrows * ROWB;
  const char* __restrict__ Vh = a.fs.V_host + ((size_t)b * Hkv + kvh) * (size_t)a.fs.lrows * ROWB;
  // lane `sub` < G looks positions up in the list of head bh0 + sub
  const int32_t* __restrict__ ot = a.miss_tok + (size_t)(bh0 + min(sub, G - 1)) * k;
  const int32_t* __restrict__ os = a.miss_slot + (size_t)(bh0 + min(sub, G - 1)) * k;
  const int onm = sub < G ? max(0, min(a.n_miss[bh0 + sub], k)) : 0;
  for (int j0 = fx * 16; j0 < nm; j0 += nfx * 16) {  // uniform trip count over the wavefront
    const int j = j0 + rgrp;
    const bool have = j < nm;
    const int32_t tok = have ? mt[j] : -1;
    const int32_t slot = have ? ms[j] : -1;
    const bool ok = tok >= 0 && tok < a.fs.l && slot >= 0 && slot < C;
    // where, if anywhere, head bh0 + sub lists this position
    int32_t oslot = -1;
    if (ok && sub < G && sub != g) {
      int lo = 0, hi = onm;
      while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (ot[mid] < tok) lo = mid + 1; else hi = mid;
      }
      if (lo < onm && ot[lo] == tok) {
        const int32_t s2 = os[lo];
        oslot = (s2 >= 0 && s2 < C) ? s2 : -2;  // -2: listed, but with an unusable slot
      }
    }
    // the lowest head that lists the position fetches it
    const unsigned long long listed = __ballot(oslot != -1);
    const unsigned mine16 = (unsigned)(listed >> (lane & 48)) & 0xffffu;
    const bool owner = ok && (mine16 & ((1u << g) - 1u)) == 0u;
    RowChunk<BF16> kc, vc;
    if (owner) {
      kc.load(Kh + (size_t)tok * ROWB, sub);
      vc.load(Vh + (size_t)tok * ROWB, sub);
      kc.store(static_cast<char*>(a.cacheK) + ((size_t)bh * C + slot) * ROWB, sub);
      vc.store(static_cast<char*>(a.cacheV) + ((size_t)bh * C + slot) * ROWB, sub);
      if (sub == 0 && a.link_rows) atomicAdd(&a.link_rows[b * Hkv + kvh], 1);
    }
    for (int g2 = g + 1; g2 < G; ++g2) {  // uniform
      const int32_t s2 = __shfl(oslot, (lane & 48) + g2);
      if (owner && s2 >= 0) {
        kc.store(static_cast<char*>(a.cacheK) + ((size_t)(bh0 + g2) * C + s2) * ROWB, sub);
        vc.store(static_cast<char*>(a.cacheV) + ((size_t)(bh0 + g2) * C + s2) * ROWB, sub);
      }
    }
  }
}

template <bool BF16>
__global__ __launch_bounds__(kAttThreads) void group_fetch_kernel(const GroupFetchArgs a) {
  group_fetch_body<BF16>(a, blockIdx.x, gridDim.x, blockIdx.y);
}

// The attention over the rows that hit and the lite rows (blocks [0, n_attend) of a head) and
// the group's shared fetch (the remaining blocks) in one launch: the two do not depend on each
// other, so the host-link reads run beside the HBM reads.
template <bool BF16>
__global__ __launch_bounds__(kAttThreads) void attend_hits_group_fetch_kernel(
    const AttendArgs a, const GroupFetchArgs f, int n_attend) {
  if ((int)blockIdx.x < n_attend)
    attend_partial_body<BF16>(a, blockIdx.x, blockIdx.y);
  else
    group_fetch_body<BF16>(f, blockIdx.x - n_attend, gridDim.x - n_attend, blockIdx.y);
}

constexpr int kCombThreads = 512;
constexpr int kCombMaxParts = 1024;

// Merge the partial softmax states of one head.  The per-part weights are computed
// once in LDS; four groups of 128 threads then walk the parts with independent,
// coalesced loads (thread = output dimension) and are summed through LDS.
__global__ __launch_bounds__(kCombThreads) void attend_combine_kernel(
    const float* __restrict__ partials, int parts_per_head, int nparts,
    float* __restrict__ out) {
  __shared__ float wgt[kCombMaxParts];
  __shared__ float red[kCombThreads / 64];
  __shared__ float accs[kCombThreads / kD][kD];
  __shared__ float sh_M, sh_S;
  const int bh = blockIdx.x, t = threadIdx.x, lane = t & 63, wv = t >> 6;
  const float* __restrict__ P = partials + (size_t)bh * parts_per_head * kPartialStride;
  // block max of the part maxima
  float m = -INFINITY;
  for (int p = t; p < nparts; p += kCombThreads) m = fmaxf(m, P[(size_t)p * kPartialStride]);
#pragma unroll
  for (int d = 32; d > 0; d >>= 1) m = fmaxf(m, __shfl_xor(m, d));
  if (lane == 0) red[wv] = m;
  __syncthreads();
  if (t == 0) {
    float M = red[0];
    for (int i = 1; i < kCombThreads / 64; ++i) M = fmaxf(M, red[i]);
    sh_M = M;
  }
  __syncthreads();
  const float M = sh_M;
  float ssum = 0.0f;
  for (int p = t; p < nparts; p += kCombThreads) {
    const float mp = P[(size_t)p * kPartialStride];
    const float g = (mp == -INFINITY) ? 0.0f : exp2f(mp - M);
    wgt[p] = g;
    ssum += P[(size_t)p * kPartialStride + 1] * g;
  }
#pragma unroll
  for (int d = 32; d > 0; d >>= 1) ssum += __shfl_xor(ssum, d);
  __syncthreads();
  if (lane == 0) red[wv] = ssum;
  __syncthreads();
  if (t == 0) {
    float S = 0.0f;
    for (int i = 0; i < kCombThreads / 64; ++i) S += red[i];
    sh_S = S;
  }
  const int dim = t & (kD - 1), grp = t / kD;
  float a = 0.0f;
#pragma unroll 8
  for (int p = grp; p < nparts; p += kCombThreads / kD)
    a = __builtin_fmaf(P[(size_t)p * kPartialStride + 4 + dim], wgt[p], a);
  accs[grp][dim] = a;
  __syncthreads();
  if (t < kD) {
    float tot = 0.0f;
#pragma unroll
    for (int g = 0; g < kCombThreads / kD; ++g) tot += accs[g][t];
    const float S = sh_S;
    out[(size_t)bh * kD + t] = S > 0.0f ? tot / S : 0.0f;
  }
}

}  // namespace

AttendGeom attend_geometry(int BHq, int k, int w) {
  const int rows = k + w;
  AttendGeom g;
  g.rows_per_block = kRowsPerPass * kUnroll;
  // fewer, larger workgroups once there are plenty of them
  while (g.rows_per_block < 512 && (long)ceil_div(rows, g.rows_per_block * 2) * BHq >= 2048)
    g.rows_per_block *= 2;
  g.nsplit = ceil_div(rows, g.rows_per_block);
  return g;
}

size_t attend_ws_bytes(int BHq, int k, int w, int phases) {
  const AttendGeom g = attend_geometry(BHq, k, w);
  const int parts = g.nsplit + (phases > 1 ? ceil_div(k, g.rows_per_block) : 0);
  return round_up((size_t)BHq * parts * kPartialStride * sizeof(float), 256);
}

static AttendArgs make_attend_args(const lrqk_shape& s, int mode, const float* q,
                                   const void* cacheK, const void* cacheV,
                                   const int32_t* sel_slot, const uint8_t* hit,
                                   const int32_t* miss_slot, const int32_t* n_miss,
                                   const void* liteK, const void* liteV, float* partials,
                                   int rows_per_block, int parts_per_head, int part_offset,
                                   const void* K_host, const void* V_host,
                                   const int32_t* sel_idx) {
  AttendArgs a;
  a.mode = mode;
  a.fs = FetchSrc{static_cast<const char*>(K_host), static_cast<const char*>(V_host), sel_idx,
                  s.l, row_cap(s)};
  a.q = q;
  a.cacheK = cacheK;
  a.cacheV = cacheV;
  a.sel_slot = sel_slot;
  a.hit = hit;
  a.miss_slot = miss_slot;
  a.n_miss = n_miss;
  a.liteK = liteK;
  a.liteV = liteV;
  a.partials = partials;
  a.Hq = s.Hq;
  a.Hkv = s.Hkv;
  a.C = s.C;
  a.k = s.k;
  a.w = s.w;
  a.rows_per_block = rows_per_block;
  a.parts_per_head = parts_per_head;
  a.part_offset = part_offset;
  a.scale = s.scale;
  return a;
}

static GroupFetchArgs make_group_fetch_args(const lrqk_shape& s, const void* K_host,
                                            const void* V_host, const int32_t* miss_tok,
                                            const int32_t* miss_slot, const int32_t* n_miss,
                                            void* cacheK, void* cacheV, int32_t* link_rows) {
  GroupFetchArgs f;
  f.fs = FetchSrc{static_cast<const char*>(K_host), static_cast<const char*>(V_host), nullptr,
                  s.l, row_cap(s)};
  f.cacheK = cacheK;
  f.cacheV = cacheV;
  f.miss_tok = miss_tok;
  f.miss_slot = miss_slot;
  f.n_miss = n_miss;
  f.link_rows = link_rows;
  f.Hq = s.Hq;
  f.Hkv = s.Hkv;
  f.C = s.C;
  f.k = s.k;
  return f;
}

hipError_t launch_attend_partial(const lrqk_shape& s, int mode, const float* q, const void* cacheK,
                                 const void* cacheV, const int32_t* sel_slot, const uint8_t* hit,
                                 const int32_t* miss_slot, const int32_t* n_miss,
                                 const void* liteK, const void* liteV, float* partials,
                                 int nblocks, int rows_per_block, int parts_per_head,
                                 int part_offset, hipStream_t st, const void* K_host,
                                 const void* V_host, const int32_t* sel_idx) {
  if (nblocks <= 0) return hipSuccess;
  if (mode == kAttendAllFetch && (!K_host || !V_host || !sel_idx || !hit))
    return hipErrorInvalidValue;
  const AttendArgs a = make_attend_args(s, mode, q, cacheK, cacheV, sel_slot, hit, miss_slot,
                                        n_miss, liteK, liteV, partials, rows_per_block,
                                        parts_per_head, part_offset, K_host, V_host, sel_idx);
  const dim3 grid(nblocks, s.B * s.Hq);
  if (s.kv_dtype == LRQK_KV_BF16)
    LRQK_LAUNCH((attend_partial_kernel<true>), grid, dim3(kAttThreads), 0, st, a);
  else
    LRQK_LAUNCH((attend_partial_kernel<false>), grid, dim3(kAttThreads), 0, st, a);
  return hipGetLastError();
}

// workgroups per head that the shared fetch is spread over (16 rows per pass each)
static int group_fetch_blocks(const lrqk_shape& s) { return min(ceil_div(s.k, 16), 32); }

hipError_t launch_group_fetch(const lrqk_shape& s, const void* K_host, const void* V_host,
                              const int32_t* miss_tok, const int32_t* miss_slot,
                              const int32_t* n_miss, void* cacheK, void* cacheV,
                              int32_t* link_rows, hipStream_t st) {
  const GroupFetchArgs f = make_group_fetch_args(s, K_host, V_host, miss_tok, miss_slot, n_miss,
                                                 cacheK, cacheV, link_rows);
  const dim3 grid(group_fetch_blocks(s), s.B * s.Hq);
  if (s.kv_dtype == LRQK_KV_BF16)
    LRQK_LAUNCH((group_fetch_kernel<true>), grid, dim3(kAttThreads), 0, st, f);
  else
    LRQK_LAUNCH((group_fetch_kernel<false>), grid, dim3(kAttThreads), 0, st, f);
  return hipGetLastError();
}

hipError_t launch_attend_hits_group_fetch(const lrqk_shape& s, const float* q, void* cacheK,
                                          void* cacheV, const int32_t* sel_slot,
                                          const uint8_t* hit, const void* liteK,
                                          const void* liteV, float* partials, int nblocks,
                                          int rows_per_block, int parts_per_head,
                                          const void* K_host, const void* V_host,
                                          const int32_t* miss_tok, const int32_t* miss_slot,
                                          const int32_t* n_miss, int32_t* link_rows,
                                          hipStream_t st) {
  const AttendArgs a = make_attend_args(s, kAttendHitsAndLite, q, cacheK, cacheV, sel_slot, hit,
                                        nullptr, nullptr, liteK, liteV, partials, rows_per_block,
                                        parts_per_head, 0, nullptr, nullptr, nullptr);
  const GroupFetchArgs f = make_group_fetch_args(s, K_host, V_host, miss_tok, miss_slot, n_miss,
                                                 cacheK, cacheV, link_rows);
  const dim3 grid(nblocks + group_fetch_blocks(s), s.B * s.Hq);
  if (s.kv_dtype == LRQK_KV_BF16)
    LRQK_LAUNCH((attend_hits_group_fetch_kernel<true>), grid, dim3(kAttThreads), 0, st, a, f,
                nblocks);
  else
    LRQK_LAUNCH((attend_hits_group_fetch_kernel<false>), grid, dim3(kAttThreads), 0, st, a, f,
                nblocks);
  return hipGetLastError();
}

hipError_t launch_attend_combine(const lrqk_shape& s, const float* partials, int parts_per_head,
                                 int nparts, float* out, hipStream_t st) {
  if (nparts > kCombMaxParts) return hipErrorInvalidValue;
  LRQK_LAUNCH(attend_combine_kernel, dim3(s.B * s.Hq), dim3(kCombThreads), 0, st,
                     partials, parts_per_head, nparts, out);
  return hipGetLastError();
}

}  // namespace lrqk
