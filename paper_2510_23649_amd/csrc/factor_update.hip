// u1 — decode-time update of the factors (Alg. 2 from the initial guess of k_hat to the
// two gradient steps; Sec. 4.2 update rules for q_hat_t, k_hat_t, B_Q, B_K; App. A.2 optimal
// step lengths).
//
// Two launches.
//
//  1. factor_gram_kernel: everything that is a sum over many rows.  For a list of rows a_i
//     (r floats each) with weights u_i it produces  S = sum_i a_i^T a_i  (r x r)  and
//     g = sum_i u_i a_i  (r).  Three kinds of jobs share the code:
//       * Omega of a query head (the k rows selected at the previous step, read from their
//         cache slots, and the w lite rows): a_i = row of A_K, u_i = q . K_i.  This gives
//         A_Om^T A_Om and q K_Om^T A_Om.  The row list of a head is cut into chunks of at most
//         144 rows, one workgroup each, so that batch-1 steps still use hundreds of CUs; K rows
//         are read by 16 lanes each exactly as the attention kernel reads them;
//       * B_Q of a query head, read column-wise: a_i = column i of B_Q, u_i = q_i, which
//         gives B_Q B_Q^T and q B_Q^T;
//       * B_K of a KV head with u = k_t: B_K B_K^T and k B_K^T.
//     The chunk's rows are staged in LDS, then every thread owns r*r/256 entries of S and
//     adds the rows' outer products to them; partial sums per chunk go to the
//     workspace and are added up, in chunk order, by the second kernel: no atomics, the
//     result does not depend on scheduling.
//
//  2. factor_solve_kernel: one workgroup per (batch, KV head), one wavefront per query
//     head of the group.  The r x r systems (r <= 64) are solved inside a wavefront: lane i
//     holds row i of the matrix in registers, a right-looking Cholesky factorisation takes
//     column j from lane registers with v_readlane (all register indices are compile-time
//     constants), the two triangular solves follow the same pattern, with one transpose of
//     the factor through LDS in between.  Only what changes between rounds is factorised
//     again: M_rq = P + lambda_d1 k_hat^T k_hat differs from the fixed
//     P = B_Q B_Q^T + lambda_d2 A_Om^T A_Om by a rank-one term, so P is factorised once and
//     each q_hat costs one pair of triangular solves (Sherman-Morrison); the k_hat system
//     changes by a rank-G term and is factorised anew each round.  The alternating updates
//     of q_hat (per query head) and k_hat (per KV head, summed over the group's heads)
//     exchange q_hat through LDS; every wavefront solves the k_hat system redundantly, which
//     is cheaper than a second exchange.  The same kernel then applies the two rank-one
//     gradient steps to B_Q and B_K in place.
//
// All arithmetic is fp32 (App. B.1 runs these updates in fp32).
#include "lrqk_device.h"
#include "lrqk_internal.h"
#include "lrqk_linalg.h"

namespace lrqk {
namespace {

using namespace linalg;

constexpr int kGramThreads = 256;
constexpr int kGramBatch = 144;  // rows staged in LDS at a time (a multiple of 16)

template <int CTRL>
__device__ __forceinline__ float fu_dpp(float v) {
  return __int_as_float(
      __builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}
__device__ __forceinline__ float row16_sum(float v) {
  v += fu_dpp<0x128>(v);  // row_ror:8
  v += fu_dpp<0x124>(v);  // row_ror:4
  v += fu_dpp<0x122>(v);  // row_ror:2
  v += fu_dpp<0x121>(v);  // row_ror:1
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
  v = row16_sum(v);
  // the four 16-lane rows of the wavefront
  const float a = __shfl(v, 0), b = __shfl(v, 16), c = __shfl(v, 32), e = __shfl(v, 48);
  return (a + b) + (c + e);
}
__device__ __forceinline__ float bf16_to_f32(uint16_t h) {
  return __uint_as_float((uint32_t)h << 16);
}
template <bool BF16>
__device__ __forceinline__ float kv_load(const void* row, int j) {
  if (BF16) return bf16_to_f32(static_cast<const uint16_t*>(row)[j]);
  return static_cast<const float*>(row)[j];
}

// q . K_row for the 16 lanes that share a row; lane c of the 16 takes elements 8c .. 8c+7.
// The load and the arithmetic are separate so that a batch of loads can be issued together.
template <bool BF16>
struct RowPiece {
  uint4 lo, hi;  // bf16: lo only
};
template <bool BF16>
__device__ __forceinline__ RowPiece<BF16> load_piece(const void* row, int c) {
  RowPiece<BF16> p;
  if (BF16) {
    p.lo = static_cast<const uint4*>(row)[c];
    p.hi = p.lo;
  } else {
    p.lo = static_cast<const uint4*>(row)[2 * c];
    p.hi = static_cast<const uint4*>(row)[2 * c + 1];
  }
  return p;
}
template <bool BF16>
__device__ __forceinline__ float dot_piece(const RowPiece<BF16>& p, const float (&qv)[8]) {
  float x[8];
  if (BF16) {
    const uint4 u = p.lo;
    x[0] = __uint_as_float(u.x << 16); x[1] = __uint_as_float(u.x & 0xffff0000u);
    x[2] = __uint_as_float(u.y << 16); x[3] = __uint_as_float(u.y & 0xffff0000u);
    x[4] = __uint_as_float(u.z << 16); x[5] = __uint_as_float(u.z & 0xffff0000u);
    x[6] = __uint_as_float(u.w << 16); x[7] = __uint_as_float(u.w & 0xffff0000u);
  } else {
    x[0] = __uint_as_float(p.lo.x); x[1] = __uint_as_float(p.lo.y);
    x[2] = __uint_as_float(p.lo.z); x[3] = __uint_as_float(p.lo.w);
    x[4] = __uint_as_float(p.hi.x); x[5] = __uint_as_float(p.hi.y);
    x[6] = __uint_as_float(p.hi.z); x[7] = __uint_as_float(p.hi.w);
  }
  float acc = 0.0f;
#pragma unroll
  for (int j = 0; j < 8; ++j) acc = __builtin_fmaf(x[j], qv[j], acc);
  return acc;
}

// S += sum_i a_i^T a_i and g += sum_i u_i a_i over the kGramBatch rows staged in LDS (a_s: row
// stride LDA floats, rows past the end are zero), by the 256 threads of a workgroup.
// S is a dense contraction over the rows and goes through v_mfma_f32_32x32x2_f32, whose two
// operands are here the same numbers: lane i + 32 kk supplies A[i][kk] = B[kk][i] = element i
// of row kk of the pair.  r <= 32: one 32 x 32 block (columns >= r read as zero), each
// wavefront sums a quarter of the rows; r = 64: wavefront (bi, bj) owns block (bi, bj) of S
// and sums all the rows.  g: thread t sums column t % r over every (256 / r)-th row.
typedef float f32x16 __attribute__((ext_vector_type(16)));
template <int R>
__device__ __forceinline__ void gram_accumulate(const float* a_s, const float* u_s, f32x16& sacc,
                                                float& gpart, int t) {
  constexpr int LDA = R + 4;
  const int wave = t >> 6, lane = t & 63, li = lane & 31, lk = lane >> 5;
  if constexpr (R <= 32) {
    constexpr int kRows = kGramBatch / 4;  // rows per wavefront
    static_assert(kRows % 2 == 0, "rows are consumed in pairs");
#pragma unroll 6
    for (int i = 0; i < kRows; i += 2) {
      const float x = li < R ? a_s[(wave * kRows + i + lk) * LDA + li] : 0.0f;
      sacc = __builtin_amdgcn_mfma_f32_32x32x2f32(x, x, sacc, 0, 0, 0);
    }
  } else {
    const int bi = wave >> 1, bj = wave & 1;
#pragma unroll 6
    for (int i = 0; i < kGramBatch; i += 2) {
      const float xa = a_s[(i + lk) * LDA + 32 * bi + li];
      const float xb = a_s[(i + lk) * LDA + 32 * bj + li];
      sacc = __builtin_amdgcn_mfma_f32_32x32x2f32(xa, xb, sacc, 0, 0, 0);
    }
  }
  constexpr int kSub = kGramThreads / R;
  const int gc = t % R;
#pragma unroll 4
  for (int i = t / R; i < kGramBatch; i += kSub) gpart = __builtin_fmaf(u_s[i], a_s[i * LDA + gc], gpart);
}

struct GramArgs {
  const float* A_K;              // [B,Hkv,l_rows,r]
  const void* cacheK;            // [B,Hq,C,d]
  const void* liteK;             // [B,Hkv,w,d], row j holds the position p of [l-w,l), p % w == j
  const int32_t* sel_idx_prev;   // [B,Hq,k]
  const int32_t* sel_slot_prev;  // [B,Hq,k]
  const float* q;                // [B,Hq,d]
  const void* k_new;             // [B,Hkv,d]
  const float* B_Q;              // [B,Hq,r,d]
  const float* B_K;              // [B,Hkv,r,d]
  float* gram_om;                // [B*Hq][nchunk][r*r + r]
  float* gram_q;                 // [B*Hq][r*r + r]
  float* gram_k;                 // [B*Hkv][r*r + r]
  int Hq, Hkv, l, l_rows, k, w, C, nchunk, chunk_rows;
};

template <int R, bool BF16>
__global__ __launch_bounds__(kGramThreads) void factor_gram_kernel(GramArgs a) {
  constexpr int kEntries = R * R;
  constexpr int LDA = R + 4;  // padded LDS row, keeps 16-byte alignment
  constexpr size_t ROWB = kD * (BF16 ? 2 : 4);
  __shared__ __align__(16) float a_s[kGramBatch * LDA];
  // r <= 32: the partial blocks of wavefronts 1..3; then the partial sums of g
  __shared__ float red_s[R <= 32 ? 3 * 1024 : kGramThreads];
  __shared__ float u_s[kGramBatch];
  __shared__ int pos_s[kGramBatch];
  __shared__ const char* krow_s[kGramBatch];

  const int bh = blockIdx.y, job = blockIdx.x, t = threadIdx.x;
  const int b = bh / a.Hq, h = bh - b * a.Hq;
  const int G = a.Hq / a.Hkv;
  const int kvh = h / G;
  const int bkv = b * a.Hkv + kvh;
  if (job == a.nchunk + 1 && h != kvh * G) return;  // the B_K job runs once per KV head

  f32x16 sacc;
#pragma unroll
  for (int v = 0; v < 16; ++v) sacc[v] = 0.0f;
  float gpart = 0.0f;

  float* out;
  if (job < a.nchunk) {
    // ---- a chunk of the rows of Omega --------------------------------------------------
    out = a.gram_om + ((size_t)bh * a.nchunk + job) * (kEntries + R);
    const int n_om = a.k + a.w;
    const int i_begin = job * a.chunk_rows;
    const int i_end = min(n_om, i_begin + a.chunk_rows);
    const float* __restrict__ Ahead = a.A_K + (size_t)bkv * (size_t)a.l_rows * R;
    const char* Kc = static_cast<const char*>(a.cacheK) + (size_t)bh * a.C * ROWB;
    const char* Kl = static_cast<const char*>(a.liteK) + (size_t)bkv * a.w * ROWB;
    const int c16 = t & 15, rsub = t >> 4;
    float qv[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) qv[j] = a.q[(size_t)bh * kD + c16 * 8 + j];
    const char* qrow = reinterpret_cast<const char*>(a.q + (size_t)bh * kD);
    const int lite0 = a.l - a.w;  // first position of the lite window
    for (int i0 = i_begin; i0 < i_end; i0 += kGramBatch) {
      __syncthreads();  // the previous batch has been consumed
      if (t < kGramBatch) {
        const int i = i0 + t;
        int pos = -1;
        const char* krow = nullptr;
        if (i < i_end) {
          if (i < a.k) {
            const int tok = a.sel_idx_prev[(size_t)bh * a.k + i];
            const int slot = a.sel_slot_prev[(size_t)bh * a.k + i];
            if (tok >= 0 && tok < a.l && slot >= 0 && slot < a.C) {
              pos = tok;
              krow = Kc + (size_t)slot * ROWB;
            }
          } else {
            const int j = i - a.k;  // row of the lite ring
            // the position in [l-w, l) that is congruent to j modulo w
            int off = (j - lite0) % a.w;
            if (off < 0) off += a.w;
            pos = lite0 + off;
            krow = Kl + (size_t)j * ROWB;
          }
        }
        pos_s[t] = pos;
        krow_s[t] = krow;
      }
      __syncthreads();
      // All the loads of the batch are issued before anything waits for one of them; rows
      // that do not exist read memory that does (the head's q, which is at least as long as
      // a K row; row 0 of A_K) and are zeroed afterwards.
      // u_i = q . K_i: 16 lanes per row, 16 rows per pass
      constexpr int kPasses = kGramBatch / 16;
      RowPiece<BF16> piece[kPasses];
#pragma unroll
      for (int pass = 0; pass < kPasses; ++pass) {
        const char* krow = krow_s[pass * 16 + rsub];
        piece[pass] = load_piece<BF16>(krow ? krow : qrow, c16);
      }
      // a_i = A_K[pos_i, :]
      constexpr int kAPieces = (kGramBatch * (R / 4) + kGramThreads - 1) / kGramThreads;
      float4 av[kAPieces];
#pragma unroll
      for (int u = 0; u < kAPieces; ++u) {
        const int idx = t + u * kGramThreads;
        const int rr = min(idx / (R / 4), kGramBatch - 1), c4 = idx % (R / 4);
        const int pos = pos_s[rr];
        av[u] = reinterpret_cast<const float4*>(Ahead + (size_t)max(pos, 0) * R)[c4];
        if (pos < 0) av[u] = make_float4(0.f, 0.f, 0.f, 0.f);
      }
#pragma unroll
      for (int pass = 0; pass < kPasses; ++pass) {
        const int rr = pass * 16 + rsub;
        float dot = krow_s[rr] ? dot_piece<BF16>(piece[pass], qv) : 0.0f;
        dot = row16_sum(dot);
        if (c16 == 0) u_s[rr] = dot;
      }
#pragma unroll
      for (int u = 0; u < kAPieces; ++u) {
        const int idx = t + u * kGramThreads;
        if (idx < kGramBatch * (R / 4))
          *reinterpret_cast<float4*>(&a_s[idx / (R / 4) * LDA + 4 * (idx % (R / 4))]) = av[u];
      }
      __syncthreads();
      gram_accumulate<R>(a_s, u_s, sacc, gpart, t);
    }
  } else {
    // ---- B_Q of this query head, or B_K of this KV head, read column by column ------------
    const bool isq = job == a.nchunk;
    out = isq ? a.gram_q + (size_t)bh * (kEntries + R) : a.gram_k + (size_t)bkv * (kEntries + R);
    const float* __restrict__ Bm =
        isq ? a.B_Q + (size_t)bh * R * kD : a.B_K + (size_t)bkv * R * kD;
    for (int i0 = 0; i0 < kD; i0 += kGramBatch) {
      __syncthreads();
      if (t < kGramBatch) {
        const int i = i0 + t;
        float u = 0.0f;
        if (i < kD)
          u = isq ? a.q[(size_t)bh * kD + i]
                  : kv_load<BF16>(static_cast<const char*>(a.k_new) + (size_t)bkv * ROWB, i);
        u_s[t] = u;
      }
      // every load is issued before the first is waited for (addresses clamped, the values
      // past the end zeroed)
      constexpr int kBPieces = (kGramBatch * R + kGramThreads - 1) / kGramThreads;
      float bv[kBPieces];
#pragma unroll
      for (int u = 0; u < kBPieces; ++u) {
        const int idx = t + u * kGramThreads;
        const int c = min(idx / kGramBatch, R - 1), ii = idx % kGramBatch;
        bv[u] = Bm[(size_t)c * kD + min(i0 + ii, kD - 1)];
        if (i0 + ii >= kD) bv[u] = 0.0f;
      }
#pragma unroll
      for (int u = 0; u < kBPieces; ++u) {
        const int idx = t + u * kGramThreads;
        if (idx < kGramBatch * R) a_s[idx % kGramBatch * LDA + idx / kGramBatch] = bv[u];
      }
      __syncthreads();
      gram_accumulate<R>(a_s, u_s, sacc, gpart, t);
    }
  }
  // Register v of lane l of an accumulator holds element [8 (v / 4) + 4 (l / 32) + v % 4][l % 32]
  // of its block.
  const int wave = t >> 6, lane = t & 63;
  if constexpr (R <= 32) {
    __syncthreads();
    if (wave > 0) {
#pragma unroll
      for (int v = 0; v < 16; ++v) red_s[(wave - 1) * 1024 + v * 64 + lane] = sacc[v];
    }
    __syncthreads();
    if (wave == 0) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const float sum = ((sacc[v] + red_s[v * 64 + lane]) + red_s[1024 + v * 64 + lane]) +
                          red_s[2048 + v * 64 + lane];
        const int pr = 8 * (v / 4) + 4 * (lane >> 5) + v % 4, qc = lane & 31;
        if (pr < R && qc < R) out[pr * R + qc] = sum;
      }
    }
  } else {
    const int bi = wave >> 1, bj = wave & 1;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int pr = 32 * bi + 8 * (v / 4) + 4 * (lane >> 5) + v % 4, qc = 32 * bj + (lane & 31);
      out[pr * R + qc] = sacc[v];
    }
  }
  __syncthreads();
  red_s[t] = gpart;
  __syncthreads();
  if (t < R) {
    float g = 0.0f;
    for (int sub = 0; sub < kGramThreads / R; ++sub) g += red_s[sub * R + t];
    out[kEntries + t] = g;
  }
}

struct SolveArgs {
  const float* gram_om;  // [B*Hq][nchunk][r*r + r]
  const float* gram_q;   // [B*Hq][r*r + r]
  const float* gram_k;   // [B*Hkv][r*r + r]
  const float* q;        // [B,Hq,d]
  const void* k_new;     // [B,Hkv,d]
  float* B_Q;            // [B,Hq,r,d]   updated in place
  float* B_K;            // [B,Hkv,r,d]  updated in place
  float* q_hat;          // [B,Hq,r]
  float* k_hat;          // [B,Hkv,r]
  int Hq, Hkv, nchunk, n_iter;
  float lam1, lam2;
};

// One exact line-search gradient step on 1/2 |x_hat B - x|^2 (App. A.2), by one wavefront:
//   resid = x_hat B - x,  grad = x_hat^T resid,  eta = <resid, x_hat grad> / |x_hat grad|^2,
//   B <- B - eta grad.  Lane i (< R) holds x_hat_i; x(j) returns element j of the target.
template <int R, typename XF>
__device__ __forceinline__ void line_search_step(float xh, float* __restrict__ Bm, XF x, int lane) {
  const float xhz = lane < R ? xh : 0.0f;
  const float nrm2 = wave_sum(xhz * xhz);
  // this lane's two columns of the residual
  float e0 = -x(lane), e1 = -x(lane + 64);
#pragma unroll
  for (int i = 0; i < R; ++i) {
    const float xi = lane_value(xh, i);
    e0 = __builtin_fmaf(xi, Bm[(size_t)i * kD + lane], e0);
    e1 = __builtin_fmaf(xi, Bm[(size_t)i * kD + lane + 64], e1);
  }
  // x_hat grad = |x_hat|^2 resid
  const float v0 = nrm2 * e0, v1 = nrm2 * e1;
  const float num = wave_sum(e0 * v0 + e1 * v1);
  const float den = wave_sum(v0 * v0 + v1 * v1);
  const float eta = den > 0.0f ? num / den : 0.0f;
#pragma unroll
  for (int i = 0; i < R; ++i) {
    const float s = eta * lane_value(xh, i);
    Bm[(size_t)i * kD + lane] = __builtin_fmaf(-s, e0, Bm[(size_t)i * kD + lane]);
    Bm[(size_t)i * kD + lane + 64] = __builtin_fmaf(-s, e1, Bm[(size_t)i * kD + lane + 64]);
  }
}

template <int R, bool BF16>
__global__ __launch_bounds__(kMaxG * 64) void factor_solve_kernel(SolveArgs a) {
  constexpr int kEntries = R * R;
  constexpr size_t ROWB = kD * (BF16 ? 2 : 4);
  extern __shared__ __align__(16) float lds[];
  const int G = a.Hq / a.Hkv;
  constexpr int NLD = R + 4;  // padded row of the LDS copy of N
  // [G][R*(R+1)] transpose space | [R][NLD] N = B_K B_K^T | [G][R] q_hat exchange | [G] q.k
  float* const lt = lds + (size_t)(threadIdx.x >> 6) * R * (R + 1);
  float* const n_s = lds + ((size_t)G * R * (R + 1) + 3) / 4 * 4;
  float* const qhat_s = n_s + R * NLD;
  float* const qk_s = qhat_s + G * R;

  const int bkv = blockIdx.x;
  const int b = bkv / a.Hkv, kvh = bkv - b * a.Hkv;
  const int g = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int bh = b * a.Hq + kvh * G + g;
  const bool row = lane < R;
  const int li = row ? lane : 0;  // keeps the loads of idle lanes in bounds
  const float* qp = a.q + (size_t)bh * kD;
  const char* kp = static_cast<const char*>(a.k_new) + (size_t)bkv * ROWB;
  const float qk_part = qp[lane] * kv_load<BF16>(kp, lane) +
                        qp[lane + 64] * kv_load<BF16>(kp, lane + 64);
  // P = B_Q B_Q^T + lambda_d2 A_Om^T A_Om,  cvec = q B_Q^T + lambda_d2 q K_Om^T A_Om;
  // N = B_K B_K^T,  nb = k B_K^T.  The chunk partials are added in chunk order.  They are
  // read with consecutive lanes on consecutive 16-byte pieces and turned into "lane = row"
  // through LDS.
  float p[R], pt[R], m[R];
  float cvec, nb;
  {
    constexpr int U = (kEntries / 4 + 63) / 64;  // 16-byte pieces of an r x r matrix per lane
    const float* gq = a.gram_q + (size_t)bh * (kEntries + R);
    const float* gk = a.gram_k + (size_t)bkv * (kEntries + R);
    constexpr bool kHoist = U <= 4;  // large r: too many registers to hold them that long
    float4 acc[U], vq[U], vk[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      acc[u] = make_float4(0.f, 0.f, 0.f, 0.f);
      const int e4 = lane + 64 * u;  // issued first: these loads overlap the first round below
      const bool on = kHoist && e4 < kEntries / 4;
      vq[u] = on ? reinterpret_cast<const float4*>(gq)[e4] : acc[u];
      vk[u] = (on && g == 0) ? reinterpret_cast<const float4*>(gk)[e4] : acc[u];
    }
    const float cq = gq[kEntries + li];
    nb = gk[kEntries + li];
    float gsum = 0.0f;
    // chunks whose loads are in flight together (the partials were written by the previous
    // kernel and come from memory, so each round of loads costs a full memory latency)
    constexpr int SB = U >= 16 ? 2 : (U >= 4 ? 8 : 16);
    const float* go0 = a.gram_om + (size_t)bh * a.nchunk * (kEntries + R);
    for (int s0 = 0; s0 < a.nchunk; s0 += SB) {
      float4 v[SB][U];
      float gv[SB];
#pragma unroll
      for (int j = 0; j < SB; ++j) {
        const bool on = s0 + j < a.nchunk;
        const float* go = go0 + (size_t)(on ? s0 + j : s0) * (kEntries + R);
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const int e4 = lane + 64 * u;
          v[j][u] = (on && e4 < kEntries / 4) ? reinterpret_cast<const float4*>(go)[e4]
                                              : make_float4(0.f, 0.f, 0.f, 0.f);
        }
        gv[j] = on ? go[kEntries + li] : 0.0f;
      }
#pragma unroll
      for (int j = 0; j < SB; ++j) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
          acc[u].x += v[j][u].x; acc[u].y += v[j][u].y;
          acc[u].z += v[j][u].z; acc[u].w += v[j][u].w;
        }
        gsum += gv[j];
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int e4 = lane + 64 * u;
      if (e4 < kEntries / 4) {
        if (!kHoist) {
          vq[u] = reinterpret_cast<const float4*>(gq)[e4];
          if (g == 0) vk[u] = reinterpret_cast<const float4*>(gk)[e4];
        }
        const int e = 4 * e4, rr = e / R, cc = e % R;
        lt[rr * (R + 1) + cc + 0] = __builtin_fmaf(a.lam2, acc[u].x, vq[u].x);
        lt[rr * (R + 1) + cc + 1] = __builtin_fmaf(a.lam2, acc[u].y, vq[u].y);
        lt[rr * (R + 1) + cc + 2] = __builtin_fmaf(a.lam2, acc[u].z, vq[u].z);
        lt[rr * (R + 1) + cc + 3] = __builtin_fmaf(a.lam2, acc[u].w, vq[u].w);
        if (g == 0) *reinterpret_cast<float4*>(&n_s[rr * NLD + cc]) = vk[u];
      }
    }
    cvec = __builtin_fmaf(a.lam2, gsum, cq);
    __syncthreads();  // n_s (and, within the wavefront, lt) is complete
#pragma unroll
    for (int c = 0; c < R; ++c) p[c] = lt[li * (R + 1) + c];
#pragma unroll
    for (int c4 = 0; c4 < R / 4; ++c4) {
      const float4 vk = *reinterpret_cast<const float4*>(&n_s[li * NLD + 4 * c4]);
      m[4 * c4 + 0] = vk.x; m[4 * c4 + 1] = vk.y; m[4 * c4 + 2] = vk.z; m[4 * c4 + 3] = vk.w;
    }
  }

  // q . k of this query head
  const float qk = wave_sum(qk_part);
  if (lane == 0) qk_s[g] = qk;
  // Factorise N (for the initial guess) and P (kept for every round) together.
  float dN, dP;
  chol_factor2<R>(m, p, dN, dP, lane);
  // initial guess (lambda_d1 = 0): k_hat = k B_K^T (B_K B_K^T)^-1
  float k_hat = tri_forward<R>(m, dN, nb, lane);
  transpose_rows<R>(m, m, lt, lane);
  k_hat = tri_backward<R>(m, dN, k_hat, lane);
  // y0 = cvec P^-1
  transpose_rows<R>(p, pt, lt, lane);
  const float y0 = tri_backward<R>(pt, dP, tri_forward<R>(p, dP, cvec, lane), lane);
  float q_hat = 0.0f;
  for (int it = 0; it < a.n_iter; ++it) {
    // q_hat = m_lq M_rq^-1 with M_rq = P + lambda_d1 k_hat^T k_hat a rank-one change of P:
    //   z = k_hat P^-1,  v = m_lq P^-1 = y0 + lambda_d1 (q.k) z,
    //   q_hat = v - z * lambda_d1 (k_hat . v) / (1 + lambda_d1 (k_hat . z))
    const float z = tri_backward<R>(pt, dP, tri_forward<R>(p, dP, k_hat, lane), lane);
    const float v = __builtin_fmaf(a.lam1 * qk, z, y0);
    const float kv_ = wave_sum(row ? k_hat * v : 0.0f);
    const float kz = wave_sum(row ? k_hat * z : 0.0f);
    q_hat = __builtin_fmaf(-z, a.lam1 * kv_ / __builtin_fmaf(a.lam1, kz, 1.0f), v);
    __syncthreads();  // the previous round's q_hat has been read by every wavefront
    if (row) qhat_s[g * R + lane] = q_hat;
    __syncthreads();
    // k_hat = (k B_K^T + lambda_d1 sum_g (q_g.k) q_hat_g)
    //         (B_K B_K^T + lambda_d1 sum_g q_hat_g^T q_hat_g)^-1
    float rhs = nb;
#pragma unroll
    for (int c4 = 0; c4 < R / 4; ++c4) {
      const float4 vk = *reinterpret_cast<const float4*>(&n_s[li * NLD + 4 * c4]);
      m[4 * c4 + 0] = vk.x; m[4 * c4 + 1] = vk.y; m[4 * c4 + 2] = vk.z; m[4 * c4 + 3] = vk.w;
    }
    for (int gg = 0; gg < G; ++gg) {
      const float qi = qhat_s[gg * R + li];
      rhs = __builtin_fmaf(a.lam1 * qk_s[gg], qi, rhs);
#pragma unroll
      for (int c = 0; c < R; ++c) m[c] = __builtin_fmaf(a.lam1 * qi, qhat_s[gg * R + c], m[c]);
    }
    const float dM = chol_factor<R>(m, lane);
    k_hat = tri_forward<R>(m, dM, rhs, lane);
    transpose_rows<R>(m, m, lt, lane);
    k_hat = tri_backward<R>(m, dM, k_hat, lane);
  }
  if (row) a.q_hat[(size_t)bh * R + lane] = q_hat;
  if (row && g == 0) a.k_hat[(size_t)bkv * R + lane] = k_hat;

  // gradient steps on B_Q (every wavefront its head) and B_K (the first wavefront)
  line_search_step<R>(q_hat, a.B_Q + (size_t)bh * R * kD, [&](int j) { return qp[j]; }, lane);
  if (g == 0)
    line_search_step<R>(k_hat, a.B_K + (size_t)bkv * R * kD,
                        [&](int j) { return kv_load<BF16>(kp, j); }, lane);
}

template <int R, bool BF16>
hipError_t launch_update_r(const lrqk_shape& s, const GramArgs& ga, const SolveArgs& sa,
                           hipStream_t st) {
  const int G = s.Hq / s.Hkv;
  hipLaunchKernelGGL((factor_gram_kernel<R, BF16>), dim3(ga.nchunk + 2, s.B * s.Hq),
                     dim3(kGramThreads), 0, st, ga);
  const size_t lds =
      (((size_t)G * R * (R + 1) + 3) / 4 * 4 + (size_t)R * (R + 4) + (size_t)G * R + G) *
      sizeof(float);
  if (lds > 64 * 1024) {  // above the default limit the kernel has to opt in, once
    static bool raised = false;
    if (!raised) {
      const hipError_t e = hipFuncSetAttribute(
          reinterpret_cast<const void*>(factor_solve_kernel<R, BF16>),
          hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
      if (e != hipSuccess) return e;
      raised = true;
    }
  }
  hipLaunchKernelGGL((factor_solve_kernel<R, BF16>), dim3(s.B * s.Hkv), dim3(G * 64), lds, st,
                     sa);
  return hipGetLastError();
}

template <int R>
hipError_t launch_update_dtype(bool bf16, const lrqk_shape& s, const GramArgs& ga,
                               const SolveArgs& sa, hipStream_t st) {
  return bf16 ? launch_update_r<R, true>(s, ga, sa, st) : launch_update_r<R, false>(s, ga, sa, st);
}

}  // namespace

bool factor_update_supported(const lrqk_shape& s) {
  return s.r == 8 || s.r == 16 || s.r == 32 || s.r == 64;
}

UpdateGeom update_geometry(const lrqk_shape& s) {
  UpdateGeom g;
  // as few chunks of at most one LDS batch as cover the k + w rows, evenly sized
  g.nchunk = ceil_div(s.k + s.w, kGramBatch);
  g.chunk_rows = ceil_div(ceil_div(s.k + s.w, g.nchunk), 16) * 16;
  g.per_gram = (size_t)s.r * s.r + s.r;
  return g;
}

size_t update_ws_bytes(const lrqk_shape& s) {
  const UpdateGeom g = update_geometry(s);
  const size_t BHq = (size_t)s.B * s.Hq, BHkv = (size_t)s.B * s.Hkv;
  return round_up((BHq * g.nchunk + BHq + BHkv) * g.per_gram * sizeof(float), 256);
}

hipError_t launch_factor_update(const lrqk_shape& s, const float* A_K, const void* cacheK,
                                const void* liteK, const int32_t* sel_idx_prev,
                                const int32_t* sel_slot_prev, const float* q, const void* k_new,
                                float* B_Q, float* B_K, float lam1, float lam2, int n_iter,
                                float* q_hat, float* k_hat, float* ws, hipStream_t st) {
  const UpdateGeom g = update_geometry(s);
  const size_t BHq = (size_t)s.B * s.Hq;
  GramArgs ga;
  ga.A_K = A_K; ga.cacheK = cacheK; ga.liteK = liteK;
  ga.sel_idx_prev = sel_idx_prev; ga.sel_slot_prev = sel_slot_prev;
  ga.q = q; ga.k_new = k_new; ga.B_Q = B_Q; ga.B_K = B_K;
  ga.gram_om = ws;
  ga.gram_q = ws + BHq * g.nchunk * g.per_gram;
  ga.gram_k = ga.gram_q + BHq * g.per_gram;
  ga.Hq = s.Hq; ga.Hkv = s.Hkv; ga.l = s.l; ga.l_rows = row_cap(s); ga.k = s.k; ga.w = s.w; ga.C = s.C;
  ga.nchunk = g.nchunk; ga.chunk_rows = g.chunk_rows;
  SolveArgs sa;
  sa.gram_om = ga.gram_om; sa.gram_q = ga.gram_q; sa.gram_k = ga.gram_k;
  sa.q = q; sa.k_new = k_new; sa.B_Q = B_Q; sa.B_K = B_K; sa.q_hat = q_hat; sa.k_hat = k_hat;
  sa.Hq = s.Hq; sa.Hkv = s.Hkv; sa.nchunk = g.nchunk; sa.n_iter = n_iter;
  sa.lam1 = lam1; sa.lam2 = lam2;
  const bool bf16 = s.kv_dtype == LRQK_KV_BF16;
  switch (s.r) {
    case 8: return launch_update_dtype<8>(bf16, s, ga, sa, st);
    case 16: return launch_update_dtype<16>(bf16, s, ga, sa, st);
    case 32: return launch_update_dtype<32>(bf16, s, ga, sa, st);
    case 64: return launch_update_dtype<64>(bf16, s, ga, sa, st);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace lrqk
