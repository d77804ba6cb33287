// p1 -- prefill factorisation (Alg. 1; Sec. 4.1 "Prefill": the four update rules; App. A.1).
//
// Every update of Alg. 1 is made of two kinds of products with one long dimension (l):
//   "reduce"  X^T Y and X^T X   (r x d and r x r, sums over the l rows)   X = A_Q or A_K
//   "apply"   X = Y M           (l x r, row by row)                      Y = Q or K, M d x r
// and r x r solves in between.  Per row of Y (256 bytes in bf16) the products cost
// 2 r (2 d + r) flops: about 50 flop per byte at r = 32, above what the chip's fp32 rate can
// do per byte of HBM traffic.  This is the one dense contraction of the method, and it runs
// on the matrix cores in fp32 (v_mfma_f32_32x32x2_f32; App. B.1 keeps these updates in fp32).
//
// prefill_pass_kernel<R, BF16, APPLY, REDUCE>: one workgroup (4 wavefronts) walks a chunk of
// 2048 rows in tiles of 128.  The tile of Y is read with coalesced 16-byte loads (the next
// tile's loads are issued before the current tile's MFMAs) and kept in LDS as it is (bf16 pairs
// are widened when an operand is read) with an odd row stride in dwords, so that both operand
// shapes the MFMAs need (a column pair of 32 rows, a row pair of 32 columns) are conflict-free
// LDS reads; with bf16 inputs a workgroup needs 66 KB of LDS at r = 32 and two of them share
// a CU, one running MFMAs while the other moves its tile.
//   APPLY : wavefront w computes rows 32w..32w+31 of X = Y M (64 MFMAs per 32 x 32 block),
//           writes them to HBM and into LDS;
//   REDUCE: wavefront w accumulates the 32-column block w of X^T Y over the tile's 128 rows
//           (64 MFMAs per block) and its quarter of the rows of X^T X; the accumulators stay
//           in registers across the chunk and leave as one partial per chunk.
// Fusing the two means Y is read once per update of A and X is never read back.
// prefill_sum_kernel adds the chunk partials (fixed order); the three solve kernels do the
// r x r work: a Cholesky factorisation inside one wavefront, then one thread per column of
// the r x d right-hand side.
#include "lrqk_device.h"
#include "lrqk_internal.h"
#include "lrqk_linalg.h"

namespace lrqk {
namespace {

using namespace linalg;

typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kPfThreads = 256;
constexpr int kPfTile = 128;          // rows per tile: 32 per wavefront
constexpr int kPfTilesPerChunk = 16;  // 2048 rows per workgroup
constexpr int kLDY = kD + 1;          // LDS row stride of the Y tile (odd: conflict-free)

__device__ __forceinline__ f32x16 mfma32(float a, float b, f32x16 c) {
  // D(32x32) = A(32x2) B(2x32) + C; lane = i + 32 k supplies A[i][k] and B[k][i];
  // register v of lane l holds D[8 (v / 4) + 4 (l / 32) + v % 4][l % 32]
  return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ int mfma_row(int v, int lane) {
  return 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
}

template <int R>
struct PfShape {
  static constexpr int RB = (R + 31) / 32;  // 32-wide blocks of the rank dimension
  static constexpr int RP = 32 * RB;        // rank padded to the MFMA block
  static constexpr int LDX = RP + 1;
  static constexpr int P = R * (kD + R);    // floats of one partial: X^T Y then X^T X
  // dwords per LDS row of the Y tile: fp32 values, or bf16 pairs as they come from memory;
  // odd in both cases, so that 32 consecutive rows fall on 32 different banks
  static constexpr int ldy(bool bf16) { return bf16 ? kD / 2 + 1 : kD + 1; }
  static constexpr size_t lds_floats(bool bf16, bool apply) {
    return (size_t)kPfTile * ldy(bf16) + (size_t)kPfTile * LDX + (apply ? (size_t)kD * RP : 0);
  }
};

template <int R, bool BF16, bool APPLY, bool REDUCE>
__global__ __launch_bounds__(kPfThreads) void prefill_pass_kernel(
    const void* __restrict__ Y,   // [heads][l][d]
    float* X,                     // [heads][xrows][R]  read (!APPLY) or written (APPLY)
    const float* __restrict__ M,  // [heads][d][RP]     (APPLY)
    float* __restrict__ part,     // [heads][nchunk][P] (REDUCE)
    int l, int xrows, int nchunk) {
  using S = PfShape<R>;
  constexpr int RB = S::RB, RP = S::RP, LDX = S::LDX;
  constexpr int ROW16 = kD * (BF16 ? 2 : 4) / 16;          // 16-byte pieces per row of Y
  constexpr int NPRE = kPfTile * ROW16 / kPfThreads;       // pieces per thread and tile
  extern __shared__ __align__(16) float pf_lds[];
  constexpr int YW = S::ldy(BF16);
  uint32_t* const Yw = reinterpret_cast<uint32_t*>(pf_lds);  // the Y tile, [kPfTile][YW] dwords
  float* const Xs = pf_lds + kPfTile * YW;
  float* const Ms = Xs + kPfTile * LDX;
  static_assert(kPfTile * (YW + LDX) >= 4 * RP * RP, "room for the final sum of X^T X");
  // element (row, col) of the Y tile as fp32
  auto y_at = [&](int row, int col) -> float {
    if (BF16) {
      const uint32_t wd = Yw[row * YW + (col >> 1)];
      return __uint_as_float((col & 1) ? (wd & 0xffff0000u) : (wd << 16));
    }
    return __uint_as_float(Yw[row * YW + col]);
  };

  const int head = blockIdx.y, chunk = blockIdx.x;
  const int t = threadIdx.x, lane = t & 63, w = t >> 6;
  const int mi = lane & 31, mk = lane >> 5;
  const uint4* __restrict__ Yh =
      reinterpret_cast<const uint4*>(static_cast<const char*>(Y) +
                                     (size_t)head * (size_t)l * (kD * (BF16 ? 2 : 4)));
  float* Xh = X + (size_t)head * (size_t)xrows * R;
  const int row_begin = chunk * kPfTile * kPfTilesPerChunk;
  const int row_end = min(l, row_begin + kPfTile * kPfTilesPerChunk);

  // padding columns of X (rank up to the MFMA block) stay zero for the whole kernel
  if (RP > R)
    for (int i = t; i < kPfTile * (RP - R); i += kPfThreads)
      Xs[(i / (RP - R)) * LDX + R + i % (RP - R)] = 0.0f;
  if (APPLY) {
    const float* Mh = M + (size_t)head * kD * RP;
    for (int i = t; i < kD * RP; i += kPfThreads) Ms[i] = Mh[i];
  }

  f32x16 accXY[RB], accXY1[RB], accXX[RB * RB];
#pragma unroll
  for (int i = 0; i < RB; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) accXY[i][v] = accXY1[i][v] = 0.0f;
#pragma unroll
  for (int i = 0; i < RB * RB; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) accXX[i][v] = 0.0f;

  uint4 pre[NPRE];
  auto prefetch = [&](int row0) {
#pragma unroll
    for (int j = 0; j < NPRE; ++j) {
      const int q = t + kPfThreads * j;
      const int row = row0 + q / ROW16;
      pre[j] = row < row_end ? Yh[(size_t)row * ROW16 + q % ROW16] : make_uint4(0u, 0u, 0u, 0u);
    }
  };
  prefetch(row_begin);

  for (int row0 = row_begin; row0 < row_end; row0 += kPfTile) {
    __syncthreads();  // the previous tile's LDS reads are done
#pragma unroll
    for (int j = 0; j < NPRE; ++j) {
      const int q = t + kPfThreads * j;
      const int rr = q / ROW16, c = q % ROW16;
      uint32_t* dst = Yw + rr * YW + 4 * c;  // bf16: 8 values in 4 dwords; fp32: 4 values
      dst[0] = pre[j].x;
      dst[1] = pre[j].y;
      dst[2] = pre[j].z;
      dst[3] = pre[j].w;
    }
    if (!APPLY) {
      // X tile from HBM: 128 consecutive rows of R floats are one contiguous span
      for (int i = t; i < kPfTile * R / 4; i += kPfThreads) {
        const int rr = (4 * i) / R, cc = (4 * i) % R;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (row0 + rr < row_end)
          v = reinterpret_cast<const float4*>(Xh + (size_t)row0 * R)[i];
        Xs[rr * LDX + cc + 0] = v.x; Xs[rr * LDX + cc + 1] = v.y;
        Xs[rr * LDX + cc + 2] = v.z; Xs[rr * LDX + cc + 3] = v.w;
      }
    }
    if (row0 + kPfTile < row_end) prefetch(row0 + kPfTile);
    __syncthreads();

    if (APPLY) {
      // rows 32w .. 32w+31 of X = Y M
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) {
        // two accumulators, so that consecutive MFMAs do not wait for each other's result
        f32x16 acc, acc1;
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[v] = acc1[v] = 0.0f;
#pragma unroll 4
        for (int kk = 0; kk < kD; kk += 4) {
          acc = mfma32(y_at(32 * w + mi, kk + mk), Ms[(kk + mk) * RP + 32 * rb + mi], acc);
          acc1 = mfma32(y_at(32 * w + mi, kk + 2 + mk), Ms[(kk + 2 + mk) * RP + 32 * rb + mi],
                        acc1);
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[v] += acc1[v];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int i = 32 * w + mfma_row(v, lane), j = 32 * rb + mi;
          if (j < R) {
            Xs[i * LDX + j] = acc[v];
            if (row0 + i < row_end) Xh[(size_t)(row0 + i) * R + j] = acc[v];
          }
        }
      }
      if (REDUCE) __syncthreads();
    }

    if (REDUCE) {
      // block w of the d columns of X^T Y over all 128 rows of the tile (two accumulator sets,
      // row pairs alternate between them), and this wavefront's quarter of the rows of X^T X,
      // interleaved with it: consecutive MFMAs never wait for each other's result
      auto xy_step = [&](int kk) {
        const float b0 = y_at(kk + mk, 32 * w + mi), b1 = y_at(kk + 2 + mk, 32 * w + mi);
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
          accXY[rb] = mfma32(Xs[(kk + mk) * LDX + 32 * rb + mi], b0, accXY[rb]);
          accXY1[rb] = mfma32(Xs[(kk + 2 + mk) * LDX + 32 * rb + mi], b1, accXY1[rb]);
        }
      };
#pragma unroll 2
      for (int kk = 0; kk < 32; kk += 4) {
        xy_step(kk);
#pragma unroll
        for (int h = 0; h < 4; h += 2) {
          float a[RB];
#pragma unroll
          for (int rb = 0; rb < RB; ++rb)
            a[rb] = Xs[(32 * w + kk + h + mk) * LDX + 32 * rb + mi];
#pragma unroll
          for (int r1 = 0; r1 < RB; ++r1)
#pragma unroll
            for (int r2 = 0; r2 < RB; ++r2)
              accXX[r1 * RB + r2] = mfma32(a[r1], a[r2], accXX[r1 * RB + r2]);
        }
      }
#pragma unroll 4
      for (int kk = 32; kk < kPfTile; kk += 4) xy_step(kk);
    }
  }

  if (REDUCE) {
    float* out = part + ((size_t)head * nchunk + chunk) * S::P;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int i = 32 * rb + mfma_row(v, lane);
        if (i < R) out[(size_t)i * kD + 32 * w + mi] = accXY[rb][v] + accXY1[rb][v];
      }
    // X^T X: add the four wavefronts' parts through LDS (the Y tile's space)
    __syncthreads();
    float* red = pf_lds;  // [4][RP * RP], over the tiles' space
#pragma unroll
    for (int r1 = 0; r1 < RB; ++r1)
#pragma unroll
      for (int r2 = 0; r2 < RB; ++r2)
#pragma unroll
        for (int v = 0; v < 16; ++v)
          red[w * RP * RP + (32 * r1 + mfma_row(v, lane)) * RP + 32 * r2 + mi] =
              accXX[r1 * RB + r2][v];
    __syncthreads();
    for (int e = t; e < R * R; e += kPfThreads) {
      const int i = e / R, c = e % R;
      out[(size_t)R * kD + e] = (red[0 * RP * RP + i * RP + c] + red[1 * RP * RP + i * RP + c]) +
                                (red[2 * RP * RP + i * RP + c] + red[3 * RP * RP + i * RP + c]);
    }
  }
}

// sum[head][e] = sum over chunks of part[head][chunk][e], chunks in order
__global__ __launch_bounds__(256) void prefill_sum_kernel(const float* __restrict__ part,
                                                          float* __restrict__ sum, int nchunk,
                                                          int P) {
  const int head = blockIdx.y;
  const int e = blockIdx.x * 256 + threadIdx.x;
  if (e >= P) return;
  const float* p = part + (size_t)head * nchunk * P + e;
  float acc = 0.0f;
  int c = 0;
  for (; c + 8 <= nchunk; c += 8) {
    float v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = p[(size_t)(c + j) * P];
#pragma unroll
    for (int j = 0; j < 8; ++j) acc += v[j];
  }
  for (; c < nchunk; ++c) acc += p[(size_t)c * P];
  sum[(size_t)head * P + e] = acc;
}

// ------------------------------------------------------------------------------------------
// LDS row stride of an r x r system: four consecutive elements of a row are one 16-byte read.
template <int R>
constexpr int kLDS = R + 4;

// Solves S Xs = Ys in place for a symmetric positive definite S (r x r, LDS, row stride
// kLDS<R> = R + 4 floats so that four consecutive elements of a row are one 16-byte read;
// destroyed) and an r x d right-hand side (LDS, row stride kLDY).  The first wavefront
// factorises S (lane = row) and leaves L and 1 / diag(L) in LDS; then thread j < d owns
// column j and runs the two triangular solves in 4 x 4 blocks: the block of the factor is
// read as broadcasts (four 16-byte reads), four elements of the column come from LDS, sixteen
// multiply-adds follow.  Called by all threads of a 256-thread workgroup.
template <int R>
__device__ void spd_solve_columns(float* Ssh, float* dinv_sh, float* Ysh) {
  constexpr int LDS_ = kLDS<R>;
  static_assert(R % 4 == 0, "4 x 4 blocks");
  const int t = threadIdx.x;
  __syncthreads();
  if (t < 64) {
    float m[R];
    const int li = t < R ? t : 0;
#pragma unroll
    for (int c = 0; c < R; ++c) m[c] = Ssh[li * LDS_ + c];
    const float dinv = chol_factor<R>(m, t);
    if (t < R) {
#pragma unroll
      for (int c = 0; c < R; ++c) Ssh[t * LDS_ + c] = m[c];  // L[t][c] for c <= t
      dinv_sh[t] = dinv;
    }
  }
  __syncthreads();
  if (t < kD) {
    float* const y = Ysh + t;  // this thread's column, element i at y[i * kLDY]
    auto lrow = [&](int row, int col) {
      return *reinterpret_cast<const float4*>(&Ssh[row * LDS_ + col]);
    };
    // L z = y
#pragma unroll 1
    for (int I = 0; I < R; I += 4) {
      float a0 = y[(I + 0) * kLDY], a1 = y[(I + 1) * kLDY], a2 = y[(I + 2) * kLDY],
            a3 = y[(I + 3) * kLDY];
#pragma unroll 2
      for (int C = 0; C < I; C += 4) {
        const float z0 = y[(C + 0) * kLDY], z1 = y[(C + 1) * kLDY], z2 = y[(C + 2) * kLDY],
                    z3 = y[(C + 3) * kLDY];
        const float4 l0 = lrow(I + 0, C), l1 = lrow(I + 1, C), l2 = lrow(I + 2, C),
                     l3 = lrow(I + 3, C);
        a0 = __builtin_fmaf(-l0.w, z3, __builtin_fmaf(-l0.z, z2, __builtin_fmaf(-l0.y, z1, __builtin_fmaf(-l0.x, z0, a0))));
        a1 = __builtin_fmaf(-l1.w, z3, __builtin_fmaf(-l1.z, z2, __builtin_fmaf(-l1.y, z1, __builtin_fmaf(-l1.x, z0, a1))));
        a2 = __builtin_fmaf(-l2.w, z3, __builtin_fmaf(-l2.z, z2, __builtin_fmaf(-l2.y, z1, __builtin_fmaf(-l2.x, z0, a2))));
        a3 = __builtin_fmaf(-l3.w, z3, __builtin_fmaf(-l3.z, z2, __builtin_fmaf(-l3.y, z1, __builtin_fmaf(-l3.x, z0, a3))));
      }
      const float4 l1 = lrow(I + 1, I), l2 = lrow(I + 2, I), l3 = lrow(I + 3, I);
      a0 *= dinv_sh[I];
      a1 = __builtin_fmaf(-l1.x, a0, a1) * dinv_sh[I + 1];
      a2 = __builtin_fmaf(-l2.y, a1, __builtin_fmaf(-l2.x, a0, a2)) * dinv_sh[I + 2];
      a3 = __builtin_fmaf(-l3.z, a2, __builtin_fmaf(-l3.y, a1, __builtin_fmaf(-l3.x, a0, a3))) *
           dinv_sh[I + 3];
      y[(I + 0) * kLDY] = a0; y[(I + 1) * kLDY] = a1;
      y[(I + 2) * kLDY] = a2; y[(I + 3) * kLDY] = a3;
    }
    // L^T x = z: the block of L^T for rows I.. and columns C.. is rows C.. of L at columns I..
#pragma unroll 1
    for (int I = R - 4; I >= 0; I -= 4) {
      float a0 = y[(I + 0) * kLDY], a1 = y[(I + 1) * kLDY], a2 = y[(I + 2) * kLDY],
            a3 = y[(I + 3) * kLDY];
#pragma unroll 2
      for (int C = I + 4; C < R; C += 4) {
        const float x0 = y[(C + 0) * kLDY], x1 = y[(C + 1) * kLDY], x2 = y[(C + 2) * kLDY],
                    x3 = y[(C + 3) * kLDY];
        const float4 l0 = lrow(C + 0, I), l1 = lrow(C + 1, I), l2 = lrow(C + 2, I),
                     l3 = lrow(C + 3, I);
        a0 = __builtin_fmaf(-l3.x, x3, __builtin_fmaf(-l2.x, x2, __builtin_fmaf(-l1.x, x1, __builtin_fmaf(-l0.x, x0, a0))));
        a1 = __builtin_fmaf(-l3.y, x3, __builtin_fmaf(-l2.y, x2, __builtin_fmaf(-l1.y, x1, __builtin_fmaf(-l0.y, x0, a1))));
        a2 = __builtin_fmaf(-l3.z, x3, __builtin_fmaf(-l2.z, x2, __builtin_fmaf(-l1.z, x1, __builtin_fmaf(-l0.z, x0, a2))));
        a3 = __builtin_fmaf(-l3.w, x3, __builtin_fmaf(-l2.w, x2, __builtin_fmaf(-l1.w, x1, __builtin_fmaf(-l0.w, x0, a3))));
      }
      const float4 l1 = lrow(I + 1, I), l2 = lrow(I + 2, I), l3 = lrow(I + 3, I);
      a3 *= dinv_sh[I + 3];
      a2 = __builtin_fmaf(-l3.z, a3, a2) * dinv_sh[I + 2];
      a1 = __builtin_fmaf(-l3.y, a3, __builtin_fmaf(-l2.y, a2, a1)) * dinv_sh[I + 1];
      a0 = __builtin_fmaf(-l3.x, a3, __builtin_fmaf(-l2.x, a2, __builtin_fmaf(-l1.x, a1, a0))) *
           dinv_sh[I];
      y[(I + 0) * kLDY] = a0; y[(I + 1) * kLDY] = a1;
      y[(I + 2) * kLDY] = a2; y[(I + 3) * kLDY] = a3;
    }
  }
  __syncthreads();
}

// S1a, one workgroup per head (the B*Hq query heads, then the B*Hkv KV heads): from the sums
// (A^T Y | A^T A) of the head,  B = (A^T A)^-1 A^T Y.
template <int R>
__global__ __launch_bounds__(256) void prefill_solve_b_kernel(const float* __restrict__ sum_q,
                                                              const float* __restrict__ sum_k,
                                                              float* __restrict__ B_Q,
                                                              float* __restrict__ B_K, int BHq) {
  using S = PfShape<R>;
  constexpr int LDS_ = kLDS<R>;
  extern __shared__ __align__(16) float pf_lds[];
  float* const Ysh = pf_lds;              // [R][kLDY]
  float* const Ssh = Ysh + R * kLDY;      // [R][R + 4]
  float* const dinv_sh = Ssh + R * LDS_;  // [R]
  const int t = threadIdx.x;
  const bool iskv = (int)blockIdx.x >= BHq;
  const size_t head = iskv ? blockIdx.x - BHq : blockIdx.x;
  const float* sm = (iskv ? sum_k : sum_q) + head * S::P;
  // (unrolled: the loads of several trips are in flight together)
#pragma unroll 8
  for (int e = t; e < R * kD; e += 256) Ysh[(e / kD) * kLDY + e % kD] = sm[e];
#pragma unroll 4
  for (int e = t; e < R * R; e += 256) Ssh[(e / R) * LDS_ + e % R] = sm[R * kD + e];
  spd_solve_columns<R>(Ssh, dinv_sh, Ysh);
  float* Bout = (iskv ? B_K : B_Q) + head * R * kD;
  for (int e = t; e < R * kD; e += 256) Bout[e] = Ysh[(e / kD) * kLDY + e % kD];
}

// S1b, one workgroup per (batch, KV head):
//   M_K = (sum_g Q_g^T A_Q,g + lambda_pK B_K^T)(sum_g A_Q,g^T A_Q,g + lambda_pK B_K B_K^T)^-1,
// the d x r operand of the A_K update, written as [d][RP] (padding columns zero).
template <int R>
__global__ __launch_bounds__(256) void prefill_solve_mk_kernel(const float* __restrict__ sum_q,
                                                               const float* __restrict__ B_K,
                                                               float* __restrict__ Mk, int Hq,
                                                               int Hkv, float lam_pK) {
  using S = PfShape<R>;
  constexpr int LDS_ = kLDS<R>, RP = S::RP;
  extern __shared__ __align__(16) float pf_lds[];
  float* const Wsh = pf_lds;              // [R][kLDY]  W^T
  float* const Bsh = Wsh + R * kLDY;      // [R][kLDY]  B_K
  float* const Ssh = Bsh + R * kLDY;      // [R][R + 4]
  float* const dinv_sh = Ssh + R * LDS_;  // [R]
  const int bkv = blockIdx.x, t = threadIdx.x;
  const int b = bkv / Hkv, kvh = bkv - b * Hkv, G = Hq / Hkv;
  const float* sq = sum_q + ((size_t)b * Hq + (size_t)kvh * G) * S::P;  // the group's G heads
  const float* Bk = B_K + (size_t)bkv * R * kD;
  // The group's sums are added head by head with the element loops innermost and unrolled, so
  // that the loads of one head are all in flight together (G is not a compile-time constant).
  constexpr int kT1 = R * kD / 256, kT2 = (R * R + 255) / 256;
  float w[kT1], gs[kT2];
#pragma unroll
  for (int u = 0; u < kT1; ++u) {
    const int e = t + 256 * u;
    const float bk = Bk[e];
    Bsh[(e / kD) * kLDY + e % kD] = bk;
    w[u] = lam_pK * bk;
  }
#pragma unroll
  for (int u = 0; u < kT2; ++u) gs[u] = 0.0f;
  for (int g = 0; g < G; ++g) {
    const float* sg = sq + (size_t)g * S::P;
#pragma unroll
    for (int u = 0; u < kT1; ++u) w[u] += sg[t + 256 * u];
#pragma unroll
    for (int u = 0; u < kT2; ++u)
      if (t + 256 * u < R * R) gs[u] += sg[R * kD + t + 256 * u];
  }
#pragma unroll
  for (int u = 0; u < kT1; ++u) {
    const int e = t + 256 * u;
    Wsh[(e / kD) * kLDY + e % kD] = w[u];
  }
  __syncthreads();
#pragma unroll
  for (int u = 0; u < kT2; ++u) {
    const int e = t + 256 * u;
    if (e < R * R) {
      const int i = e / R, c = e % R;
      float bb = 0.0f;
#pragma unroll 16
      for (int j = 0; j < kD; ++j) bb = __builtin_fmaf(Bsh[i * kLDY + j], Bsh[c * kLDY + j], bb);
      Ssh[i * LDS_ + c] = __builtin_fmaf(lam_pK, bb, gs[u]);
    }
  }
  spd_solve_columns<R>(Ssh, dinv_sh, Wsh);  // M_K^T = S^-1 W^T
  float* Mo = Mk + (size_t)bkv * kD * RP;
  for (int e = t; e < kD * RP; e += 256) {
    const int j = e / RP, i = e % RP;
    Mo[e] = i < R ? Wsh[i * kLDY + j] : 0.0f;
  }
}

// S2, one workgroup per (batch, query head): with the sums of the new A_K,
//   M_Q = (K^T A_K + lambda_pQ B_Q^T)(A_K^T A_K + lambda_pQ B_Q B_Q^T)^-1,  written as [d][RP].
template <int R>
__global__ __launch_bounds__(256) void prefill_solve_q_kernel(const float* __restrict__ sum_k,
                                                              const float* __restrict__ B_Q,
                                                              float* __restrict__ Mq, int Hq,
                                                              int Hkv, float lam_pQ) {
  using S = PfShape<R>;
  constexpr int LDS_ = kLDS<R>, RP = S::RP;
  extern __shared__ __align__(16) float pf_lds[];
  float* const Ysh = pf_lds;              // [R][kLDY]
  float* const Bsh = Ysh + R * kLDY;      // [R][kLDY]
  float* const Ssh = Bsh + R * kLDY;      // [R][R + 4]
  float* const dinv_sh = Ssh + R * LDS_;  // [R]
  const int bh = blockIdx.x, t = threadIdx.x;
  const int b = bh / Hq, h = bh - b * Hq, kvh = h / (Hq / Hkv);
  const float* sm = sum_k + ((size_t)b * Hkv + kvh) * S::P;
  const float* Bq = B_Q + (size_t)bh * R * kD;
#pragma unroll 8
  for (int e = t; e < R * kD; e += 256) {
    const float bq = Bq[e];
    Bsh[(e / kD) * kLDY + e % kD] = bq;
    Ysh[(e / kD) * kLDY + e % kD] = __builtin_fmaf(lam_pQ, bq, sm[e]);
  }
  __syncthreads();
  for (int e = t; e < R * R; e += 256) {
    const int i = e / R, c = e % R;
    float acc = 0.0f;
#pragma unroll 16
    for (int j = 0; j < kD; ++j) acc = __builtin_fmaf(Bsh[i * kLDY + j], Bsh[c * kLDY + j], acc);
    Ssh[i * LDS_ + c] = __builtin_fmaf(lam_pQ, acc, sm[R * kD + e]);
  }
  spd_solve_columns<R>(Ssh, dinv_sh, Ysh);
  float* Mo = Mq + (size_t)bh * kD * RP;
  for (int e = t; e < kD * RP; e += 256) {
    const int j = e / RP, i = e % RP;
    Mo[e] = i < R ? Ysh[i * kLDY + j] : 0.0f;
  }
}

// Kernels that use more than 64 KB of dynamic LDS have to opt in (once per kernel).
template <typename K>
hipError_t allow_lds(K kernel, size_t bytes) {
  static bool done = false;  // one flag per kernel type
  if (bytes <= 64 * 1024 || done) return hipSuccess;
  const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
  if (e == hipSuccess) done = true;
  return e;
}
template <int R>
constexpr size_t solve_lds_bytes() {
  return ((size_t)2 * R * kLDY + (size_t)R * kLDS<R> + R) * sizeof(float);
}

template <int R, bool BF16, bool APPLY, bool REDUCE>
hipError_t launch_pass(const void* Y, float* X, const float* M, float* part, int heads, int l,
                       int xrows, int nchunk, hipStream_t st) {
  const size_t lds = PfShape<R>::lds_floats(BF16, APPLY) * sizeof(float);
  auto kernel = prefill_pass_kernel<R, BF16, APPLY, REDUCE>;
  const hipError_t e = allow_lds(kernel, lds);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kernel, dim3(nchunk, heads), dim3(kPfThreads), lds, st, Y, X, M, part, l,
                     xrows, nchunk);
  return hipGetLastError();
}

struct PrefillWs {
  float *part_q, *part_k, *sum_q, *sum_k, *Mq, *Mk;
  size_t floats;
};
template <int R>
PrefillWs carve_prefill(float* base, const lrqk_shape& s) {
  using S = PfShape<R>;
  const size_t BHq = (size_t)s.B * s.Hq, BHkv = (size_t)s.B * s.Hkv;
  const size_t nchunk = (size_t)ceil_div(s.l, kPfTile * kPfTilesPerChunk);
  PrefillWs w;
  size_t off = 0;
  auto take = [&](size_t n) {
    float* p = base ? base + off : nullptr;
    off += (n + 63) / 64 * 64;
    return p;
  };
  w.part_q = take(BHq * nchunk * S::P);
  w.part_k = take(BHkv * nchunk * S::P);
  w.sum_q = take(BHq * S::P);
  w.sum_k = take(BHkv * S::P);
  w.Mq = take(BHq * kD * S::RP);
  w.Mk = take(BHkv * kD * S::RP);
  w.floats = off;
  return w;
}

template <int R, bool BF16>
hipError_t run_prefill(const lrqk_shape& s, const void* Q, const void* K, float* A_Q, float* A_K,
                       float* B_Q, float* B_K, float lam_pQ, float lam_pK, int n_iter, float* ws,
                       hipStream_t st) {
  using S = PfShape<R>;
  const PrefillWs w = carve_prefill<R>(ws, s);
  const int BHq = s.B * s.Hq, BHkv = s.B * s.Hkv, l = s.l, lk = row_cap(s);
  const int nchunk = ceil_div(l, kPfTile * kPfTilesPerChunk);
  const dim3 sum_grid_q(ceil_div(S::P, 256), BHq), sum_grid_k(ceil_div(S::P, 256), BHkv);
  hipError_t e;
#define PF_TRY(x)                  \
  do {                             \
    e = (x);                       \
    if (e != hipSuccess) return e; \
  } while (0)
  // sums of the initial factors
  PF_TRY((launch_pass<R, BF16, false, true>(Q, A_Q, nullptr, w.part_q, BHq, l, l, nchunk, st)));
  PF_TRY((launch_pass<R, BF16, false, true>(K, A_K, nullptr, w.part_k, BHkv, l, lk, nchunk, st)));
  hipLaunchKernelGGL(prefill_sum_kernel, sum_grid_q, dim3(256), 0, st, w.part_q, w.sum_q, nchunk,
                     S::P);
  hipLaunchKernelGGL(prefill_sum_kernel, sum_grid_k, dim3(256), 0, st, w.part_k, w.sum_k, nchunk,
                     S::P);
  for (int it = 0; it < n_iter; ++it) {
    PF_TRY(allow_lds(prefill_solve_b_kernel<R>, solve_lds_bytes<R>()));
    PF_TRY(allow_lds(prefill_solve_mk_kernel<R>, solve_lds_bytes<R>()));
    PF_TRY(allow_lds(prefill_solve_q_kernel<R>, solve_lds_bytes<R>()));
    hipLaunchKernelGGL((prefill_solve_b_kernel<R>), dim3(BHq + BHkv), dim3(256),
                       solve_lds_bytes<R>(), st, w.sum_q, w.sum_k, B_Q, B_K, BHq);
    hipLaunchKernelGGL((prefill_solve_mk_kernel<R>), dim3(BHkv), dim3(256), solve_lds_bytes<R>(),
                       st, w.sum_q, B_K, w.Mk, s.Hq, s.Hkv, lam_pK);
    PF_TRY((launch_pass<R, BF16, true, true>(K, A_K, w.Mk, w.part_k, BHkv, l, lk, nchunk, st)));
    hipLaunchKernelGGL(prefill_sum_kernel, sum_grid_k, dim3(256), 0, st, w.part_k, w.sum_k,
                       nchunk, S::P);
    hipLaunchKernelGGL((prefill_solve_q_kernel<R>), dim3(BHq), dim3(256), solve_lds_bytes<R>(),
                       st, w.sum_k, B_Q, w.Mq, s.Hq, s.Hkv, lam_pQ);
    if (it + 1 < n_iter) {
      PF_TRY((launch_pass<R, BF16, true, true>(Q, A_Q, w.Mq, w.part_q, BHq, l, l, nchunk, st)));
      hipLaunchKernelGGL(prefill_sum_kernel, sum_grid_q, dim3(256), 0, st, w.part_q, w.sum_q,
                         nchunk, S::P);
    } else {  // nothing reads the sums of the final A_Q
      PF_TRY((launch_pass<R, BF16, true, false>(Q, A_Q, w.Mq, nullptr, BHq, l, l, nchunk, st)));
    }
  }
#undef PF_TRY
  return hipGetLastError();
}

template <int R>
hipError_t run_prefill_dtype(const lrqk_shape& s, const void* Q, const void* K, float* A_Q,
                             float* A_K, float* B_Q, float* B_K, float lam_pQ, float lam_pK,
                             int n_iter, float* ws, hipStream_t st) {
  return s.kv_dtype == LRQK_KV_BF16
             ? run_prefill<R, true>(s, Q, K, A_Q, A_K, B_Q, B_K, lam_pQ, lam_pK, n_iter, ws, st)
             : run_prefill<R, false>(s, Q, K, A_Q, A_K, B_Q, B_K, lam_pQ, lam_pK, n_iter, ws, st);
}

}  // namespace

bool prefill_supported(const lrqk_shape& s) {
  return s.r == 8 || s.r == 16 || s.r == 32 || s.r == 64;
}

size_t prefill_ws_bytes(const lrqk_shape& s) {
  size_t f = 0;
  switch (s.r) {
    case 8: f = carve_prefill<8>(nullptr, s).floats; break;
    case 16: f = carve_prefill<16>(nullptr, s).floats; break;
    case 32: f = carve_prefill<32>(nullptr, s).floats; break;
    case 64: f = carve_prefill<64>(nullptr, s).floats; break;
    default: return 0;
  }
  return round_up(f * sizeof(float), 256);
}

hipError_t launch_prefill(const lrqk_shape& s, const void* Q, const void* K, float* A_Q,
                          float* A_K, float* B_Q, float* B_K, float lam_pQ, float lam_pK,
                          int n_iter, float* ws, hipStream_t st) {
  switch (s.r) {
    case 8:
      return run_prefill_dtype<8>(s, Q, K, A_Q, A_K, B_Q, B_K, lam_pQ, lam_pK, n_iter, ws, st);
    case 16:
      return run_prefill_dtype<16>(s, Q, K, A_Q, A_K, B_Q, B_K, lam_pQ, lam_pK, n_iter, ws, st);
    case 32:
      return run_prefill_dtype<32>(s, Q, K, A_Q, A_K, B_Q, B_K, lam_pQ, lam_pK, n_iter, ws, st);
    case 64:
      return run_prefill_dtype<64>(s, Q, K, A_Q, A_K, B_Q, B_K, lam_pQ, lam_pK, n_iter, ws, st);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace lrqk
