// Internal declarations shared by the HIP sources of liblrqk (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include <atomic>

#include "lrqk.h"

namespace lrqk {

constexpr int kWave = 64;           // CDNA wavefront width
constexpr int kD = 128;             // supported head dimension
constexpr int kMaxG = 8;            // query heads per KV head
constexpr int kMaxK = 4096;         // active tokens per head
constexpr int kMaxC = 8192;         // cache slots per head
constexpr int kMaxW = 1024;         // lite tokens
constexpr int kBins = 4096;         // first-level histogram: top 12 bits of the order key
constexpr int kBinShift = 20;
constexpr int kCandCap = 4096;      // candidates of the threshold bin kept per head

// Record a failing HIP call for lrqk_last_hip_error(); returns LRQK_EHIP.
int record_hip_error(hipError_t e);

#define LRQK_HIP(call)                                          \
  do {                                                          \
    hipError_t e__ = (call);                                    \
    if (e__ != hipSuccess) return ::lrqk::record_hip_error(e__); \
  } while (0)

// Instrumentation: kernel launches made through LRQK_LAUNCH by the calling thread attach the
// next pair of these events to the kernel (they then hold the kernel's own start and end) for
// as long as pairs are left; with none left a launch is a plain launch.
struct LaunchTimer {
  hipEvent_t* ev = nullptr;  // pairs: start, stop, start, stop, ...
  int pairs_left = 0;
  unsigned* recorded = nullptr;  // bit i set when pair i of the armed sequence was used
  int next = 0;
};
LaunchTimer& launch_timer();
#define LRQK_LAUNCH(kern, grid, block, lds, st, ...)                                        \
  do {                                                                                      \
    ::lrqk::LaunchTimer& lt__ = ::lrqk::launch_timer();                                     \
    if (lt__.pairs_left > 0) {                                                              \
      hipExtLaunchKernelGGL(kern, grid, block, lds, st, lt__.ev[0], lt__.ev[1], 0,          \
                            __VA_ARGS__);                                                   \
      if (lt__.recorded) *lt__.recorded |= 1u << lt__.next;                                 \
      lt__.ev += 2;                                                                         \
      ++lt__.next;                                                                          \
      --lt__.pairs_left;                                                                    \
    } else {                                                                                \
      hipLaunchKernelGGL(kern, grid, block, lds, st, __VA_ARGS__);                          \
    }                                                                                       \
  } while (0)

// Raises a kernel's dynamic-LDS ceiling once per device (bit d of `done` = done on device d);
// safe to call from several threads (a repeated call is harmless).
template <typename K>
inline hipError_t raise_dynamic_lds_once(K kernel, size_t bytes, std::atomic<uint64_t>& done) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const uint64_t bit = 1ull << (dev & 63);
  if (done.load(std::memory_order_acquire) & bit) return hipSuccess;
  e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
  if (e == hipSuccess) done.fetch_or(bit, std::memory_order_release);
  return e;
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline bool aligned256(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 255u) == 0; }
inline size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline int ceil_div(int a, int b) { return (a + b - 1) / b; }
inline int next_pow2(int x) {
  int p = 1;
  while (p < x) p <<= 1;
  return p;
}
// Rows allocated per head in A_K, the K/V store and slot_of (their row stride).
inline int row_cap(const lrqk_shape& s) { return s.l_cap > 0 ? s.l_cap : s.l; }
inline size_t kv_elem_bytes(int kv_dtype) { return kv_dtype == LRQK_KV_BF16 ? 2 : 4; }

// Layout of the selection workspace (all offsets multiples of 256 bytes).
struct SelectWs {
  uint32_t* hist;      // [BHq][kBins]
  uint32_t* counters;  // [BHq][8]: 0 ticket_hist, 1 ticket_collect, 2 n_out, 3 n_cand, 4 bin, 5 n_above
  int32_t* out_list;   // [BHq][k]      unordered positions in bins above the threshold bin
  uint64_t* cand;      // [BHq][kCandCap]  (key << 32 | ~pos) of the threshold bin
  size_t bytes;
};
SelectWs carve_select_ws(void* base, int BHq, int k);

// Layout of the attention workspace: partial softmax states.
// One partial = [m, s, pad, pad, acc[128]] = 132 floats.
constexpr int kPartialStride = 132;
struct AttendGeom {
  int rows_per_block;  // rows of Omega handled by one workgroup
  int nsplit;          // workgroups per head for k + w rows
};
AttendGeom attend_geometry(int BHq, int k, int w);
size_t attend_ws_bytes(int BHq, int k, int w, int phases);

// ---- kernel launchers (each validates nothing; callers have done so) -------------------
hipError_t launch_proxy_scores(const lrqk_shape& s, const float* A_K, const float* q_hat,
                               float* scores, hipStream_t st);
// Filtered variant of the proxy-score pass (fast shapes only): a sampled threshold bin per
// head, then scores plus a bitmap of the positions at or above that bin.
inline int filter_words64(int n) { return (n + 63) / 64; }
bool proxy_filter_supported(const lrqk_shape& s);
constexpr int kThrMaxSamples = 16384;  // sample scores kept per head
// samples: [BHq][kThrMaxSamples] floats
hipError_t launch_proxy_threshold(const lrqk_shape& s, const float* A_K, const float* q_hat,
                                  float* samples, uint32_t* thr, hipStream_t st);
constexpr int kCandPerGroup = 8;  // candidate scores kept per head and 64-row group
// cand_scores: [BHq][words64][kCandPerGroup] floats
// The threshold key of each head comes from `thr` (keys, e.g. from launch_proxy_threshold) or,
// if `thr` is null, from thr_norm[head] * |q_hat[head]| (the value the previous step's
// selection left for this layer).  Exactly one of the two is given.  thr_out [BHq] receives
// the keys used.
hipError_t launch_proxy_scores_filter(const lrqk_shape& s, const float* A_K, const float* q_hat,
                                      float* scores, const uint32_t* thr, const float* thr_norm,
                                      uint32_t* thr_out, unsigned long long* bitmap,
                                      float* cand_scores, hipStream_t st);
hipError_t launch_select_topk(const lrqk_shape& s, const float* scores, int32_t* sel_idx,
                              const SelectWs& ws, hipStream_t st);
// One workgroup per head, everything in LDS (select_resolve.hip); usable when the
// bitmap of l bits and the other buffers fit (select_resolve_fits).
bool select_resolve_fits(const lrqk_shape& s, bool resolve);
hipError_t launch_select_only(const lrqk_shape& s, const float* scores, int32_t* sel_idx,
                              hipStream_t st);
// ext_bitmap: candidate bitmap written by the filtered proxy-score pass ([BHq][words64]
// 64-bit words); the scores are then recomputed from A_K / q_hat where needed and `scores`
// is only scratch for heads that take the safe route.  With ext_bitmap == nullptr the
// kernel works from the materialised `scores` and A_K / q_hat are ignored.
hipError_t launch_select_resolve(const lrqk_shape& s, float* scores,
                                 const unsigned long long* ext_bitmap, const float* cand_scores,
                                 const float* A_K, const float* q_hat, int32_t* sel_idx,
                                 int32_t step, int32_t* slot_of, int32_t* token_of,
                                 int32_t* last_used, int32_t* sel_slot, uint8_t* hit,
                                 int32_t* miss_tok, int32_t* miss_slot, int32_t* n_miss,
                                 hipStream_t st);
// Selection and resolution straight from the bitmap and packed scores of the filtered
// proxy-score pass (select_packed.hip); usable when select_packed_fits.  thr_used [BHq]: the
// keys that pass filtered with.  sel_thr (may be null) [BHq]: receives the threshold, divided
// by |q_hat|, that the layer's next step should filter with.  scores_w [BHq][l]: scratch for
// heads that need every score.
bool select_packed_fits(const lrqk_shape& s);
hipError_t launch_select_packed(const lrqk_shape& s, const unsigned long long* bitmap,
                                const float* cand_scores, const uint32_t* thr_used,
                                const float* A_K, const float* q_hat, float* scores_w,
                                float* sel_thr, int32_t* sel_idx, int32_t step, int32_t* slot_of,
                                int32_t* token_of, int32_t* last_used, int32_t* sel_slot,
                                uint8_t* hit, int32_t* miss_tok, int32_t* miss_slot,
                                int32_t* n_miss, hipStream_t st);
hipError_t launch_fill_i32(int32_t* p, size_t n, int32_t v, hipStream_t st);
hipError_t launch_cache_init(const lrqk_shape& s, int32_t* slot_of, int32_t* token_of,
                             int32_t* last_used, hipStream_t st);
hipError_t launch_cache_resolve(const lrqk_shape& s, const int32_t* sel_idx, int32_t step,
                                int32_t* slot_of, int32_t* token_of, int32_t* last_used,
                                int32_t* sel_slot, uint8_t* hit, int32_t* miss_tok,
                                int32_t* miss_slot, int32_t* n_miss, hipStream_t st);
// which rows of Omega an attention launch covers
enum AttendMode { kAttendAll = 0, kAttendHitsAndLite = 1, kAttendMisses = 2, kAttendAllFetch = 3 };
hipError_t launch_attend_partial(const lrqk_shape& s, int mode, const float* q, const void* cacheK,
                                 const void* cacheV, const int32_t* sel_slot, const uint8_t* hit,
                                 const int32_t* miss_slot, const int32_t* n_miss,
                                 const void* liteK, const void* liteV, float* partials,
                                 int nblocks, int rows_per_block, int parts_per_head,
                                 int part_offset, hipStream_t st, const void* K_host = nullptr,
                                 const void* V_host = nullptr, const int32_t* sel_idx = nullptr);
// The fetch shared by the query heads of a KV group (one host read per position the group
// misses), alone or in one launch with the attention over the rows that hit.
// link_rows [B,Hkv] (may be null): incremented by the rows read from the host store.
hipError_t launch_group_fetch(const lrqk_shape& s, const void* K_host, const void* V_host,
                              const int32_t* miss_tok, const int32_t* miss_slot,
                              const int32_t* n_miss, void* cacheK, void* cacheV,
                              int32_t* link_rows, hipStream_t st);
hipError_t launch_attend_hits_group_fetch(const lrqk_shape& s, const float* q, void* cacheK,
                                          void* cacheV, const int32_t* sel_slot,
                                          const uint8_t* hit, const void* liteK,
                                          const void* liteV, float* partials, int nblocks,
                                          int rows_per_block, int parts_per_head,
                                          const void* K_host, const void* V_host,
                                          const int32_t* miss_tok, const int32_t* miss_slot,
                                          const int32_t* n_miss, int32_t* link_rows,
                                          hipStream_t st);
hipError_t launch_attend_combine(const lrqk_shape& s, const float* partials, int parts_per_head,
                                 int nparts, float* out, hipStream_t st);
hipError_t launch_fetch_direct(const lrqk_shape& s, const void* K_host, const void* V_host,
                               const int32_t* miss_tok, const int32_t* miss_slot,
                               const int32_t* n_miss, void* cacheK, void* cacheV, hipStream_t st);
// rows staged contiguously as [row][K bytes | V bytes]; row_dst[i] = (bh * C + slot)
hipError_t launch_scatter_staged(const lrqk_shape& s, const void* staging, const int64_t* row_dst,
                                 int64_t n_rows, void* cacheK, void* cacheV, hipStream_t st);

// Decode-time factor update (factor_update.hip): r in {8, 16, 32, 64}.
struct UpdateGeom {
  int chunk_rows;   // rows of Omega summed by one workgroup
  int nchunk;       // workgroups per query head
  size_t per_gram;  // floats of one partial result: r*r + r
};
bool factor_update_supported(const lrqk_shape& s);
UpdateGeom update_geometry(const lrqk_shape& s);
size_t update_ws_bytes(const lrqk_shape& s);
hipError_t launch_factor_update(const lrqk_shape& s, const float* A_K, const void* cacheK,
                                const void* liteK, const int32_t* sel_idx_prev,
                                const int32_t* sel_slot_prev, const float* q, const void* k_new,
                                float* B_Q, float* B_K, float lam1, float lam2, int n_iter,
                                float* q_hat, float* k_hat, float* ws, hipStream_t st);

// The new token's rows: A_K[., l, :], K/V store row l, lite ring row l % w, slot_of[., l] = -1.
hipError_t launch_append_token(const lrqk_shape& s, float* A_K, void* K_host, void* V_host,
                               void* liteK, void* liteV, int32_t* slot_of, const float* k_hat,
                               const void* k_new, const void* v_new, hipStream_t st);

// Prefill factorisation (prefill.hip): r in {8, 16, 32, 64}.
bool prefill_supported(const lrqk_shape& s);
size_t prefill_ws_bytes(const lrqk_shape& s);
hipError_t launch_prefill(const lrqk_shape& s, const void* Q, const void* K, float* A_Q,
                          float* A_K, float* B_Q, float* B_K, float lam_pQ, float lam_pK,
                          int n_iter, float* ws, hipStream_t st);

}  // namespace lrqk
