// C ABI of liblrqk: argument validation, the plan object, the fetch leg's host
// side and the fused decode step.  Every kernel lives in its own source file;
// this file only checks, carves workspaces and enqueues.
#include <atomic>
#include <cmath>
#include <condition_variable>
#include <cstdlib>
#include <cstring>
#include <functional>
#include <mutex>
#include <new>
#include <thread>
#include <vector>

#include "lrqk_internal.h"

namespace lrqk {

static thread_local int g_last_hip_error = 0;

LaunchTimer& launch_timer() {
  static thread_local LaunchTimer t;
  return t;
}

int record_hip_error(hipError_t e) {
  g_last_hip_error = static_cast<int>(e);
  (void)hipGetLastError();  // clear the sticky slot so later calls report their own errors
  return LRQK_EHIP;
}

static int check_shape(const lrqk_shape* s) {
  if (!s) return LRQK_EINVAL;
  if (s->kv_dtype != LRQK_KV_BF16 && s->kv_dtype != LRQK_KV_F32) return LRQK_EINVAL;
  if (s->B < 1 || s->Hq < 1 || s->Hkv < 1 || s->l < 1) return LRQK_ESHAPE;
  if (s->Hq % s->Hkv != 0 || s->Hq / s->Hkv > kMaxG) return LRQK_ESHAPE;
  if (s->d != kD) return LRQK_ESHAPE;
  if (s->r < 4 || s->r > 128 || s->r % 4 != 0) return LRQK_ESHAPE;
  if (s->l >= (1 << 24)) return LRQK_ESHAPE;
  if (s->w < 0 || s->w > kMaxW || s->w > s->l) return LRQK_ESHAPE;
  if (s->k < 1 || s->k > s->l - s->w || s->k > kMaxK) return LRQK_ESHAPE;
  if (s->C < s->k || s->C > kMaxC) return LRQK_ESHAPE;
  if ((long)s->B * s->Hq > 65535) return LRQK_ESHAPE;
  if (!std::isfinite(s->scale)) return LRQK_ESHAPE;
  if (s->l_cap != 0 && (s->l_cap < s->l || s->l_cap >= (1 << 24))) return LRQK_ESHAPE;
  return LRQK_OK;
}

static bool all_aligned16(std::initializer_list<const void*> ps) {
  for (const void* p : ps)
    if (!p || !aligned16(p)) return false;
  return true;
}

// A few host threads that split the row gather of the staged fetch (random 256..512-byte
// reads from the pinned K/V store: one thread is bound by memory latency).
class HostPool {
 public:
  explicit HostPool(int n) {
    for (int i = 0; i < n; ++i) workers_.emplace_back([this, i] { loop(i); });
  }
  ~HostPool() {
    {
      std::lock_guard<std::mutex> g(mu_);
      stop_ = true;
      ++epoch_;
    }
    cv_.notify_all();
    for (auto& w : workers_) w.join();
  }
  int size() const { return (int)workers_.size(); }
  // run fn(worker_index, n_workers) on every worker and wait for all of them
  void run(const std::function<void(int, int)>& fn) {
    {
      std::lock_guard<std::mutex> g(mu_);
      fn_ = &fn;
      pending_ = (int)workers_.size();
      ++epoch_;
    }
    cv_.notify_all();
    std::unique_lock<std::mutex> g(mu_);
    done_.wait(g, [this] { return pending_ == 0; });
    fn_ = nullptr;
  }

 private:
  void loop(int idx) {
    unsigned long seen = 0;
    for (;;) {
      const std::function<void(int, int)>* fn;
      {
        std::unique_lock<std::mutex> g(mu_);
        cv_.wait(g, [&] { return epoch_ != seen; });
        seen = epoch_;
        if (stop_) return;
        fn = fn_;
      }
      (*fn)(idx, (int)workers_.size());
      {
        std::lock_guard<std::mutex> g(mu_);
        if (--pending_ == 0) done_.notify_all();
      }
    }
  }
  std::vector<std::thread> workers_;
  std::mutex mu_;
  std::condition_variable cv_, done_;
  const std::function<void(int, int)>* fn_ = nullptr;
  unsigned long epoch_ = 0;
  int pending_ = 0;
  bool stop_ = false;
};

}  // namespace lrqk

using namespace lrqk;

struct lrqk_plan {
  lrqk_shape max;
  int device;
  int BHq;
  // device
  float* scores;
  uint32_t* thr;               // [BHq] threshold key of each head estimated from a sample
  uint32_t* thr_used;          // [BHq] the keys the last filtered proxy-score pass used
  float* samples;              // [BHq][kThrMaxSamples] sample scores behind thr
  unsigned long long* filter;  // [BHq][words64] candidate bitmap from the proxy-score pass
  float* cand_scores;          // [BHq][words64][kCandPerGroup] the candidates' scores
  void* select_ws;
  size_t select_bytes;
  float* partials;
  size_t partial_bytes;
  int32_t *sel_idx, *sel_slot, *miss_tok, *miss_slot, *n_miss;
  uint8_t* hit;
  void* d_stage;
  int64_t* d_rowdst;
  // pinned host
  int32_t *h_nmiss, *h_miss_tok, *h_miss_slot;
  void* h_stage;
  int64_t* h_rowdst;
  size_t stage_rows;
  hipStream_t side;
  hipEvent_t ev_main, ev_side;
  // optional per-kernel timing of lrqk_decode_step (lrqk_plan_profile)
  int prof_cap, prof_n;
  hipEvent_t* prof_ev;   // [prof_cap][LRQK_PROFILE_SLOTS][start, stop]
  unsigned* prof_used;   // [prof_cap] bit i: slot i was recorded in that step
  HostPool* pool;       // host threads of the staged fetch (created on first use)
  int64_t* h_rowbase;   // [BHq + 1] first staging row of each head (host, not pinned)
};

static void prof_free(lrqk_plan* p) {
  if (p->prof_ev) {
    for (int i = 0; i < p->prof_cap * LRQK_PROFILE_SLOTS * 2; ++i)
      if (p->prof_ev[i]) (void)hipEventDestroy(p->prof_ev[i]);
    std::free(p->prof_ev);
  }
  std::free(p->prof_used);
  p->prof_ev = nullptr;
  p->prof_used = nullptr;
  p->prof_cap = p->prof_n = 0;
}

// The next `count` kernels launched by this thread go to the slots slot, slot + 1, ... of the
// current profiled step (nothing happens when profiling is off or no step is left).
static inline void prof_arm(lrqk_plan* p, int slot, int count) {
  LaunchTimer& t = launch_timer();
  t = LaunchTimer{};
  if (!p->prof_ev || p->prof_n >= p->prof_cap) return;
  t.ev = p->prof_ev + ((size_t)p->prof_n * LRQK_PROFILE_SLOTS + slot) * 2;
  t.pairs_left = count;
  t.recorded = p->prof_used + p->prof_n;
  t.next = slot;
}
// Leaves no events armed for later launches of this thread, whichever way a function returns.
struct LaunchTimerReset {
  ~LaunchTimerReset() { launch_timer() = LaunchTimer{}; }
};
static inline void prof_step_done(lrqk_plan* p) {
  launch_timer() = LaunchTimer{};
  if (p->prof_ev && p->prof_n < p->prof_cap) ++p->prof_n;
}

extern "C" {
#pragma GCC visibility push(default)

int lrqk_version(void) { return LRQK_VERSION; }

const char* lrqk_status_string(int status) {
  switch (status) {
    case LRQK_OK: return "ok";
    case LRQK_EINVAL: return "invalid argument (null or misaligned pointer, bad enum or handle)";
    case LRQK_ESHAPE: return "shape inconsistent or outside the supported range";
    case LRQK_EHIP: return "HIP runtime error (see lrqk_last_hip_error)";
    case LRQK_ENOMEM: return "workspace too small or allocation failed";
    case LRQK_ESTATE: return "unusable cache state";
    default: return "unknown status";
  }
}

int lrqk_last_hip_error(void) { return g_last_hip_error; }

int lrqk_validate_shape(const lrqk_shape* shape) { return check_shape(shape); }

size_t lrqk_workspace_bytes(const lrqk_shape* shape, int which) {
  if (check_shape(shape) != LRQK_OK) return 0;
  const int BHq = shape->B * shape->Hq;
  if (which == LRQK_WS_SELECT) return carve_select_ws(nullptr, BHq, shape->k).bytes;
  if (which == LRQK_WS_ATTEND) return attend_ws_bytes(BHq, shape->k, shape->w, 1);
  if (which == LRQK_WS_UPDATE) return factor_update_supported(*shape) ? update_ws_bytes(*shape) : 0;
  if (which == LRQK_WS_PREFILL) return prefill_supported(*shape) ? prefill_ws_bytes(*shape) : 0;
  return 0;
}

int lrqk_proxy_scores(const lrqk_shape* shape, const float* A_K, const float* q_hat,
                      float* scores, void* stream) {
  const int rc = check_shape(shape);
  if (rc != LRQK_OK) return rc;
  if (!all_aligned16({A_K, q_hat, scores})) return LRQK_EINVAL;
  LRQK_HIP(launch_proxy_scores(*shape, A_K, q_hat, scores, static_cast<hipStream_t>(stream)));
  return LRQK_OK;
}

int lrqk_select_topk(const lrqk_shape* shape, const float* scores, int32_t* sel_idx,
                     void* workspace, size_t ws_bytes, void* stream) {
  const int rc = check_shape(shape);
  if (rc != LRQK_OK) return rc;
  if (!all_aligned16({scores, sel_idx}) || !workspace || !aligned256(workspace)) return LRQK_EINVAL;
  const SelectWs ws = carve_select_ws(workspace, shape->B * shape->Hq, shape->k);
  if (ws_bytes < ws.bytes) return LRQK_ENOMEM;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (select_resolve_fits(*shape, false))
    LRQK_HIP(launch_select_only(*shape, scores, sel_idx, st));
  else
    LRQK_HIP(launch_select_topk(*shape, scores, sel_idx, ws, st));
  return LRQK_OK;
}

int lrqk_cache_init(const lrqk_shape* shape, int32_t* slot_of, int32_t* token_of,
                    int32_t* last_used, void* stream) {
  const int rc = check_shape(shape);
  if (rc != LRQK_OK) return rc;
  if (!all_aligned16({slot_of, token_of, last_used})) return LRQK_EINVAL;
  LRQK_HIP(launch_cache_init(*shape, slot_of, token_of, last_used,
                             static_cast<hipStream_t>(stream)));
  return LRQK_OK;
}

int lrqk_select_state_init(const lrqk_shape* shape, float* sel_thr, void* stream) {
  const int rc = check_shape(shape);
  if (rc != LRQK_OK) return rc;
  if (!all_aligned16({sel_thr})) return LRQK_EINVAL;
  LRQK_HIP(launch_fill_i32(reinterpret_cast<int32_t*>(sel_thr), (size_t)shape->B * shape->Hq,
                           0x7fc00000, static_cast<hipStream_t>(stream)));  // quiet NaN
  return LRQK_OK;
}

int lrqk_cache_resolve(const lrqk_shape* shape, const int32_t* sel_idx, int32_t step,
                       int32_t* slot_of, int32_t* token_of, int32_t* last_used,
                       int32_t* sel_slot, uint8_t* hit, int32_t* miss_tok, int32_t* miss_slot,
                       int32_t* n_miss, void* stream) {
  const int rc = check_shape(shape);
  if (rc != LRQK_OK) return rc;
  if (step < 0 || step == INT32_MAX) return LRQK_EINVAL;
  if (!all_aligned16({sel_idx, slot_of, token_of, last_used, sel_slot, hit, miss_tok, miss_slot,
                      n_miss}))
    return LRQK_EINVAL;
  LRQK_HIP(launch_cache_resolve(*shape, sel_idx, step, slot_of, token_of, last_used, sel_slot,
                                hit, miss_tok, miss_slot, n_miss,
                                static_cast<hipStream_t>(stream)));
  return LRQK_OK;
}

int lrqk_sparse_attend(const lrqk_shape* shape, const float* q, const void* cacheK,
                       const void* cacheV, const int32_t* sel_slot, const void* liteK,
                       const void* liteV, float* out, void* workspace, size_t ws_bytes,
                       void* stream) {
  const int rc = check_shape(shape);
  if (rc != LRQK_OK) return rc;
  if (!all_aligned16({q, cacheK, cacheV, sel_slot, out}) || !workspace || !aligned256(workspace))
    return LRQK_EINVAL;
  if (shape->w > 0 && !all_aligned16({liteK, liteV})) return LRQK_EINVAL;
  const int BHq = shape->B * shape->Hq;
  if (ws_bytes < attend_ws_bytes(BHq, shape->k, shape->w, 1)) return LRQK_ENOMEM;
  const AttendGeom g = attend_geometry(BHq, shape->k, shape->w);
  hipStream_t st = static_cast<hipStream_t>(stream);
  float* partials = static_cast<float*>(workspace);
  LRQK_HIP(launch_attend_partial(*shape, kAttendAll, q, cacheK, cacheV, sel_slot, nullptr, nullptr,
                                 nullptr, liteK, liteV, partials, g.nsplit, g.rows_per_block,
                                 g.nsplit, 0, st));
  LRQK_HIP(launch_attend_combine(*shape, partials, g.nsplit, g.nsplit, out, st));
  return LRQK_OK;
}

int lrqk_factor_update(const lrqk_shape* shape, const lrqk_layer* layer,
                       const int32_t* sel_idx_prev, const int32_t* sel_slot_prev, const float* q,
                       const void* k_new, float* B_Q, float* B_K, float lambda_d1,
                       float lambda_d2, int32_t n_iter, float* q_hat, float* k_hat,
                       void* workspace, size_t ws_bytes, void* stream) {
  const int rc = check_shape(shape);
  if (rc != LRQK_OK) return rc;
  if (!factor_update_supported(*shape)) return LRQK_ESHAPE;
  if (!layer || n_iter < 1 || n_iter > 64) return LRQK_EINVAL;
  if (!(lambda_d1 >= 0.0f) || !(lambda_d2 >= 0.0f) || std::isinf(lambda_d1) ||
      std::isinf(lambda_d2))
    return LRQK_EINVAL;
  if (!all_aligned16({layer->A_K, layer->cacheK, sel_idx_prev, sel_slot_prev, q, k_new, B_Q, B_K,
                      q_hat, k_hat}) ||
      !workspace || !aligned256(workspace))
    return LRQK_EINVAL;
  if (shape->w > 0 && !all_aligned16({layer->liteK})) return LRQK_EINVAL;
  if (ws_bytes < update_ws_bytes(*shape)) return LRQK_ENOMEM;
  LRQK_HIP(launch_factor_update(*shape, layer->A_K, layer->cacheK, layer->liteK, sel_idx_prev,
                                sel_slot_prev, q, k_new, B_Q, B_K, lambda_d1, lambda_d2, n_iter,
                                q_hat, k_hat, static_cast<float*>(workspace),
                                static_cast<hipStream_t>(stream)));
  return LRQK_OK;
}

int lrqk_append_token(const lrqk_shape* shape, const lrqk_layer* layer, const float* k_hat,
                      const void* k_new, const void* v_new, void* stream) {
  const int rc = check_shape(shape);
  if (rc != LRQK_OK) return rc;
  if (row_cap(*shape) <= shape->l) return LRQK_ESHAPE;  // no room for row l
  if (!layer) return LRQK_EINVAL;
  if (!all_aligned16({layer->A_K, layer->K_host, layer->V_host, layer->slot_of, k_hat, k_new,
                      v_new}))
    return LRQK_EINVAL;
  if (shape->w > 0 && !all_aligned16({layer->liteK, layer->liteV})) return LRQK_EINVAL;
  LRQK_HIP(launch_append_token(*shape, layer->A_K, layer->K_host, layer->V_host, layer->liteK,
                               layer->liteV, layer->slot_of, k_hat, k_new, v_new,
                               static_cast<hipStream_t>(stream)));
  return LRQK_OK;
}

int lrqk_prefill_factorize(const lrqk_shape* shape, const void* Q, const void* K, float* A_Q,
                           float* A_K, float* B_Q, float* B_K, float lambda_pQ, float lambda_pK,
                           int32_t n_iter, void* workspace, size_t ws_bytes, void* stream) {
  const int rc = check_shape(shape);
  if (rc != LRQK_OK) return rc;
  if (!prefill_supported(*shape)) return LRQK_ESHAPE;
  if (n_iter < 1 || n_iter > 64) return LRQK_EINVAL;
  if (!(lambda_pQ >= 0.0f) || !(lambda_pK >= 0.0f) || std::isinf(lambda_pQ) ||
      std::isinf(lambda_pK))
    return LRQK_EINVAL;
  if (!all_aligned16({Q, K, A_Q, A_K, B_Q, B_K}) || !workspace || !aligned256(workspace))
    return LRQK_EINVAL;
  if (ws_bytes < prefill_ws_bytes(*shape)) return LRQK_ENOMEM;
  LRQK_HIP(launch_prefill(*shape, Q, K, A_Q, A_K, B_Q, B_K, lambda_pQ, lambda_pK, n_iter,
                          static_cast<float*>(workspace), static_cast<hipStream_t>(stream)));
  return LRQK_OK;
}

// ---------------------------------------------------------------------------- plan

int lrqk_plan_destroy(lrqk_plan* p) {
  if (!p) return LRQK_EINVAL;
  int prev = -1;
  (void)hipGetDevice(&prev);
  (void)hipSetDevice(p->device);
  if (p->side) (void)hipStreamSynchronize(p->side);
  void* dev[] = {p->thr_used, p->scores,   p->thr,      p->samples,  p->filter,    p->cand_scores,
                 p->select_ws, p->partials, p->sel_idx,  p->sel_slot,  p->miss_tok,
                 p->miss_slot, p->n_miss,   p->hit,      p->d_stage,   p->d_rowdst};
  for (void* q : dev)
    if (q) (void)hipFree(q);
  void* host[] = {p->h_nmiss, p->h_miss_tok, p->h_miss_slot, p->h_stage, p->h_rowdst};
  for (void* q : host)
    if (q) (void)hipHostFree(q);
  prof_free(p);
  delete p->pool;
  std::free(p->h_rowbase);
  if (p->ev_main) (void)hipEventDestroy(p->ev_main);
  if (p->ev_side) (void)hipEventDestroy(p->ev_side);
  if (p->side) (void)hipStreamDestroy(p->side);
  if (prev >= 0) (void)hipSetDevice(prev);
  delete p;
  return LRQK_OK;
}

int lrqk_plan_create(const lrqk_shape* max_shape, lrqk_plan** plan_out) {
  if (!plan_out) return LRQK_EINVAL;
  *plan_out = nullptr;
  const int rc = check_shape(max_shape);
  if (rc != LRQK_OK) return rc;
  lrqk_plan* p = new (std::nothrow) lrqk_plan();
  if (!p) return LRQK_ENOMEM;
  std::memset(p, 0, sizeof(*p));
  p->max = *max_shape;
  const lrqk_shape& s = p->max;
  const size_t BHq = (size_t)s.B * s.Hq;
  p->BHq = (int)BHq;
  const size_t rowB = (size_t)s.d * kv_elem_bytes(s.kv_dtype);
  p->select_bytes = carve_select_ws(nullptr, (int)BHq, s.k).bytes;
  p->partial_bytes = attend_ws_bytes((int)BHq, s.k, s.w, 2);
  p->stage_rows = BHq * s.k;
  hipError_t e = hipGetDevice(&p->device);
  auto dmalloc = [&](void** q, size_t bytes) {
    if (e == hipSuccess) e = hipMalloc(q, bytes ? bytes : 256);
  };
  auto hmalloc = [&](void** q, size_t bytes) {
    if (e == hipSuccess) e = hipHostMalloc(q, bytes ? bytes : 256, hipHostMallocDefault);
  };
  dmalloc((void**)&p->scores, BHq * s.l * sizeof(float));
  dmalloc((void**)&p->thr, BHq * 4);
  dmalloc((void**)&p->thr_used, BHq * 4);
  dmalloc((void**)&p->samples, BHq * (size_t)kThrMaxSamples * 4);
  dmalloc((void**)&p->filter, BHq * (size_t)filter_words64(s.l) * 8);
  dmalloc((void**)&p->cand_scores, BHq * (size_t)filter_words64(s.l) * kCandPerGroup * 4);
  dmalloc(&p->select_ws, p->select_bytes);
  dmalloc((void**)&p->partials, p->partial_bytes);
  dmalloc((void**)&p->sel_idx, BHq * s.k * 4);
  dmalloc((void**)&p->sel_slot, BHq * s.k * 4);
  dmalloc((void**)&p->miss_tok, BHq * s.k * 4);
  dmalloc((void**)&p->miss_slot, BHq * s.k * 4);
  dmalloc((void**)&p->n_miss, BHq * 4);
  dmalloc((void**)&p->hit, BHq * s.k);
  dmalloc(&p->d_stage, p->stage_rows * 2 * rowB);
  dmalloc((void**)&p->d_rowdst, p->stage_rows * 8);
  hmalloc((void**)&p->h_nmiss, BHq * 4);
  hmalloc((void**)&p->h_miss_tok, BHq * s.k * 4);
  hmalloc((void**)&p->h_miss_slot, BHq * s.k * 4);
  hmalloc(&p->h_stage, p->stage_rows * 2 * rowB);
  hmalloc((void**)&p->h_rowdst, p->stage_rows * 8);
  if (e == hipSuccess) e = hipStreamCreateWithFlags(&p->side, hipStreamNonBlocking);
  if (e == hipSuccess) e = hipEventCreateWithFlags(&p->ev_main, hipEventDisableTiming);
  if (e == hipSuccess) e = hipEventCreateWithFlags(&p->ev_side, hipEventDisableTiming);
  if (e != hipSuccess) {
    const int code = (e == hipErrorOutOfMemory) ? LRQK_ENOMEM : record_hip_error(e);
    lrqk_plan_destroy(p);
    return code;
  }
  *plan_out = p;
  return LRQK_OK;
}

static int check_plan_fits(const lrqk_plan* p, const lrqk_shape* s) {
  if (!p) return LRQK_EINVAL;
  const lrqk_shape& m = p->max;
  if ((long)s->B * s->Hq > p->BHq || s->l > m.l || s->k > m.k || s->w > m.w || s->C > m.C ||
      s->kv_dtype != m.kv_dtype)
    return LRQK_ESHAPE;
  // the attention partial buffer is sized from (BHq, k, w) of the plan's shape
  if (attend_ws_bytes(s->B * s->Hq, s->k, s->w, 2) > p->partial_bytes) return LRQK_ESHAPE;
  if (carve_select_ws(nullptr, s->B * s->Hq, s->k).bytes > p->select_bytes) return LRQK_ESHAPE;
  return LRQK_OK;
}

// Host side of the staged fetch.  `stream` must already hold the resolve kernel.
// Returns the largest n_miss over heads through *max_nmiss.
static int staged_fetch(lrqk_plan* p, const lrqk_shape& s, const void* K_host, const void* V_host,
                        const int32_t* miss_tok, const int32_t* miss_slot, const int32_t* n_miss,
                        void* cacheK, void* cacheV, hipStream_t stream, bool sync_lists,
                        int64_t* total_out, int* max_nmiss) {
  const size_t BHq = (size_t)s.B * s.Hq;
  const size_t rowB = (size_t)s.d * kv_elem_bytes(s.kv_dtype);
  if (sync_lists) {
    LRQK_HIP(hipMemcpyAsync(p->h_nmiss, n_miss, BHq * 4, hipMemcpyDeviceToHost, stream));
    LRQK_HIP(hipMemcpyAsync(p->h_miss_tok, miss_tok, BHq * s.k * 4, hipMemcpyDeviceToHost, stream));
    LRQK_HIP(hipMemcpyAsync(p->h_miss_slot, miss_slot, BHq * s.k * 4, hipMemcpyDeviceToHost,
                            stream));
    LRQK_HIP(hipStreamSynchronize(stream));
  }
  const int G = s.Hq / s.Hkv;
  const char* Kh = static_cast<const char*>(K_host);
  const char* Vh = static_cast<const char*>(V_host);
  char* stage = static_cast<char*>(p->h_stage);
  // staging rows are laid out head after head: prefix sums of the per-head counts
  if (!p->h_rowbase) {
    p->h_rowbase = static_cast<int64_t*>(std::malloc(((size_t)p->BHq + 1) * sizeof(int64_t)));
    if (!p->h_rowbase) return LRQK_ENOMEM;
  }
  int64_t total = 0;
  int mx = 0;
  // a head whose resolution failed (out of victims, reused step, unusable map) reports -1: its
  // missing rows cannot be fetched, so nothing further is enqueued
  for (size_t bh = 0; bh < BHq; ++bh)
    if (p->h_nmiss[bh] < 0) return LRQK_ESTATE;
  for (size_t bh = 0; bh < BHq; ++bh) {
    const int nm = p->h_nmiss[bh];
    const int cnt = nm <= 0 ? 0 : (nm < s.k ? nm : s.k);
    if (cnt > mx) mx = cnt;
    p->h_rowbase[bh] = total;
    total += cnt;
  }
  p->h_rowbase[BHq] = total;
  auto gather = [&](int widx, int nworkers) {
    // worker widx takes the staging rows [lo, hi)
    const int64_t lo = total * widx / nworkers, hi = total * (widx + 1) / nworkers;
    size_t bh = 0;
    for (int64_t i = lo; i < hi; ++i) {
      while (p->h_rowbase[bh + 1] <= i) ++bh;
      const int j = (int)(i - p->h_rowbase[bh]);
      const size_t b = bh / s.Hq, h = bh % s.Hq, kvh = h / G;
      const int32_t tok = p->h_miss_tok[bh * s.k + j];
      const int32_t slot = p->h_miss_slot[bh * s.k + j];
      if (tok < 0 || tok >= s.l || slot < 0 || slot >= s.C) {
        p->h_rowdst[i] = -1;  // skipped by the scatter kernel
        continue;
      }
      const char* Ks = Kh + ((b * s.Hkv + kvh) * (size_t)row_cap(s) + (size_t)tok) * rowB;
      const char* Vs = Vh + ((b * s.Hkv + kvh) * (size_t)row_cap(s) + (size_t)tok) * rowB;
      std::memcpy(stage + (size_t)i * 2 * rowB, Ks, rowB);
      std::memcpy(stage + (size_t)i * 2 * rowB + rowB, Vs, rowB);
      p->h_rowdst[i] = (int64_t)bh * s.C + slot;
    }
  };
  if (total >= 256) {
    if (!p->pool) {
      unsigned hw = std::thread::hardware_concurrency();
      int nthreads = hw == 0 ? 4 : (hw > 16 ? 8 : (int)(hw / 2));
      if (nthreads < 1) nthreads = 1;
      p->pool = new (std::nothrow) HostPool(nthreads);
      if (!p->pool) return LRQK_ENOMEM;
    }
    p->pool->run(gather);
  } else if (total > 0) {
    gather(0, 1);
  }
  if (max_nmiss) *max_nmiss = mx;
  if (total_out) *total_out = total;
  if (total > 0) {
    LRQK_HIP(hipMemcpyAsync(p->d_stage, p->h_stage, (size_t)total * 2 * rowB,
                            hipMemcpyHostToDevice, p->side));
    LRQK_HIP(hipMemcpyAsync(p->d_rowdst, p->h_rowdst, (size_t)total * 8, hipMemcpyHostToDevice,
                            p->side));
    LRQK_HIP(launch_scatter_staged(s, p->d_stage, p->d_rowdst, total, cacheK, cacheV, p->side));
    LRQK_HIP(hipEventRecord(p->ev_side, p->side));
    LRQK_HIP(hipStreamWaitEvent(stream, p->ev_side, 0));
  }
  return LRQK_OK;
}

int lrqk_fetch_misses(lrqk_plan* plan, const lrqk_shape* shape, const void* K_host,
                      const void* V_host, const int32_t* miss_tok, const int32_t* miss_slot,
                      const int32_t* n_miss, void* cacheK, void* cacheV, int mode,
                      int64_t* total_miss_out, void* stream) {
  int rc = check_shape(shape);
  if (rc != LRQK_OK) return rc;
  if (mode != LRQK_FETCH_STAGED && mode != LRQK_FETCH_DIRECT && mode != LRQK_FETCH_GROUP)
    return LRQK_EINVAL;
  if (!all_aligned16({K_host, V_host, miss_tok, miss_slot, n_miss, cacheK, cacheV}))
    return LRQK_EINVAL;
  rc = check_plan_fits(plan, shape);
  if (rc != LRQK_OK) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (mode == LRQK_FETCH_DIRECT) {
    LRQK_HIP(launch_fetch_direct(*shape, K_host, V_host, miss_tok, miss_slot, n_miss, cacheK,
                                 cacheV, st));
    if (total_miss_out) *total_miss_out = -1;
    return LRQK_OK;
  }
  if (mode == LRQK_FETCH_GROUP) {
    LRQK_HIP(launch_group_fetch(*shape, K_host, V_host, miss_tok, miss_slot, n_miss, cacheK,
                                cacheV, nullptr, st));
    if (total_miss_out) *total_miss_out = -1;
    return LRQK_OK;
  }
  return staged_fetch(plan, *shape, K_host, V_host, miss_tok, miss_slot, n_miss, cacheK, cacheV,
                      st, true, total_miss_out, nullptr);
}

int lrqk_decode_step(lrqk_plan* plan, const lrqk_shape* shape, int32_t step,
                     const lrqk_layer* L, const float* q_hat, const float* q, float* out,
                     int mode_flags, const lrqk_step_debug* dbg, int64_t* total_miss_out,
                     void* stream) {
  int rc = check_shape(shape);
  if (rc != LRQK_OK) return rc;
  if (!L || step < 0 || step == INT32_MAX) return LRQK_EINVAL;
  const int mode = mode_flags & ~LRQK_SELECT_FRESH;
  if (mode != LRQK_FETCH_STAGED && mode != LRQK_FETCH_DIRECT && mode != LRQK_FETCH_GROUP)
    return LRQK_EINVAL;
  if (dbg && dbg->link_rows && !aligned16(dbg->link_rows)) return LRQK_EINVAL;
  if (L->sel_thr && !aligned16(L->sel_thr)) return LRQK_EINVAL;
  if (!all_aligned16({L->A_K, L->K_host, L->V_host, L->slot_of, L->token_of, L->last_used,
                      L->cacheK, L->cacheV, q_hat, q, out}))
    return LRQK_EINVAL;
  if (shape->w > 0 && !all_aligned16({L->liteK, L->liteV})) return LRQK_EINVAL;
  rc = check_plan_fits(plan, shape);
  if (rc != LRQK_OK) return rc;
  const lrqk_shape& s = *shape;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int BHq = s.B * s.Hq;
  LaunchTimerReset timer_reset;

  int32_t* sel_idx = (dbg && dbg->sel_idx) ? dbg->sel_idx : plan->sel_idx;
  int32_t* sel_slot = (dbg && dbg->sel_slot) ? dbg->sel_slot : plan->sel_slot;
  uint8_t* hit = (dbg && dbg->hit) ? dbg->hit : plan->hit;
  int32_t* miss_tok = (dbg && dbg->miss_tok) ? dbg->miss_tok : plan->miss_tok;
  int32_t* miss_slot = (dbg && dbg->miss_slot) ? dbg->miss_slot : plan->miss_slot;
  int32_t* n_miss = (dbg && dbg->n_miss) ? dbg->n_miss : plan->n_miss;
  if (!all_aligned16({sel_idx, sel_slot, hit, miss_tok, miss_slot, n_miss})) return LRQK_EINVAL;

  const SelectWs ws = carve_select_ws(plan->select_ws, BHq, s.k);
  if (plan->prof_ev && plan->prof_n < plan->prof_cap) plan->prof_used[plan->prof_n] = 0u;
  const bool packed = select_packed_fits(s) && proxy_filter_supported(s);
  const bool one_wg = packed || select_resolve_fits(s, true);
  const bool filtered = one_wg && proxy_filter_supported(s);
  if (filtered) {
    // candidate thresholds: carried over from the layer's previous step, or estimated from a
    // sample of this step's scores; then one pass over A_K that leaves only the candidate
    // bitmap and the candidates' scores
    const bool fresh = !packed || !L->sel_thr || (mode_flags & LRQK_SELECT_FRESH);
    if (fresh) {
      prof_arm(plan, LRQK_SLOT_SAMPLE, 2);
      LRQK_HIP(launch_proxy_threshold(s, L->A_K, q_hat, plan->samples, plan->thr, st));
    }
    prof_arm(plan, LRQK_SLOT_PROXY, 1);
    LRQK_HIP(launch_proxy_scores_filter(s, L->A_K, q_hat, plan->scores,
                                        fresh ? plan->thr : nullptr, fresh ? nullptr : L->sel_thr,
                                        plan->thr_used, plan->filter, plan->cand_scores, st));
  } else {
    prof_arm(plan, LRQK_SLOT_PROXY, 1);
    LRQK_HIP(launch_proxy_scores(s, L->A_K, q_hat, plan->scores, st));
  }
  prof_arm(plan, LRQK_SLOT_SELECT, 1);
  if (packed) {
    // selection and resolution in one launch
    LRQK_HIP(launch_select_packed(s, plan->filter, plan->cand_scores, plan->thr_used, L->A_K,
                                  q_hat, plan->scores, L->sel_thr, sel_idx, step, L->slot_of,
                                  L->token_of, L->last_used, sel_slot, hit, miss_tok, miss_slot,
                                  n_miss, st));
  } else if (one_wg) {
    LRQK_HIP(launch_select_resolve(s, plan->scores, filtered ? plan->filter : nullptr,
                                   plan->cand_scores, L->A_K, q_hat, sel_idx, step, L->slot_of,
                                   L->token_of, L->last_used, sel_slot, hit, miss_tok, miss_slot,
                                   n_miss, st));
  } else {
    // several launches; only the first is timed when profiling
    LRQK_HIP(launch_select_topk(s, plan->scores, sel_idx, ws, st));
    prof_arm(plan, LRQK_SLOT_RESOLVE, 1);
    LRQK_HIP(launch_cache_resolve(s, sel_idx, step, L->slot_of, L->token_of, L->last_used,
                                  sel_slot, hit, miss_tok, miss_slot, n_miss, st));
  }
  const AttendGeom g = attend_geometry(BHq, s.k, s.w);
  const int parts_per_head = g.nsplit + ceil_div(s.k, g.rows_per_block);

  if (mode == LRQK_FETCH_DIRECT) {
    // fetch and attention in one kernel: a row that missed is read from the pinned host store,
    // used, and written into its slot, while the other rows stream from HBM
    prof_arm(plan, LRQK_SLOT_ATTEND, 1);
    LRQK_HIP(launch_attend_partial(s, kAttendAllFetch, q, L->cacheK, L->cacheV, sel_slot, hit,
                                   nullptr, nullptr, L->liteK, L->liteV, plan->partials, g.nsplit,
                                   g.rows_per_block, parts_per_head, 0, st, L->K_host, L->V_host,
                                   sel_idx));
    prof_arm(plan, LRQK_SLOT_COMBINE, 1);
    LRQK_HIP(launch_attend_combine(s, plan->partials, parts_per_head, g.nsplit, out, st));
    prof_step_done(plan);
    if (total_miss_out) *total_miss_out = -1;
    return LRQK_OK;
  }

  if (mode == LRQK_FETCH_GROUP) {
    // the group's shared fetch in one launch with the attention over the rows that hit; then
    // the fetched rows (at most k of them per head: the launch covers the longest possible list)
    int32_t* link_rows = dbg ? dbg->link_rows : nullptr;
    if (link_rows) {
      launch_timer() = LaunchTimer{};
      LRQK_HIP(launch_fill_i32(link_rows, (size_t)s.B * s.Hkv, 0, st));
    }
    prof_arm(plan, LRQK_SLOT_ATTEND, 1);
    LRQK_HIP(launch_attend_hits_group_fetch(s, q, L->cacheK, L->cacheV, sel_slot, hit, L->liteK,
                                            L->liteV, plan->partials, g.nsplit, g.rows_per_block,
                                            parts_per_head, L->K_host, L->V_host, miss_tok,
                                            miss_slot, n_miss, link_rows, st));
    const int nblk_miss = ceil_div(s.k, g.rows_per_block);
    prof_arm(plan, LRQK_SLOT_ATTEND_MISS, 1);
    LRQK_HIP(launch_attend_partial(s, kAttendMisses, q, L->cacheK, L->cacheV, sel_slot, hit,
                                   miss_slot, n_miss, L->liteK, L->liteV, plan->partials,
                                   nblk_miss, g.rows_per_block, parts_per_head, g.nsplit, st));
    prof_arm(plan, LRQK_SLOT_COMBINE, 1);
    LRQK_HIP(launch_attend_combine(s, plan->partials, parts_per_head, g.nsplit + nblk_miss, out,
                                   st));
    prof_step_done(plan);
    if (total_miss_out) *total_miss_out = -1;
    return LRQK_OK;
  }

  // STAGED: bring the miss list to the host (the one synchronisation of the step) ...
  launch_timer() = LaunchTimer{};
  const size_t nb = (size_t)BHq;
  LRQK_HIP(hipMemcpyAsync(plan->h_nmiss, n_miss, nb * 4, hipMemcpyDeviceToHost, st));
  LRQK_HIP(hipMemcpyAsync(plan->h_miss_tok, miss_tok, nb * s.k * 4, hipMemcpyDeviceToHost, st));
  LRQK_HIP(hipMemcpyAsync(plan->h_miss_slot, miss_slot, nb * s.k * 4, hipMemcpyDeviceToHost, st));
  LRQK_HIP(hipStreamSynchronize(st));
  // ... attend the rows already resident and the lite rows while the host packs the misses
  prof_arm(plan, LRQK_SLOT_ATTEND, 1);
  LRQK_HIP(launch_attend_partial(s, kAttendHitsAndLite, q, L->cacheK, L->cacheV, sel_slot, hit,
                                 nullptr, nullptr, L->liteK, L->liteV, plan->partials, g.nsplit,
                                 g.rows_per_block, parts_per_head, 0, st));
  int max_nmiss = 0;
  prof_arm(plan, LRQK_SLOT_FETCH, 1);   // the scatter kernel on the side stream
  rc = staged_fetch(plan, s, L->K_host, L->V_host, miss_tok, miss_slot, n_miss, L->cacheK,
                    L->cacheV, st, false, total_miss_out, &max_nmiss);
  if (rc != LRQK_OK) {
    launch_timer() = LaunchTimer{};
    return rc;
  }
  const int nblk_miss = ceil_div(max_nmiss, g.rows_per_block);
  prof_arm(plan, LRQK_SLOT_ATTEND_MISS, 1);
  LRQK_HIP(launch_attend_partial(s, kAttendMisses, q, L->cacheK, L->cacheV, sel_slot, hit,
                                 miss_slot, n_miss, L->liteK, L->liteV, plan->partials, nblk_miss,
                                 g.rows_per_block, parts_per_head, g.nsplit, st));
  prof_arm(plan, LRQK_SLOT_COMBINE, 1);
  LRQK_HIP(launch_attend_combine(s, plan->partials, parts_per_head, g.nsplit + nblk_miss, out, st));
  prof_step_done(plan);
  return LRQK_OK;
}

int lrqk_plan_time_proxy_pass(lrqk_plan* plan, const lrqk_shape* shape,
                              const float* const* A_K_list, int n_list, const float* q_hat,
                              const float* sel_thr, int n_launches, float* avg_us_out,
                              void* stream) {
  int rc = check_shape(shape);
  if (rc != LRQK_OK) return rc;
  if (!A_K_list || n_list < 1 || n_launches < 1 || !avg_us_out || !all_aligned16({q_hat}))
    return LRQK_EINVAL;
  if (sel_thr && !aligned16(sel_thr)) return LRQK_EINVAL;
  for (int i = 0; i < n_list; ++i)
    if (!all_aligned16({A_K_list[i]})) return LRQK_EINVAL;
  rc = check_plan_fits(plan, shape);
  if (rc != LRQK_OK) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  LaunchTimerReset timer_reset;
  // the same choices as lrqk_decode_step makes for this shape
  const bool packed = select_packed_fits(*shape) && proxy_filter_supported(*shape);
  const bool filtered =
      (packed || select_resolve_fits(*shape, true)) && proxy_filter_supported(*shape);
  if (!packed) sel_thr = nullptr;  // thresholds are carried only into the packed selection
  auto pass = [&](const float* A_K) -> hipError_t {
    if (filtered)
      return launch_proxy_scores_filter(*shape, A_K, q_hat, plan->scores,
                                        sel_thr ? nullptr : plan->thr, sel_thr, plan->thr_used,
                                        plan->filter, plan->cand_scores, st);
    return launch_proxy_scores(*shape, A_K, q_hat, plan->scores, st);
  };
  // thresholds for this q_hat, then a few untimed launches
  if (filtered && !sel_thr)
    LRQK_HIP(launch_proxy_threshold(*shape, A_K_list[0], q_hat, plan->samples, plan->thr, st));
  for (int i = 0; i < (n_list < 4 ? n_list : 4); ++i) LRQK_HIP(pass(A_K_list[i]));
  hipEvent_t e0 = nullptr, e1 = nullptr;
  LRQK_HIP(hipEventCreate(&e0));
  hipError_t e = hipEventCreate(&e1);
  if (e != hipSuccess) {
    (void)hipEventDestroy(e0);
    LRQK_HIP(e);
  }
  if (e == hipSuccess) e = hipEventRecord(e0, st);
  for (int i = 0; i < n_launches && e == hipSuccess; ++i) e = pass(A_K_list[i % n_list]);
  if (e == hipSuccess) e = hipEventRecord(e1, st);
  if (e == hipSuccess) e = hipEventSynchronize(e1);
  float ms = 0.f;
  if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
  (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  LRQK_HIP(e);
  const float bracketed_us = 1e3f * ms / (float)n_launches;
  *avg_us_out = bracketed_us;
  if (!filtered) return LRQK_OK;
  // The bracketed average includes the gap between consecutive launches.  A second series
  // attaches a pair of events to every kernel, which then hold that kernel's own start and
  // end; their average is reported if it is plausible (positive, not above the bracketed one).
  const int n2 = n_launches < 64 ? n_launches : 64;
  hipEvent_t ev[128] = {};
  e = hipSuccess;
  for (int i = 0; i < 2 * n2 && e == hipSuccess; ++i) e = hipEventCreate(&ev[i]);
  for (int i = 0; i < n2 && e == hipSuccess; ++i) {
    LaunchTimer& lt = launch_timer();
    lt = LaunchTimer{};
    lt.ev = &ev[2 * i];
    lt.pairs_left = 1;
    e = pass(A_K_list[i % n_list]);
  }
  launch_timer() = LaunchTimer{};
  if (e == hipSuccess) e = hipStreamSynchronize(st);
  double sum_us = 0.0;
  for (int i = 0; i < n2 && e == hipSuccess; ++i) {
    float k_ms = 0.f;
    e = hipEventElapsedTime(&k_ms, ev[2 * i], ev[2 * i + 1]);
    sum_us += 1e3 * k_ms;
  }
  for (int i = 0; i < 2 * n2; ++i)
    if (ev[i]) (void)hipEventDestroy(ev[i]);
  if (e != hipSuccess) {
    (void)hipGetLastError();  // the bracketed figure stands
    return LRQK_OK;
  }
  const float per_kernel_us = (float)(sum_us / n2);
  if (per_kernel_us > 0.f && per_kernel_us <= bracketed_us) *avg_us_out = per_kernel_us;
  return LRQK_OK;
}

int lrqk_plan_profile(lrqk_plan* plan, int n_steps) {
  if (!plan || n_steps < 0 || n_steps > 65536) return LRQK_EINVAL;
  prof_free(plan);
  if (n_steps == 0) return LRQK_OK;
  const size_t n = (size_t)n_steps * LRQK_PROFILE_SLOTS * 2;
  plan->prof_ev = static_cast<hipEvent_t*>(std::calloc(n, sizeof(hipEvent_t)));
  plan->prof_used = static_cast<unsigned*>(std::calloc((size_t)n_steps, sizeof(unsigned)));
  if (!plan->prof_ev || !plan->prof_used) {
    prof_free(plan);
    return LRQK_ENOMEM;
  }
  plan->prof_cap = n_steps;
  for (size_t i = 0; i < n; ++i) {
    const hipError_t e = hipEventCreate(&plan->prof_ev[i]);
    if (e != hipSuccess) {
      prof_free(plan);
      return record_hip_error(e);
    }
  }
  return LRQK_OK;
}

int lrqk_plan_profile_read(lrqk_plan* plan, double* ms_sum, int* n_steps_out) {
  if (!plan || !ms_sum || !n_steps_out) return LRQK_EINVAL;
  for (int m = 0; m < LRQK_PROFILE_SLOTS; ++m) ms_sum[m] = 0.0;
  *n_steps_out = plan->prof_n;
  for (int i = 0; i < plan->prof_n; ++i) {
    hipEvent_t* ev = plan->prof_ev + (size_t)i * LRQK_PROFILE_SLOTS * 2;
    for (int m = 0; m < LRQK_PROFILE_SLOTS; ++m) {
      if (!(plan->prof_used[i] & (1u << m))) continue;
      LRQK_HIP(hipEventSynchronize(ev[2 * m + 1]));
      float ms = 0.f;
      LRQK_HIP(hipEventElapsedTime(&ms, ev[2 * m], ev[2 * m + 1]));
      ms_sum[m] += ms;
    }
  }
  plan->prof_n = 0;
  return LRQK_OK;
}

#pragma GCC visibility pop
}  // extern "C"
