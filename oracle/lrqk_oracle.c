/*
 * lrqk_oracle.c — plain CPU reference of the LRQK decode step.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the yardstick the HIP library is
 * compared against; it is used by tests/, by the smoke check and by the
 * benchmark's cpu_baseline leg, and by nothing else.  It shares no code,
 * header, table or helper with the HIP path.
 *
 * Everything is written as the definition reads: straight loops, double
 * accumulation, no blocking, no fusion.  The only parallelism is an OpenMP
 * loop over independent (batch, head) units, which the paper states are
 * independent (Sec. 4, preliminaries).
 *
 * Steps and where they come from
 *   oracle_proxy_scores   Alg. 2, "compute proxy attention": s = A_K q_hat^T
 *   oracle_select_topk    Alg. 2, top(s, k); Sec. 4.1 active tokens Omega_k and
 *                         lite tokens Omega_l (the last w positions)
 *   oracle_cache_resolve  Sec. 4.1 hit-and-miss cache; Sec. 5.3 miss count
 *   oracle_fetch          Alg. 2, "Fetch missing" and "merge"
 *   oracle_sparse_attend  Sec. 4.3, Attention(q_t, K_Omega, V_Omega)
 *   oracle_attend_store   the same attention with rows read from the full
 *                         K/V store instead of through the cache
 *
 * Readings of points the paper leaves open (each also listed in the design notes)
 *   - GQA: A_K, K, V per KV head; scores, selection, cache per query head;
 *     query head h reads KV head h / G.
 *   - top-k ranks positions [0, l-w) only; the lite window [l-w, l) is always
 *     attended; the two sets are disjoint, |Omega| = k + w.
 *   - scores are raw dot products (no scaling, no softmax) before top-k.
 *   - equal scores: lower position wins.
 *   - the cache has C >= k slots; replacement is least-recently-selected,
 *     ties by lower slot, misses assigned in ascending position order.
 *   - softmax scale is a parameter (1/sqrt(d) in all workloads).
 *
 * Pins: see tests/test_oracle_pins.py (dense attention when k + w = l, numpy
 * sort for top-k, closed forms for attention, cache invariants).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* bf16 is the upper half of an IEEE binary32. */
static double bf16_to_double(uint16_t h) {
  uint32_t u = ((uint32_t)h) << 16;
  float f;
  memcpy(&f, &u, sizeof f);
  return (double)f;
}

/* element j of a K/V row stored as bf16 (kv_dtype 0) or fp32 (kv_dtype 1) */
static double kv_elem(const void* row, int kv_dtype, int j) {
  if (kv_dtype == 0) return bf16_to_double(((const uint16_t*)row)[j]);
  return (double)((const float*)row)[j];
}

static size_t kv_bytes(int kv_dtype) { return kv_dtype == 0 ? 2 : 4; }

/*
 * s[b,h,i] = sum_j A_K[b,h/G,i,j] * q_hat[b,h,j].
 * s64: products and sums in double (each fp32*fp32 product is exact in double).
 * s32: the same sum as a single-precision fused-multiply-add chain, j ascending,
 *      starting from 0.0f — the arithmetic a GPU kernel can reproduce exactly.
 * Either output may be NULL.
 */
void oracle_proxy_scores(int B, int Hq, int Hkv, int l, int r, const float* A_K,
                         const float* q_hat, double* s64, float* s32) {
  const int G = Hq / Hkv;
#pragma omp parallel for schedule(static)
  for (int bh = 0; bh < B * Hq; ++bh) {
    const int b = bh / Hq, h = bh % Hq, kv = h / G;
    const float* A = A_K + ((size_t)b * Hkv + kv) * (size_t)l * r;
    const float* qh = q_hat + (size_t)bh * r;
    for (int i = 0; i < l; ++i) {
      double acc = 0.0;
      float accf = 0.0f;
      for (int j = 0; j < r; ++j) {
        acc += (double)A[(size_t)i * r + j] * (double)qh[j];
        accf = fmaf(A[(size_t)i * r + j], qh[j], accf);
      }
      if (s64) s64[(size_t)bh * l + i] = acc;
      if (s32) s32[(size_t)bh * l + i] = accf;
    }
  }
}

typedef struct {
  double s;
  int32_t i;
} scored;

/* larger score first; equal scores: lower position first */
static int by_score_then_pos(const void* pa, const void* pb) {
  const scored* a = (const scored*)pa;
  const scored* b = (const scored*)pb;
  if (a->s > b->s) return -1;
  if (a->s < b->s) return 1;
  return (a->i > b->i) - (a->i < b->i);
}

static int by_int(const void* pa, const void* pb) {
  const int32_t a = *(const int32_t*)pa, b = *(const int32_t*)pb;
  return (a > b) - (a < b);
}

/*
 * Omega_k of every head: sort positions [0, l-w) by (score descending,
 * position ascending), keep the first k, list them in ascending position.
 * scores: double [n_heads, l].  sel_idx: int32 [n_heads, k].
 */
void oracle_select_topk(int n_heads, int l, int w, int k, const double* scores,
                        int32_t* sel_idx) {
  const int n = l - w;
#pragma omp parallel for schedule(dynamic, 1)
  for (int bh = 0; bh < n_heads; ++bh) {
    scored* v = (scored*)malloc((size_t)(n > 0 ? n : 1) * sizeof(scored));
    for (int i = 0; i < n; ++i) {
      v[i].s = scores[(size_t)bh * l + i];
      v[i].i = i;
    }
    qsort(v, (size_t)n, sizeof(scored), by_score_then_pos);
    int32_t* out = sel_idx + (size_t)bh * k;
    for (int j = 0; j < k; ++j) out[j] = v[j].i;
    qsort(out, (size_t)k, sizeof(int32_t), by_int);
    free(v);
  }
}

typedef struct {
  int32_t lu;
  int32_t slot;
} victim;

static int by_age_then_slot(const void* pa, const void* pb) {
  const victim* a = (const victim*)pa;
  const victim* b = (const victim*)pb;
  if (a->lu != b->lu) return (a->lu > b->lu) - (a->lu < b->lu);
  return (a->slot > b->slot) - (a->slot < b->slot);
}

/*
 * Hit/miss resolution with least-recently-selected replacement.
 * Per head: walk Omega_k in ascending position; a resident token is a hit and
 * refreshes its slot; the others are misses.  Then list the slots not used in
 * this step by (last_used, slot) and hand the j-th of them to the j-th miss.
 * Returns 0, or -1 if some head ran out of victims or saw a position outside
 * [0, l) (inputs that break the contract).
 */
int oracle_cache_resolve(int n_heads, int l, int C, int k, const int32_t* sel_idx, int32_t step,
                         int32_t* slot_of, int32_t* token_of, int32_t* last_used,
                         int32_t* sel_slot, uint8_t* hit, int32_t* miss_tok,
                         int32_t* miss_slot, int32_t* n_miss) {
  int bad = 0;
#pragma omp parallel for schedule(dynamic, 1) reduction(| : bad)
  for (int bh = 0; bh < n_heads; ++bh) {
    const int32_t* sel = sel_idx + (size_t)bh * k;
    int32_t* so = slot_of + (size_t)bh * l;
    int32_t* to = token_of + (size_t)bh * C;
    int32_t* lu = last_used + (size_t)bh * C;
    int32_t* ss = sel_slot + (size_t)bh * k;
    uint8_t* ht = hit + (size_t)bh * k;
    int32_t* mt = miss_tok + (size_t)bh * k;
    int32_t* ms = miss_slot + (size_t)bh * k;
    int nm = 0, head_bad = 0;
    int* miss_pos = (int*)malloc((size_t)k * sizeof(int));
    for (int j = 0; j < k; ++j) {
      const int32_t tok = sel[j];
      if (tok < 0 || tok >= l) {
        head_bad = 1;
        ss[j] = -1;
        ht[j] = 0;
        continue;
      }
      if (so[tok] >= 0) {
        ss[j] = so[tok];
        ht[j] = 1;
        lu[so[tok]] = step;
      } else {
        ht[j] = 0;
        mt[nm] = tok;
        miss_pos[nm] = j;
        ++nm;
      }
    }
    victim* vs = (victim*)malloc((size_t)C * sizeof(victim));
    int nv = 0;
    for (int s = 0; s < C; ++s)
      if (lu[s] != step) {
        vs[nv].lu = lu[s];
        vs[nv].slot = s;
        ++nv;
      }
    qsort(vs, (size_t)nv, sizeof(victim), by_age_then_slot);
    for (int j = 0; j < nm; ++j) {
      if (j >= nv) {
        head_bad = 1;
        ss[miss_pos[j]] = -1;
        ms[j] = -1;
        continue;
      }
      const int32_t s = vs[j].slot;
      const int32_t old = to[s];
      if (old >= 0) so[old] = -1;
      to[s] = mt[j];
      so[mt[j]] = s;
      lu[s] = step;
      ms[j] = s;
      ss[miss_pos[j]] = s;
    }
    n_miss[bh] = head_bad ? -1 : nm;
    bad |= head_bad;
    free(vs);
    free(miss_pos);
  }
  return bad ? -1 : 0;
}

/*
 * cache[b,h,miss_slot[j],:] <- store[b,h/G,miss_tok[j],:] for j < n_miss[b,h]; a bit copy.
 */
void oracle_fetch(int B, int Hq, int Hkv, int l, int C, int d, int k, int kv_dtype,
                  const void* K_store, const void* V_store, const int32_t* miss_tok,
                  const int32_t* miss_slot, const int32_t* n_miss, void* cacheK, void* cacheV) {
  const int G = Hq / Hkv;
  const size_t row = (size_t)d * kv_bytes(kv_dtype);
  for (int bh = 0; bh < B * Hq; ++bh) {
    const int b = bh / Hq, h = bh % Hq, kv = h / G;
    const char* Ks = (const char*)K_store + ((size_t)b * Hkv + kv) * (size_t)l * row;
    const char* Vs = (const char*)V_store + ((size_t)b * Hkv + kv) * (size_t)l * row;
    char* Kc = (char*)cacheK + (size_t)bh * C * row;
    char* Vc = (char*)cacheV + (size_t)bh * C * row;
    for (int j = 0; j < n_miss[bh]; ++j) {
      const int32_t tok = miss_tok[(size_t)bh * k + j], s = miss_slot[(size_t)bh * k + j];
      if (s < 0) continue;
      memcpy(Kc + (size_t)s * row, Ks + (size_t)tok * row, row);
      memcpy(Vc + (size_t)s * row, Vs + (size_t)tok * row, row);
    }
  }
}

/*
 * Softmax attention of one query over n rows given by pointers.
 *   logit_i = scale * (q . K_i);  p_i = exp(logit_i - max);  out = sum p_i V_i / sum p_i
 * all in double.
 */
static void attend_rows(int d, int kv_dtype, double scale, const float* q, int n,
                        const void* const* Krows, const void* const* Vrows, double* out) {
  double* logit = (double*)malloc((size_t)(n > 0 ? n : 1) * sizeof(double));
  double mx = -INFINITY;
  for (int i = 0; i < n; ++i) {
    double acc = 0.0;
    for (int j = 0; j < d; ++j) acc += (double)q[j] * kv_elem(Krows[i], kv_dtype, j);
    logit[i] = scale * acc;
    if (logit[i] > mx) mx = logit[i];
  }
  double denom = 0.0;
  for (int j = 0; j < d; ++j) out[j] = 0.0;
  for (int i = 0; i < n; ++i) {
    const double p = exp(logit[i] - mx);
    denom += p;
    for (int j = 0; j < d; ++j) out[j] += p * kv_elem(Vrows[i], kv_dtype, j);
  }
  for (int j = 0; j < d; ++j) out[j] = n > 0 ? out[j] / denom : 0.0;
  free(logit);
}

/*
 * Attention over Omega = {cache rows sel_slot[b,h,0..k)} U {lite rows 0..w)}.
 * Rows with sel_slot outside [0, C) are left out.  out: double [B,Hq,d].
 */
void oracle_sparse_attend(int B, int Hq, int Hkv, int C, int d, int k, int w, int kv_dtype,
                          double scale, const float* q, const void* cacheK, const void* cacheV,
                          const int32_t* sel_slot, const void* liteK, const void* liteV,
                          double* out) {
  const int G = Hq / Hkv;
  const size_t row = (size_t)d * kv_bytes(kv_dtype);
#pragma omp parallel for schedule(static)
  for (int bh = 0; bh < B * Hq; ++bh) {
    const int b = bh / Hq, h = bh % Hq, kv = h / G;
    const void** Kr = (const void**)malloc((size_t)(k + w + 1) * sizeof(void*));
    const void** Vr = (const void**)malloc((size_t)(k + w + 1) * sizeof(void*));
    int n = 0;
    for (int j = 0; j < k; ++j) {
      const int32_t s = sel_slot[(size_t)bh * k + j];
      if (s < 0 || s >= C) continue;
      Kr[n] = (const char*)cacheK + ((size_t)bh * C + s) * row;
      Vr[n] = (const char*)cacheV + ((size_t)bh * C + s) * row;
      ++n;
    }
    for (int j = 0; j < w; ++j) {
      Kr[n] = (const char*)liteK + (((size_t)b * Hkv + kv) * w + j) * row;
      Vr[n] = (const char*)liteV + (((size_t)b * Hkv + kv) * w + j) * row;
      ++n;
    }
    attend_rows(d, kv_dtype, scale, q + (size_t)bh * d, n, Kr, Vr, out + (size_t)bh * d);
    free(Kr);
    free(Vr);
  }
}

/*
 * The same attention with rows taken straight from the full store:
 * Omega = sel_idx[b,h,0..k) U [l-w, l).  Used to check that the cache is
 * transparent (reading through it changes nothing).
 */
void oracle_attend_store(int B, int Hq, int Hkv, int l, int d, int k, int w, int kv_dtype,
                         double scale, const float* q, const void* K_store, const void* V_store,
                         const int32_t* sel_idx, double* out) {
  const int G = Hq / Hkv;
  const size_t row = (size_t)d * kv_bytes(kv_dtype);
#pragma omp parallel for schedule(static)
  for (int bh = 0; bh < B * Hq; ++bh) {
    const int b = bh / Hq, h = bh % Hq, kv = h / G;
    const char* Ks = (const char*)K_store + ((size_t)b * Hkv + kv) * (size_t)l * row;
    const char* Vs = (const char*)V_store + ((size_t)b * Hkv + kv) * (size_t)l * row;
    const void** Kr = (const void**)malloc((size_t)(k + w + 1) * sizeof(void*));
    const void** Vr = (const void**)malloc((size_t)(k + w + 1) * sizeof(void*));
    int n = 0;
    for (int j = 0; j < k; ++j) {
      const int32_t t = sel_idx[(size_t)bh * k + j];
      Kr[n] = Ks + (size_t)t * row;
      Vr[n] = Vs + (size_t)t * row;
      ++n;
    }
    for (int t = l - w; t < l; ++t) {
      Kr[n] = Ks + (size_t)t * row;
      Vr[n] = Vs + (size_t)t * row;
      ++n;
    }
    attend_rows(d, kv_dtype, scale, q + (size_t)bh * d, n, Kr, Vr, out + (size_t)bh * d);
    free(Kr);
    free(Vr);
  }
}
