/*
 * CPU oracle for the MoE decode step with an offloaded-expert cache.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the
 * HIP path is checked against; it shares no code with that path and the
 * product never calls it.  Only tests, the smoke check and the benchmark's
 * CPU-baseline leg may load it.
 *
 * What it follows (paper section 2, "Problem Setup and Motivation"):
 *   Eq. 1   p = softmax(W_r x),  r = Top-K(p)
 *   Eq. 2   y = sum over selected i of  p_i * E_i(x)
 *   Eq. 3   E_i(x) = W_d ( phi(W_g x) (.) W_u x ),  phi = SiLU
 * and the offloading runtime of the "Expert Offloading Systems" paragraph and
 * section 3.2: a per-layer cache of C resident experts, fetch on demand on a
 * miss, eviction by the cache policy.  Policies are members of the
 * gamma-discounted family of Definition C.1 (appendix C.1): LRU is its
 * gamma -> 0+ limit, LFU its gamma = 1 case (Remark after Definition C.1).
 *
 * All inputs are float32 arrays (bf16 data is widened exactly beforehand);
 * every sum is accumulated in double, in index order.  No blocking, no
 * fusion, no reordering.
 *
 * Pins (tests/test_oracle_*.py): closed forms (identity weights, zero gate),
 * softmax invariants, brute-force top-K, dense-masked vs sparse evaluation,
 * a second LRU formulation (move-to-front list), Definition C.1 evaluated
 * literally with gamma < 1/2, Mattson inclusion, counting identities, a
 * library matmul cross-check, and the paper's 5-6 ms transfer figure for the
 * byte model.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static int g_threads = 1;

void orc_set_threads(int n) { g_threads = n < 1 ? 1 : n; }
int orc_get_threads(void) { return g_threads; }

/* ---- Eq. 1, first half: logits[b,e] = sum_j W_r[e,j] x[b,j] (+ bias[b,e]) ---- */
void orc_router_logits(const float* x, const float* w_r, const float* bias,
                       int B, int E, int d, double* logits) {
  for (int b = 0; b < B; ++b)
    for (int e = 0; e < E; ++e) {
      double s = 0.0;
      for (int j = 0; j < d; ++j) s += (double)w_r[(size_t)e * d + j] * (double)x[(size_t)b * d + j];
      if (bias) s += (double)bias[(size_t)b * E + e];
      logits[(size_t)b * E + e] = s;
    }
}

/* ---- Eq. 1: softmax over all E experts (max subtracted) ---- */
void orc_softmax(const double* logits, int B, int E, double* p) {
  for (int b = 0; b < B; ++b) {
    const double* z = logits + (size_t)b * E;
    double m = z[0];
    for (int e = 1; e < E; ++e) if (z[e] > m) m = z[e];
    double s = 0.0;
    for (int e = 0; e < E; ++e) { p[(size_t)b * E + e] = exp(z[e] - m); s += p[(size_t)b * E + e]; }
    for (int e = 0; e < E; ++e) p[(size_t)b * E + e] /= s;
  }
}

/* ---- Eq. 1: Top-K.  The K largest scores; equal scores go to the lower id.
 * idx[b,:] is returned in ascending expert id; ||r||_1 = K. ---- */
void orc_topk(const double* scores, int B, int E, int K, int32_t* idx) {
  char* taken = (char*)malloc((size_t)E);
  for (int b = 0; b < B; ++b) {
    const double* z = scores + (size_t)b * E;
    memset(taken, 0, (size_t)E);
    for (int k = 0; k < K; ++k) {
      int best = -1;
      for (int e = 0; e < E; ++e)
        if (!taken[e] && (best < 0 || z[e] > z[best])) best = e;
      taken[best] = 1;
    }
    int n = 0;
    for (int e = 0; e < E; ++e) if (taken[e]) idx[(size_t)b * K + n++] = e;
  }
  free(taken);
}

/* ---- gate weights for Eq. 2: literal p_i, or p_i renormalised over the K selected ---- */
void orc_gate_weights(const double* p, const int32_t* idx, int B, int E, int K,
                      int norm_topk, double* w) {
  for (int b = 0; b < B; ++b) {
    double s = 0.0;
    for (int k = 0; k < K; ++k) s += p[(size_t)b * E + idx[(size_t)b * K + k]];
    for (int k = 0; k < K; ++k) {
      double v = p[(size_t)b * E + idx[(size_t)b * K + k]];
      w[(size_t)b * K + k] = norm_topk ? v / s : v;
    }
  }
}

/* ---- Eq. 3: one expert on one token.  W_g, W_u are [f,d]; W_d is [d,f]. ---- */
void orc_expert_swiglu(const float* x, const float* w_g, const float* w_u, const float* w_d,
                       int d, int f, double* out) {
  double* h = (double*)malloc((size_t)f * sizeof(double));
#pragma omp parallel for num_threads(g_threads) schedule(static)
  for (int j = 0; j < f; ++j) {
    double g = 0.0, u = 0.0;
    for (int i = 0; i < d; ++i) {
      g += (double)w_g[(size_t)j * d + i] * (double)x[i];
      u += (double)w_u[(size_t)j * d + i] * (double)x[i];
    }
    double silu = g / (1.0 + exp(-g));
    h[j] = silu * u;
  }
#pragma omp parallel for num_threads(g_threads) schedule(static)
  for (int i = 0; i < d; ++i) {
    double s = 0.0;
    for (int j = 0; j < f; ++j) s += (double)w_d[(size_t)i * f + j] * h[j];
    out[i] = s;
  }
  free(h);
}

/* ---- expert cache ------------------------------------------------------
 * One cache per layer, C slots.  A lookup of expert e:
 *   resident  -> hit, its recency/count is refreshed;
 *   otherwise -> miss: the lowest-index empty slot if one exists, else the
 *                victim chosen by the policy is evicted; e is inserted.
 * Lazy update (Remark after Definition C.1): contents change only by
 * inserting the requested expert.
 *
 * policy 0 (LRU): victim = resident expert with the smallest last-use tick
 *                 (ticks are unique, so the victim is unique).
 * policy 1 (gamma-discounted count, Definition C.1): every expert carries
 *   score_{t+1} = gamma * score_t + r_t, advanced once per token by
 *   orc_cache_end_token(); victim = resident expert, not requested by the
 *   current token, with the smallest score, ties to the older last-use tick.
 *   gamma = 1 is LFU.  Each pinned expert counts as a token of its own.
 */
typedef struct {
  int E, C, policy;
  double gamma;
  int32_t* expert_in;   /* [C], -1 = empty */
  int64_t* tick;        /* [C] last-use tick of the slot's expert */
  int32_t* slot_of;     /* [E], -1 = not resident */
  double* score;        /* [E] discounted request count (policy 1) */
  double* pending;      /* [E] requests of the current token (policy 1) */
  int64_t clock;
  uint64_t lookups, hits, misses, evictions, pin_loads;
} orc_cache_t;

void orc_cache_reset(orc_cache_t* c, int clear_stats) {
  for (int s = 0; s < c->C; ++s) { c->expert_in[s] = -1; c->tick[s] = 0; }
  for (int e = 0; e < c->E; ++e) { c->slot_of[e] = -1; c->score[e] = 0.0; c->pending[e] = 0.0; }
  c->clock = 0;
  if (clear_stats) c->lookups = c->hits = c->misses = c->evictions = c->pin_loads = 0;
}

orc_cache_t* orc_cache_new(int E, int C, int policy, double gamma) {
  orc_cache_t* c = (orc_cache_t*)calloc(1, sizeof(orc_cache_t));
  c->E = E; c->C = C; c->policy = policy; c->gamma = gamma;
  c->expert_in = (int32_t*)malloc((size_t)C * sizeof(int32_t));
  c->tick = (int64_t*)malloc((size_t)C * sizeof(int64_t));
  c->slot_of = (int32_t*)malloc((size_t)E * sizeof(int32_t));
  c->score = (double*)malloc((size_t)E * sizeof(double));
  c->pending = (double*)malloc((size_t)E * sizeof(double));
  orc_cache_reset(c, 1);
  return c;
}

void orc_cache_free(orc_cache_t* c) {
  if (!c) return;
  free(c->expert_in); free(c->tick); free(c->slot_of); free(c->score); free(c->pending); free(c);
}

static int victim_slot(const orc_cache_t* c) {
  if (c->policy == 0) {
    int v = 0;
    for (int s = 1; s < c->C; ++s)
      if (c->tick[s] < c->tick[v]) v = s;
    return v;
  }
  /* policy 1: experts already requested by the current token are needed for
   * its computation and are never victims (C >= K leaves a candidate). */
  int v = -1;
  for (int s = 0; s < c->C; ++s) {
    if (c->pending[c->expert_in[s]] > 0.0) continue;
    if (v < 0) { v = s; continue; }
    double a = c->score[c->expert_in[s]], b = c->score[c->expert_in[v]];
    if (a < b || (a == b && c->tick[s] < c->tick[v])) v = s;
  }
  return v;
}

/* Definition C.1, count update: applied once after all K requests of a token. */
void orc_cache_end_token(orc_cache_t* c) {
  if (c->policy == 0) return;
  for (int e = 0; e < c->E; ++e) { c->score[e] = c->gamma * c->score[e] + c->pending[e]; c->pending[e] = 0.0; }
}

/* returns 1 on hit, 0 on miss; *evicted = expert evicted, or -1 */
static int touch(orc_cache_t* c, int e, int32_t* evicted) {
  *evicted = -1;
  c->clock += 1;
  c->pending[e] += 1.0;
  int s = c->slot_of[e];
  if (s >= 0) { c->tick[s] = c->clock; return 1; }
  s = -1;
  for (int i = 0; i < c->C; ++i) if (c->expert_in[i] < 0) { s = i; break; }
  if (s < 0) {
    s = victim_slot(c);
    *evicted = c->expert_in[s];
    c->slot_of[*evicted] = -1;
  }
  c->expert_in[s] = e; c->slot_of[e] = s; c->tick[s] = c->clock;
  return 0;
}

int orc_cache_lookup(orc_cache_t* c, int e, int32_t* evicted) {
  int hit = touch(c, e, evicted);
  c->lookups += 1;
  if (hit) c->hits += 1; else { c->misses += 1; if (*evicted >= 0) c->evictions += 1; }
  return hit;
}

/* Prefetch before generation (section 3.2): the listed experts are looked up
 * in list order; loads count as pin_loads, not as hits or misses. */
void orc_cache_pin(orc_cache_t* c, const int32_t* ids, int n) {
  for (int i = 0; i < n; ++i) {
    int32_t ev;
    int hit = touch(c, ids[i], &ev);
    if (!hit) { c->pin_loads += 1; if (ev >= 0) c->evictions += 1; }
    orc_cache_end_token(c);
  }
}

int orc_cache_resident(const orc_cache_t* c, int32_t* out) {
  int n = 0;
  for (int e = 0; e < c->E; ++e) if (c->slot_of[e] >= 0) out[n++] = e;
  return n;
}

void orc_cache_stats(const orc_cache_t* c, uint64_t* out6, uint64_t expert_bytes) {
  out6[0] = c->lookups; out6[1] = c->hits; out6[2] = c->misses; out6[3] = c->evictions;
  out6[4] = c->pin_loads; out6[5] = (c->misses + c->pin_loads) * expert_bytes;
}

/* ---- cache-simulation loss (section 3.1.1; appendix C.1, Proposition C.2) ----------------
 * Forward value of L_cs and of the hard miss count L_cs^hard for ONE layer over a routing trace
 * idx[T][K] (the request vectors r^(t), ||r||_1 = K).
 *
 * Soft cache (Proposition C.2): Gamma^(1) = 1,
 *     c^(t+1) = (gamma Gamma^(t) c^(t) + r^(t)) / Gamma^(t+1),   Gamma^(t+1) = gamma Gamma^(t) + K/C,
 * started from c1[E] with ||c1||_1 = C (uniform C/E when c1 is NULL: the initialisation that skips the
 * fill phase).  soft = sum_t <r^(t), 1 - c^(t)>.
 *
 * Hard cache (Definition C.1): Ctilde^(t+1) = gamma Ctilde^(t) + r^(t), Chat = Top-C(Ctilde) with ties to
 * the lower id, started from Ctilde^(1) = c1.  hard = sum_t <r^(t), 1 - Chat^(t)>.
 * The caller divides by L*T.
 */
void orc_cache_sim_loss(const int32_t* idx, int T, int K, int E, int C, double gamma, const double* c1,
                        double* soft_out, double* hard_out) {
  double* c = (double*)malloc((size_t)E * sizeof(double));
  double* ct = (double*)malloc((size_t)E * sizeof(double));
  char* in_top = (char*)malloc((size_t)E);
  for (int e = 0; e < E; ++e) { c[e] = c1 ? c1[e] : (double)C / (double)E; ct[e] = c[e]; }
  double Gamma = 1.0, soft = 0.0, hard = 0.0;
  for (int t = 0; t < T; ++t) {
    const int32_t* r = idx + (size_t)t * K;
    /* Top-C of the discounted counts */
    memset(in_top, 0, (size_t)E);
    for (int j = 0; j < C && j < E; ++j) {
      int best = -1;
      for (int e = 0; e < E; ++e)
        if (!in_top[e] && (best < 0 || ct[e] > ct[best])) best = e;
      in_top[best] = 1;
    }
    for (int k = 0; k < K; ++k) {
      soft += 1.0 - c[r[k]];
      hard += in_top[r[k]] ? 0.0 : 1.0;
    }
    const double Gamma_next = gamma * Gamma + (double)K / (double)C;
    for (int e = 0; e < E; ++e) { c[e] = gamma * Gamma * c[e]; ct[e] = gamma * ct[e]; }
    for (int k = 0; k < K; ++k) { c[r[k]] += 1.0; ct[r[k]] += 1.0; }
    for (int e = 0; e < E; ++e) c[e] = c[e] / Gamma_next;
    Gamma = Gamma_next;
  }
  *soft_out = soft;
  *hard_out = hard;
  free(c); free(ct); free(in_top);
}
