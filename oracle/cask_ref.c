/*
 * CASK compression-event ORACLE (test infrastructure; see cask_ref.h).
 *
 * Plain C, double precision, one loop nest per definition.  OpenMP is used only
 * across independent (sequence, layer, KV head) units.
 */
#define _GNU_SOURCE
#include "cask_ref.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------ element access */

double cask_ref_bf16_to_double(uint16_t h) {
  uint32_t bits = ((uint32_t)h) << 16;
  float f;
  memcpy(&f, &bits, 4);
  return (double)f;
}

/* Nearest bf16 (8 significant bits, exponent range of float), ties to even.  The value
 * is rounded directly from double on the bf16 grid, so there is no double rounding. */
uint16_t cask_ref_bf16_from_double(double x) {
  if (isnan(x)) return 0x7FC0;
  if (isinf(x)) return x > 0 ? 0x7F80 : 0xFF80;
  if (x == 0.0) return signbit(x) ? 0x8000 : 0x0000;
  int e;
  (void)frexp(x, &e);             /* |x| = m * 2^e, m in [0.5, 1) */
  int q = e - 8;                  /* spacing of bf16 numbers near x is 2^(e-8) */
  if (q < -133) q = -133;         /* subnormal spacing */
  double r = ldexp(nearbyint(ldexp(x, -q)), q); /* nearbyint: round-half-even (default mode) */
  if (fabs(r) >= ldexp(1.0, 128)) return r > 0 ? 0x7F80 : 0xFF80;
  float f = (float)r;             /* exact: r is on the bf16 grid */
  uint32_t bits;
  memcpy(&bits, &f, 4);
  return (uint16_t)(bits >> 16);
}

static size_t elem_size(int dtype) { return dtype == CASK_REF_BF16 ? 2 : 4; }

static double load_elem(const void* base, int dtype, int64_t idx) {
  if (dtype == CASK_REF_BF16) return cask_ref_bf16_to_double(((const uint16_t*)base)[idx]);
  return (double)((const float*)base)[idx];
}

static void store_elem(void* base, int dtype, int64_t idx, double x) {
  if (dtype == CASK_REF_BF16)
    ((uint16_t*)base)[idx] = cask_ref_bf16_from_double(x);
  else
    ((float*)base)[idx] = (float)x;
}

/* ------------------------------------------------------------------ parameter checks */

static int resolved_recent(const cask_ref_params* p) { return p->recent < 0 ? p->window : p->recent; }

static int check_shape(const cask_ref_params* p) {
  if (!p) return -1;
  if (p->dtype != CASK_REF_F32 && p->dtype != CASK_REF_BF16) return -1;
  if (p->head_dim < 1 || p->q_per_kv < 1 || p->window < 1) return -1;
  return 0;
}

static int check_params(const cask_ref_params* p) {
  if (check_shape(p)) return -1;
  if (p->budget < resolved_recent(p) + 1) return -1;
  if (p->merge_radius < 0 || p->merge_geometry < 0 || p->merge_geometry > 1) return -1;
  if (p->seed_dedup < 0 || (p->seed_dedup > 0 && p->merge_geometry != 0)) return -1;
  if (p->merge_geometry == 1) {
    if (!p->band_weight || !(p->dist_threshold >= 0.0f)) return -1;
    for (int f = 0; f < p->head_dim / 2; ++f)
      if (!(p->band_weight[f] >= 0.0f)) return -1;
  }
  return 0;
}

static int check_unit(const cask_ref_params* p, int64_t N, int64_t P) {
  if (N < p->window || P < 0 || P > N || N > 0x7fffffff) return -1;
  return 0;
}

/* ------------------------------------------------------------------ budget split
 *
 * Two-stage compression (Section 2.2): stage 1 evicts in the prefix only to leave room for
 * the decode stage; stage 2 keeps a protected core and consolidates scratch into the slots
 * that remain (Section 2.3: scratch is consolidated only within the remaining budget).  The
 * paper gives no split rule; the reading taken here:
 *   - the last R_eff = min(R, D) decode tokens ("recent reasoning pivots", Section 2.1) are
 *     always kept and are counted outside the core;
 *   - N <= B: nothing to do (identity);
 *   - the prefix keeps B_p tokens (default max(B/4, ceil(P/64))), more if the decode trace
 *     cannot use the space, never more than B - R_eff;
 *   - the decode trace outside the recent tail gets slots = B - R_eff - P_keep;
 *     slots = 0 with decode tokens waiting is the prefix_budget_exhausted regime (Section 5.2);
 *   - of the slots, C (default 4/5) go to the protected core and M = slots - C to
 *     representatives.
 */
void cask_ref_plan(const cask_ref_params* p, int32_t P, int32_t N, cask_ref_plan_t* out) {
  const int32_t B = p->budget;
  const int32_t decode = N - P;
  const int32_t recent = resolved_recent(p) < decode ? resolved_recent(p) : decode;
  const int32_t scratch_span = decode - recent; /* decode tokens that compete for slots */
  memset(out, 0, sizeof(*out));
  out->r_eff = recent;
  if (N <= B) { /* everything fits: every token is kept as it is */
    out->p_keep = P;
    out->slots = scratch_span;
    out->core = scratch_span;
    out->status = CASK_REF_ST_IDENTITY;
    return;
  }
  /* What the prefix may claim: its own budget B_p, or the space the decode trace would leave
   * empty, whichever is larger.  Stage 1 keeps the largest prefix count that respects this
   * claim, the prefix length and the room beside the recent tail: the conditions are tested
   * one candidate count after the other, from the top. */
  int32_t own = p->prefix_budget;
  if (own < 0) {
    own = B / 4;
    while ((int64_t)own * 64 < P) ++own; /* at least one kept token per 64 prefix tokens, rounded up */
  }
  const int32_t beside_recent = B - recent;
  const int32_t idle = beside_recent - scratch_span; /* negative when the decode trace overflows */
  const int32_t claim = own > idle ? own : idle;
  int32_t keep = P < beside_recent ? P : beside_recent;
  while (keep > 0 && keep > claim) --keep;
  out->p_keep = keep;
  out->slots = beside_recent - keep;
  /* decode tokens that cannot be kept verbatim in the slots */
  const int32_t overflow = scratch_span - out->slots;
  if (overflow <= 0) { /* all of them fit (also: no such token at all): nothing to consolidate */
    out->core = scratch_span;
    out->status = CASK_REF_ST_MERGE_INACTIVE;
    return;
  }
  if (out->slots == 0) { /* tokens wait and the prefix left them nothing (Section 5.2) */
    out->status = CASK_REF_ST_PREFIX_BUDGET_EXHAUSTED;
    return;
  }
  if (p->core >= 0)
    out->core = p->core < out->slots ? p->core : out->slots;
  else
    out->core = (int32_t)(((int64_t)out->slots * 4) / 5);
  out->seeds = out->slots - out->core;
  out->status = out->seeds > 0 ? CASK_REF_ST_ACTIVE : CASK_REF_ST_MERGE_INACTIVE;
}

/* ------------------------------------------------------------------ scoring
 *
 * The paper inherits an eviction-style scalar importance (Section 1) and leaves the deployed
 * form open; a_i is "local score mass" (Section 2.4).  Reading taken: window row (w, g) sits
 * at cache slot t_w = N - W + w; its attention over the keys it can see is
 * softmax_j(scale * <q_{w,g}, k_j>), j <= t_w (all j when causal = 0); the score of key j is
 * the mean of that probability over all W*G rows.  Rounded once to float.
 */
static void score_unit(const cask_ref_params* p, int64_t N, const void* K, int64_t k_row0,
                       const void* Q, int64_t q_row0, float* s_out) {
  const int d = p->head_dim, W = p->window, G = p->q_per_kv;
  const double scale = p->softmax_scale > 0.0f ? (double)p->softmax_scale : 1.0 / sqrt((double)d);
  double* kd = (double*)malloc(sizeof(double) * (size_t)N * d);
  double* logit = (double*)malloc(sizeof(double) * (size_t)N);
  double* acc = (double*)calloc((size_t)N, sizeof(double));
  double* q = (double*)malloc(sizeof(double) * d);
  for (int64_t j = 0; j < N; ++j)
    for (int c = 0; c < d; ++c) kd[j * d + c] = load_elem(K, p->dtype, (k_row0 + j) * d + c);
  for (int w = 0; w < W; ++w) {
    int64_t t = N - W + w;
    int64_t last = p->causal ? t : N - 1;
    for (int g = 0; g < G; ++g) {
      int64_t qrow = q_row0 + (int64_t)w * G + g;
      for (int c = 0; c < d; ++c) q[c] = load_elem(Q, p->dtype, qrow * d + c);
      double mx = -INFINITY;
      for (int64_t j = 0; j <= last; ++j) {
        double dot = 0.0;
        for (int c = 0; c < d; ++c) dot += q[c] * kd[j * d + c];
        logit[j] = scale * dot;
        if (logit[j] > mx) mx = logit[j];
      }
      double z = 0.0;
      for (int64_t j = 0; j <= last; ++j) z += exp(logit[j] - mx);
      for (int64_t j = 0; j <= last; ++j) acc[j] += exp(logit[j] - mx) / z;
    }
  }
  for (int64_t j = 0; j < N; ++j) s_out[j] = (float)(acc[j] / ((double)W * (double)G));
  free(kd);
  free(logit);
  free(acc);
  free(q);
}

int cask_ref_score(const cask_ref_params* p, int32_t n_units, const int64_t* row_off,
                   const void* K, const void* Q, float* scores, int n_threads) {
  if (check_shape(p) || n_units < 0) return -1;
  for (int32_t u = 0; u < n_units; ++u)
    if (check_unit(p, row_off[u + 1] - row_off[u], 0)) return -1;
#ifdef _OPENMP
  if (n_threads > 0) omp_set_num_threads(n_threads);
#endif
  (void)n_threads;
#pragma omp parallel for schedule(dynamic, 1)
  for (int32_t u = 0; u < n_units; ++u) {
    int64_t N = row_off[u + 1] - row_off[u];
    score_unit(p, N, K, row_off[u], Q, (int64_t)u * p->window * p->q_per_kv, scores + row_off[u]);
  }
  return 0;
}

/* ------------------------------------------------------------------ ordering
 *
 * "Retain the top tokens" (Section 1).  Total order: higher float score first, equal scores
 * in ascending cache index.  top-k = the first k of the range under this order.
 */
typedef struct {
  float s;
  int32_t i;
} ranked_t;

static int ranked_cmp(const void* a, const void* b) {
  const ranked_t* x = (const ranked_t*)a;
  const ranked_t* y = (const ranked_t*)b;
  if (x->s > y->s) return -1;
  if (x->s < y->s) return 1;
  if (x->i < y->i) return -1;
  if (x->i > y->i) return 1;
  return 0;
}

/* order[0..n) := unit-local rows lo..hi-1 sorted by the total order */
static ranked_t* rank_range(const float* s, int32_t lo, int32_t hi) {
  int32_t n = hi - lo;
  ranked_t* r = (ranked_t*)malloc(sizeof(ranked_t) * (size_t)(n > 0 ? n : 1));
  for (int32_t t = 0; t < n; ++t) {
    r[t].s = s[lo + t];
    r[t].i = lo + t;
  }
  qsort(r, (size_t)n, sizeof(ranked_t), ranked_cmp);
  return r;
}

/* Stage 1 (Section 2.2): eviction in the prefix; survivors are the top P_keep. */
static void prefix_evict_unit(const cask_ref_plan_t* pl, int32_t P, const float* s, uint8_t* role) {
  ranked_t* r = rank_range(s, 0, P);
  for (int32_t t = 0; t < P; ++t)
    role[r[t].i] = t < pl->p_keep ? CASK_REF_PREFIX_KEEP : CASK_REF_PREFIX_DROP;
  free(r);
}

/* Stage 2 decomposition (Section 2.1): the protected core is decided first (top C of the
 * decode trace outside the recent tail), then the next M become the seeds of the
 * representatives, and the rest is mergeable scratch offered to them (donors). */
static void partition_unit(const cask_ref_plan_t* pl, int32_t P, int32_t N, const float* s,
                           uint8_t* role) {
  int32_t hi = N - pl->r_eff;
  for (int32_t j = hi; j < N; ++j) role[j] = CASK_REF_RECENT;
  if (pl->status & CASK_REF_ST_PREFIX_BUDGET_EXHAUSTED) {
    for (int32_t j = P; j < hi; ++j) role[j] = CASK_REF_DECODE_EVICT;
    return;
  }
  ranked_t* r = rank_range(s, P, hi);
  for (int32_t t = 0; t < hi - P; ++t) {
    uint8_t x;
    if (t < pl->core)
      x = CASK_REF_CORE;
    else if (t < pl->core + pl->seeds)
      x = CASK_REF_SEED;
    else
      x = CASK_REF_DONOR;
    role[r[t].i] = x;
  }
  free(r);
}

/* De-duplicated seeding (an option; the paper does not say how representatives are seeded,
 * and with the default rule two copies of one token can both become seeds and split their
 * group).  The scratch rows are the decode rows outside the recent tail that are not core,
 * in the total order.  Walk the first min(#scratch, h*M) of them: a row becomes a seed unless
 * its key cosine with some seed chosen earlier is >= tau (then it is a donor, and the
 * consolidation will fold it into a seed it resembles); stop when M seeds are chosen.
 * Everything else in the scratch is a donor. */
static void dedup_seeds_unit(const cask_ref_params* p, const cask_ref_plan_t* pl, int32_t P, int32_t N,
                             const void* K, int64_t row0, const float* s, uint8_t* role,
                             double* min_gap) {
  if (min_gap) *min_gap = INFINITY;
  if (pl->status & CASK_REF_ST_PREFIX_BUDGET_EXHAUSTED) return;
  const int32_t hi = N - pl->r_eff, n = hi - P, d = p->head_dim;
  if (pl->seeds <= 0 || n <= pl->core + pl->seeds) return; /* no donors: nothing to de-duplicate for */
  const double tau = (double)p->sim_threshold;
  ranked_t* r = rank_range(s, P, hi);
  int64_t horizon = (int64_t)p->seed_dedup * pl->seeds;
  if (horizon > n - pl->core) horizon = n - pl->core;
  for (int32_t t = pl->core; t < n; ++t) role[r[t].i] = CASK_REF_DONOR;
  double* seed_k = (double*)malloc(sizeof(double) * (size_t)pl->seeds * d);
  double* seed_norm = (double*)malloc(sizeof(double) * (size_t)pl->seeds);
  double* ki = (double*)malloc(sizeof(double) * d);
  int32_t chosen = 0;
  for (int64_t t = pl->core; t < pl->core + horizon && chosen < pl->seeds; ++t) {
    const int32_t i = r[t].i;
    double nn = 0.0;
    for (int c = 0; c < d; ++c) {
      ki[c] = load_elem(K, p->dtype, (row0 + i) * d + c);
      nn += ki[c] * ki[c];
    }
    const double ni = sqrt(nn);
    int blocked = 0;
    for (int32_t q = 0; q < chosen; ++q) {
      double dot = 0.0;
      for (int c = 0; c < d; ++c) dot += ki[c] * seed_k[(size_t)q * d + c];
      const double sim = (ni == 0.0 || seed_norm[q] == 0.0) ? 0.0 : dot / (ni * seed_norm[q]);
      if (min_gap && fabs(sim - tau) < *min_gap) *min_gap = fabs(sim - tau);
      if (sim >= tau) blocked = 1;
    }
    if (blocked) continue;
    memcpy(seed_k + (size_t)chosen * d, ki, sizeof(double) * d);
    seed_norm[chosen] = ni;
    ++chosen;
    role[i] = CASK_REF_SEED;
  }
  free(seed_k);
  free(seed_norm);
  free(ki);
  free(r);
}

int cask_ref_prefix_evict(const cask_ref_params* p, int32_t n_units, const int64_t* row_off,
                          const int32_t* prefix_len, const float* scores, uint8_t* role,
                          int32_t* status) {
  if (check_params(p) || n_units < 0) return -1;
  for (int32_t u = 0; u < n_units; ++u)
    if (check_unit(p, row_off[u + 1] - row_off[u], prefix_len[u])) return -1;
  for (int32_t u = 0; u < n_units; ++u) {
    int32_t N = (int32_t)(row_off[u + 1] - row_off[u]);
    cask_ref_plan_t pl;
    cask_ref_plan(p, prefix_len[u], N, &pl);
    prefix_evict_unit(&pl, prefix_len[u], scores + row_off[u], role + row_off[u]);
    if (status) status[u] = pl.status;
  }
  return 0;
}

int cask_ref_partition(const cask_ref_params* p, int32_t n_units, const int64_t* row_off,
                       const int32_t* prefix_len, const float* scores, uint8_t* role,
                       int32_t* status) {
  if (check_params(p) || n_units < 0) return -1;
  for (int32_t u = 0; u < n_units; ++u)
    if (check_unit(p, row_off[u + 1] - row_off[u], prefix_len[u])) return -1;
  for (int32_t u = 0; u < n_units; ++u) {
    int32_t N = (int32_t)(row_off[u + 1] - row_off[u]);
    cask_ref_plan_t pl;
    cask_ref_plan(p, prefix_len[u], N, &pl);
    partition_unit(&pl, prefix_len[u], N, scores + row_off[u], role + row_off[u]);
    if (status) status[u] = pl.status;
  }
  return 0;
}

int cask_ref_partition_keys(const cask_ref_params* p, int32_t n_units, const int64_t* row_off,
                            const int32_t* prefix_len, const void* K, const float* scores,
                            uint8_t* role, int32_t* status, double* min_gap) {
  if (check_params(p) || n_units < 0 || !K) return -1;
  for (int32_t u = 0; u < n_units; ++u)
    if (check_unit(p, row_off[u + 1] - row_off[u], prefix_len[u])) return -1;
  for (int32_t u = 0; u < n_units; ++u) {
    int32_t N = (int32_t)(row_off[u + 1] - row_off[u]);
    cask_ref_plan_t pl;
    cask_ref_plan(p, prefix_len[u], N, &pl);
    partition_unit(&pl, prefix_len[u], N, scores + row_off[u], role + row_off[u]);
    if (min_gap) min_gap[u] = INFINITY;
    if (p->seed_dedup > 0)
      dedup_seeds_unit(p, &pl, prefix_len[u], N, K, row_off[u], scores + row_off[u], role + row_off[u],
                       min_gap ? &min_gap[u] : NULL);
    if (status) status[u] = pl.status;
  }
  return 0;
}

/* ------------------------------------------------------------------ consolidation
 *
 * A scratch token can go once a representative close enough to it stays in the cache
 * (Section 1); similarity is raw cosine between cached keys (Section 2.5 names raw cosine as
 * the plain geometry).  Reading taken: each donor looks at every seed, picks the
 * seed of largest cosine (ties: lowest cache index), and folds into it when that cosine is
 * >= tau; otherwise it is evicted.  Core tokens neither give nor receive merges (Section 2.1).
 */
static void consolidate_unit(const cask_ref_params* p, int32_t N, const void* K, int64_t row0,
                             const uint8_t* role, int32_t* assign, double* best_sim,
                             double* second_sim) {
  const int d = p->head_dim;
  const double tau = (double)p->sim_threshold;
  int32_t n_seed = 0;
  for (int32_t j = 0; j < N; ++j) n_seed += role[j] == CASK_REF_SEED;
  int32_t* seed_row = (int32_t*)malloc(sizeof(int32_t) * (size_t)(n_seed > 0 ? n_seed : 1));
  double* seed_k = (double*)malloc(sizeof(double) * (size_t)(n_seed > 0 ? n_seed : 1) * d);
  double* seed_norm = (double*)malloc(sizeof(double) * (size_t)(n_seed > 0 ? n_seed : 1));
  double* ki = (double*)malloc(sizeof(double) * d);
  int32_t t = 0;
  for (int32_t j = 0; j < N; ++j) {
    if (role[j] != CASK_REF_SEED) continue;
    double nn = 0.0;
    for (int c = 0; c < d; ++c) {
      double x = load_elem(K, p->dtype, (row0 + j) * d + c);
      seed_k[(size_t)t * d + c] = x;
      nn += x * x;
    }
    seed_norm[t] = sqrt(nn);
    seed_row[t] = j;
    ++t;
  }
  for (int32_t i = 0; i < N; ++i) {
    if (best_sim) best_sim[i] = NAN;
    if (second_sim) second_sim[i] = NAN;
    switch (role[i]) {
      case CASK_REF_PREFIX_KEEP:
      case CASK_REF_CORE:
      case CASK_REF_SEED:
      case CASK_REF_RECENT:
        assign[i] = i;
        continue;
      case CASK_REF_DONOR:
        break;
      default:
        assign[i] = -1;
        continue;
    }
    double nn = 0.0;
    for (int c = 0; c < d; ++c) {
      ki[c] = load_elem(K, p->dtype, (row0 + i) * d + c);
      nn += ki[c] * ki[c];
    }
    double ni = sqrt(nn);
    double best = -INFINITY, second = -INFINITY;
    int32_t best_r = -1;
    for (int32_t r = 0; r < n_seed; ++r) { /* ascending cache index */
      /* locality (Section 5.2): seeds further away than the radius are not candidates */
      if (p->merge_radius > 0 && abs(seed_row[r] - i) > p->merge_radius) continue;
      double sim;
      if (p->merge_geometry == 1) {
        /* kappa-weighted merge distance (Section 2.5): sum over rotary bands f = channels
         * (f, f + d/2) of w_f times the Euclidean distance inside the band; kept as the
         * NEGATED distance so that "larger is closer" like the cosine */
        double dist = 0.0;
        for (int f = 0; f < d / 2; ++f) {
          const double a = ki[f] - seed_k[(size_t)r * d + f];
          const double b = ki[f + d / 2] - seed_k[(size_t)r * d + f + d / 2];
          dist += (double)p->band_weight[f] * sqrt(a * a + b * b);
        }
        sim = -dist;
      } else {
        double dot = 0.0;
        for (int c = 0; c < d; ++c) dot += ki[c] * seed_k[(size_t)r * d + c];
        sim = (ni == 0.0 || seed_norm[r] == 0.0) ? 0.0 : dot / (ni * seed_norm[r]);
      }
      if (sim > best) {
        second = best;
        best = sim;
        best_r = r;
      } else if (sim > second) {
        second = sim;
      }
    }
    if (best_sim) best_sim[i] = best;
    if (second_sim) second_sim[i] = second;
    /* geometry 1 compares the negated distance with -theta */
    const double bar = p->merge_geometry == 1 ? -(double)p->dist_threshold : tau;
    assign[i] = (best_r >= 0 && best >= bar) ? seed_row[best_r] : -1;
  }
  free(seed_row);
  free(seed_k);
  free(seed_norm);
  free(ki);
}

int cask_ref_consolidate(const cask_ref_params* p, int32_t n_units, const int64_t* row_off,
                         const int32_t* prefix_len, const void* K, const float* scores,
                         const uint8_t* role, int32_t* assign, double* best_sim,
                         double* second_sim) {
  (void)scores;
  if (check_params(p) || n_units < 0) return -1;
  for (int32_t u = 0; u < n_units; ++u)
    if (check_unit(p, row_off[u + 1] - row_off[u], prefix_len[u])) return -1;
#pragma omp parallel for schedule(dynamic, 1)
  for (int32_t u = 0; u < n_units; ++u) {
    int32_t N = (int32_t)(row_off[u + 1] - row_off[u]);
    consolidate_unit(p, N, K, row_off[u], role + row_off[u], assign + row_off[u],
                     best_sim ? best_sim + row_off[u] : NULL,
                     second_sim ? second_sim + row_off[u] : NULL);
  }
  return 0;
}

/* ------------------------------------------------------------------ fold + compaction
 *
 * m-folding (Section 2.4): for a group G (a seed and the donors assigned to it)
 *   m = sum a_i,  k~ = sum a_i k_i / m,  v~ = sum a_i v_i / m,
 * with a_i the token's score (its local score mass).  A cache row may itself stand for
 * several original tokens (a representative of an earlier event): `count` says how many, 1
 * when no counts are given, and folding adds the counts.  If every a_i is zero the weights
 * become the counts (the uniform mean over the original tokens).  A group of one is the
 * token itself, copied without arithmetic.  The
 * output keeps ascending source order (a representative sits at its seed's index); kept
 * tokens pass through bit-identically (C subset of R, |R| <= B; Section 2.3).
 */
static void emit_unit(const cask_ref_params* p, int32_t N, const void* K, const void* V,
                      int64_t row0, const float* s, const uint8_t* role, const int32_t* assign_src,
                      void* K_out, void* V_out, int64_t out_row0, int32_t* out_len,
                      int32_t* out_src, float* out_mass, int32_t* slot_of, int32_t* n_merged,
                      const int32_t* count, int32_t* out_count) {
  const int d = p->head_dim;
  const size_t es = elem_size(p->dtype);
  double* ksum = (double*)malloc(sizeof(double) * d);
  double* vsum = (double*)malloc(sizeof(double) * d);
  int32_t* slot = (int32_t*)malloc(sizeof(int32_t) * (size_t)N);
  int32_t t = 0, merged = 0;
  for (int32_t j = 0; j < N; ++j) {
    slot[j] = -1;
    uint8_t x = role[j];
    if (x != CASK_REF_PREFIX_KEEP && x != CASK_REF_CORE && x != CASK_REF_RECENT &&
        x != CASK_REF_SEED)
      continue;
    int32_t members = 1;
    if (x == CASK_REF_SEED)
      for (int32_t i = 0; i < N; ++i)
        if (role[i] == CASK_REF_DONOR && assign_src[i] == j) ++members;
    char* ko = (char*)K_out + (size_t)(out_row0 + t) * d * es;
    char* vo = (char*)V_out + (size_t)(out_row0 + t) * d * es;
    double mass;
    int64_t cnt = count ? count[j] : 1;
    if (members == 1) {
      memcpy(ko, (const char*)K + (size_t)(row0 + j) * d * es, d * es);
      memcpy(vo, (const char*)V + (size_t)(row0 + j) * d * es, d * es);
      mass = (double)s[j];
    } else {
      double m = (double)s[j];
      for (int32_t i = 0; i < N; ++i)
        if (role[i] == CASK_REF_DONOR && assign_src[i] == j) {
          m += (double)s[i];
          cnt += count ? count[i] : 1;
        }
      int uniform = (m == 0.0);
      double denom = uniform ? (double)cnt : m;
      for (int c = 0; c < d; ++c) ksum[c] = vsum[c] = 0.0;
      for (int32_t i = 0; i < N; ++i) {
        if (!(i == j || (role[i] == CASK_REF_DONOR && assign_src[i] == j))) continue;
        double a = uniform ? (double)(count ? count[i] : 1) : (double)s[i];
        for (int c = 0; c < d; ++c) {
          ksum[c] += a * load_elem(K, p->dtype, (row0 + i) * d + c);
          vsum[c] += a * load_elem(V, p->dtype, (row0 + i) * d + c);
        }
      }
      for (int c = 0; c < d; ++c) {
        store_elem(K_out, p->dtype, (out_row0 + t) * d + c, ksum[c] / denom);
        store_elem(V_out, p->dtype, (out_row0 + t) * d + c, vsum[c] / denom);
      }
      mass = m;
      merged += members - 1;
    }
    out_src[t] = j;
    if (out_mass) out_mass[t] = (float)mass;
    if (out_count) out_count[t] = (int32_t)cnt;
    slot[j] = t;
    ++t;
  }
  *out_len = t;
  *n_merged = merged;
  if (slot_of) {
    for (int32_t i = 0; i < N; ++i) {
      if (role[i] == CASK_REF_DONOR)
        slot_of[i] = assign_src[i] >= 0 ? slot[assign_src[i]] : -1;
      else
        slot_of[i] = slot[i];
    }
  }
  free(ksum);
  free(vsum);
  free(slot);
}

int cask_ref_compress_step(const cask_ref_params* p, int32_t n_units, const int64_t* row_off,
                           const int32_t* prefix_len, const void* K, const void* V, const void* Q,
                           int scores_given, float* scores, const int32_t* in_count, void* K_out,
                           void* V_out, int32_t out_stride_rows, int32_t* out_len,
                           int32_t* out_src, float* out_mass, int32_t* out_count,
                           int32_t* assign, uint8_t* role_out, int32_t* status, int n_threads) {
  if (check_params(p) || n_units < 0 || !scores || out_stride_rows < p->budget) return -1;
  if (in_count)
    for (int64_t i = 0; i < row_off[n_units]; ++i)
      if (in_count[i] < 1) return -1;
  for (int32_t u = 0; u < n_units; ++u)
    if (check_unit(p, row_off[u + 1] - row_off[u], prefix_len[u])) return -1;
#ifdef _OPENMP
  if (n_threads > 0) omp_set_num_threads(n_threads);
#endif
  (void)n_threads;
  const int32_t B = p->budget;
#pragma omp parallel for schedule(dynamic, 1)
  for (int32_t u = 0; u < n_units; ++u) {
    const int64_t row0 = row_off[u];
    const int32_t N = (int32_t)(row_off[u + 1] - row0);
    const int32_t P = prefix_len[u];
    float* s = scores + row0;
    cask_ref_plan_t pl;
    cask_ref_plan(p, P, N, &pl);
    if (!scores_given)
      score_unit(p, N, K, row0, Q, (int64_t)u * p->window * p->q_per_kv, s);
    uint8_t* role = (uint8_t*)malloc((size_t)N);
    int32_t* asrc = (int32_t*)malloc(sizeof(int32_t) * (size_t)N);
    prefix_evict_unit(&pl, P, s, role);
    partition_unit(&pl, P, N, s, role);
    if (p->seed_dedup > 0) dedup_seeds_unit(p, &pl, P, N, K, row0, s, role, NULL);
    consolidate_unit(p, N, K, row0, role, asrc, NULL, NULL);
    int32_t merged = 0;
    emit_unit(p, N, K, V, row0, s, role, asrc, K_out, V_out, (int64_t)u * out_stride_rows,
              &out_len[u], out_src + (int64_t)u * B, out_mass ? out_mass + (int64_t)u * B : NULL,
              assign ? assign + row0 : NULL, &merged, in_count ? in_count + row0 : NULL,
              out_count ? out_count + (int64_t)u * B : NULL);
    int32_t st = pl.status;
    if (merged == 0 && !(st & (CASK_REF_ST_IDENTITY | CASK_REF_ST_PREFIX_BUDGET_EXHAUSTED)))
      st |= CASK_REF_ST_MERGE_INACTIVE;
    if (status) status[u] = st;
    if (role_out) memcpy(role_out + row0, role, (size_t)N);
    free(role);
    free(asrc);
  }
  return 0;
}

int cask_ref_compress(const cask_ref_params* p, int32_t n_units, const int64_t* row_off,
                      const int32_t* prefix_len, const void* K, const void* V, const void* Q,
                      int scores_given, float* scores, void* K_out, void* V_out,
                      int32_t* out_len, int32_t* out_src, float* out_mass, int32_t* assign,
                      uint8_t* role_out, int32_t* status, int n_threads) {
  return cask_ref_compress_step(p, n_units, row_off, prefix_len, K, V, Q, scores_given, scores, NULL,
                                K_out, V_out, p ? p->budget : 0, out_len, out_src, out_mass, NULL,
                                assign, role_out, status, n_threads);
}

/* Representative-set mass diagnostics (Section 2.6):
 *   rho_core = sum_{k in C} s_k / sum_{k in TopK} s_k,
 *   rho_rep  = sum_{k in R} s_k / sum_{k in TopK} s_k.
 * Readings (the paper names an oracle scorer and a k without fixing either):
 *   s     the event's own score vector -- no other scorer exists at this boundary;
 *   TopK  the min(B, N) best rows of the unit in the order (score descending, index
 *         ascending): what plain top-k eviction to the same budget would keep;
 *   C     the rows protection keeps verbatim: prefix survivors, decode core, recent tail;
 *   R     the output rows; a representative counts with the mass of its whole group, so the
 *         sum over R is the sum of out_mass (rho_rep can exceed 1 when folding recovers mass
 *         from outside TopK).
 * A unit whose TopK mass is zero reports 1 for both: there is nothing to lose. */
int cask_ref_mass_diagnostics(const cask_ref_params* p, int32_t n_units, const int64_t* row_off,
                              const float* scores, const uint8_t* role, const float* out_mass,
                              const int32_t* out_len, float* rho) {
  if (!p || !row_off || !scores || !role || !out_mass || !out_len || !rho || n_units < 0) return -1;
  if (check_shape(p) != 0) return -1;
  for (int32_t u = 0; u < n_units; ++u) {
    const int64_t row0 = row_off[u];
    const int32_t N = (int32_t)(row_off[u + 1] - row0);
    const float* s = scores + row0;
    ranked_t* r = rank_range(s, 0, N);
    const int32_t k = N < p->budget ? N : p->budget;
    double top = 0.0, core = 0.0, rep = 0.0;
    for (int32_t t = 0; t < k; ++t) top += (double)r[t].s;
    free(r);
    for (int32_t i = 0; i < N; ++i) {
      const uint8_t ro = role[row0 + i];
      if (ro == CASK_REF_PREFIX_KEEP || ro == CASK_REF_CORE || ro == CASK_REF_RECENT) core += (double)s[i];
    }
    for (int32_t t = 0; t < out_len[u]; ++t) rep += (double)out_mass[(int64_t)u * p->budget + t];
    rho[2 * u + 0] = top > 0.0 ? (float)(core / top) : 1.0f;
    rho[2 * u + 1] = top > 0.0 ? (float)(rep / top) : 1.0f;
  }
  return 0;
}

int cask_ref_group_diagnostics(const cask_ref_params* p, int32_t n_units, const int64_t* row_off,
                               const void* K, const float* scores, const int32_t* assign,
                               const void* K_out, int32_t out_stride_rows, float* dispersion,
                               float* lost_mass) {
  if (!p || !row_off || !K || !scores || !assign || !K_out || !dispersion || !lost_mass || n_units < 0)
    return -1;
  if (check_shape(p) != 0 || out_stride_rows < p->budget) return -1;
  const int d = p->head_dim;
  if (p->band_weight)
    for (int f = 0; f < d / 2; ++f)
      if (!(p->band_weight[f] >= 0.0f)) return -1;
  for (int32_t u = 0; u < n_units; ++u) {
    const int64_t row0 = row_off[u];
    const int32_t N = (int32_t)(row_off[u + 1] - row0);
    double disp = 0.0, lost = 0.0;
    for (int32_t i = 0; i < N; ++i) {
      const double a = (double)scores[row0 + i];
      const int32_t t = assign[row0 + i];
      if (t < 0) {
        lost += a;
        continue;
      }
      if (t >= p->budget) return -1;
      const int64_t rep = ((int64_t)u * out_stride_rows + t) * d;
      double norm = 0.0;
      for (int f = 0; f < d / 2; ++f) {
        const double x = load_elem(K, p->dtype, (row0 + i) * d + f) - load_elem(K_out, p->dtype, rep + f);
        const double y = load_elem(K, p->dtype, (row0 + i) * d + f + d / 2) -
                         load_elem(K_out, p->dtype, rep + f + d / 2);
        const double w = p->band_weight ? (double)p->band_weight[f] : 1.0;
        norm += w * sqrt(x * x + y * y);
      }
      disp += a * norm;
    }
    dispersion[u] = (float)disp;
    lost_mass[u] = (float)lost;
  }
  return 0;
}

int cask_ref_attend(const cask_ref_params* p, int32_t n_units, const void* Q, const void* K_c,
                    const void* V_c, int32_t stride_rows, const int32_t* len, const int32_t* count,
                    int32_t count_pitch, double* out) {
  if (!p || !Q || !K_c || !V_c || !len || !out || n_units < 0) return -1;
  if (check_shape(p) != 0) return -1;
  const int d = p->head_dim, G = p->q_per_kv;
  const double scale = p->softmax_scale > 0.0f ? (double)p->softmax_scale : 1.0 / sqrt((double)d);
  for (int32_t u = 0; u < n_units; ++u) {
    const int32_t L = len[u];
    if (L < 1 || L > stride_rows || (count && L > count_pitch)) return -1;
    double* logit = (double*)malloc(sizeof(double) * (size_t)L);
    if (!logit) return -2;
    for (int g = 0; g < G; ++g) {
      const int64_t qrow = ((int64_t)u * G + g) * d;
      double top = -INFINITY;
      for (int32_t t = 0; t < L; ++t) {
        const int64_t krow = ((int64_t)u * stride_rows + t) * d;
        double dot = 0.0;
        for (int c = 0; c < d; ++c) dot += load_elem(Q, p->dtype, qrow + c) * load_elem(K_c, p->dtype, krow + c);
        double x = scale * dot;
        if (count) {
          const int32_t n = count[(int64_t)u * count_pitch + t];
          if (n < 1) {
            free(logit);
            return -1;
          }
          x += log((double)n);
        }
        logit[t] = x;
        if (x > top) top = x;
      }
      double den = 0.0;
      for (int32_t t = 0; t < L; ++t) {
        logit[t] = exp(logit[t] - top);
        den += logit[t];
      }
      for (int c = 0; c < d; ++c) {
        double acc = 0.0;
        for (int32_t t = 0; t < L; ++t)
          acc += logit[t] * load_elem(V_c, p->dtype, ((int64_t)u * stride_rows + t) * d + c);
        out[qrow + c] = acc / den;
      }
    }
    free(logit);
  }
  return 0;
}
