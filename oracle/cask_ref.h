/*
 * CASK compression-event ORACLE -- test infrastructure, not product code.
 *
 * A plain, slow, single-pass-per-definition CPU implementation of the decode-time
 * KV compression event of CASK (core-aware selective KV compression): score the
 * cached tokens from a window of recent queries, evict in the prefix (two-stage
 * compression, Section 2.2), split the decode trace into protected core and
 * mergeable scratch (Section 2.1), fold near-duplicate scratch into weighted
 * representatives (Section 2.4, the m-folding equations), and compact to the
 * budget (|R| <= B and C subset of R, Section 2.3).
 *
 * Everything is computed in double precision on the exact input values; the score
 * vector is rounded once to float and that float vector decides every ordering.
 * Nothing here is blocked, fused or reordered beyond what the rules state.  It
 * shares no code with the HIP library; only tests, the smoke check and the
 * benchmark's cpu_baseline leg may call it.
 *
 * Where the paper leaves a rule open (deployed score form, similarity threshold,
 * budget split, tie-break) the reading taken is stated at the function that
 * implements it.  The constants of those readings (tau = 0.9, the quarter share
 * and 1/64 floor of the prefix budget, the 4/5 core share, softmax-mean scoring)
 * have no external anchor: "parity unpinned" for those constants -- they are
 * parameters with defaults, pinned only by self-consistency tests.  The same holds for
 * the choice of two later rules the paper leaves open altogether -- how attention weighs a
 * representative (cask_ref_attend: count-proportional) and how seeds avoid duplicates
 * (seed_dedup: the greedy walk): what each function computes is pinned (library softmax and
 * the repeated-row identity; the properties that characterise the walk), that the paper
 * would choose these rules is not.
 *
 * All pointers are HOST pointers owned by the caller.
 */
#ifndef CASK_REF_H
#define CASK_REF_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { CASK_REF_F32 = 0, CASK_REF_BF16 = 1 };

/* per-unit regime bits (Section 5.2 names prefix_budget_exhausted and merge_inactive) */
enum {
  CASK_REF_ST_ACTIVE = 0,
  CASK_REF_ST_IDENTITY = 1,
  CASK_REF_ST_PREFIX_BUDGET_EXHAUSTED = 2,
  CASK_REF_ST_MERGE_INACTIVE = 4
};

/* token roles */
enum {
  CASK_REF_PREFIX_DROP = 0,
  CASK_REF_PREFIX_KEEP = 1,
  CASK_REF_CORE = 2,
  CASK_REF_SEED = 3,
  CASK_REF_DONOR = 4,
  CASK_REF_RECENT = 5,
  CASK_REF_DECODE_EVICT = 6 /* decode token dropped without a merge attempt (exhausted regime) */
};

typedef struct {
  int32_t dtype;         /* element type of K, V, Q and of K_out, V_out */
  int32_t head_dim;      /* d */
  int32_t q_per_kv;      /* G query heads per KV head */
  int32_t window;        /* W query positions = the last W cache slots */
  int32_t recent;        /* R always-kept tail; < 0 means W */
  int32_t budget;        /* B */
  int32_t core;          /* C; < 0 means floor(4*slots/5) */
  int32_t prefix_budget; /* B_p; < 0 means max(floor(B/4), ceil(P/64)) */
  float sim_threshold;   /* tau */
  float softmax_scale;   /* <= 0 means 1/sqrt(d) */
  int32_t causal;        /* 1: query at slot t sees keys j <= t */
  /* Merge geometry (Sections 2.5 and 5.2).  All zero / NULL = raw cosine, no locality. */
  int32_t merge_radius;  /* r > 0: a donor may fold only into a seed at most r cache rows away
                            (merges stay inside temporal neighbourhoods); 0: anywhere */
  int32_t merge_geometry; /* 0: key cosine >= sim_threshold; 1: kappa-weighted band distance
                             d(k_i, k_j) = sum_f w_f |k_i,f - k_j,f|_2 <= dist_threshold, f the
                             rotary band made of channels (f, f + d/2) */
  float dist_threshold;  /* theta of geometry 1 */
  const float* band_weight; /* geometry 1: w_f = |kappa(omega_f)| >= 0, d/2 values; the paper
                               never fixes the horizon distribution behind kappa, so the caller
                               supplies the weights */
  /* De-duplicated seeding.  0: the seeds are the M best-scored scratch rows.  h > 0: walk the
     best h*M scratch rows in the order (score descending, index ascending); a row becomes a
     seed unless its key cosine with a seed chosen before it is >= sim_threshold; stop at M
     seeds.  Rows passed over, and everything behind the walk, are donors.  Fewer than M seeds
     may result.  Needs merge_geometry 0. */
  int32_t seed_dedup;
} cask_ref_params;

typedef struct {
  int32_t r_eff;  /* min(R, D) */
  int32_t p_keep; /* prefix tokens kept */
  int32_t slots;  /* decode slots outside the recent tail */
  int32_t core;   /* C */
  int32_t seeds;  /* M */
  int32_t status; /* regime bits known from sizes alone */
} cask_ref_plan_t;

/* Budget split for one unit with prefix length P and cache length N. */
void cask_ref_plan(const cask_ref_params* p, int32_t P, int32_t N, cask_ref_plan_t* out);

/* Round a double to the nearest bf16 (ties to even); returns the 16-bit pattern. */
uint16_t cask_ref_bf16_from_double(double x);
double cask_ref_bf16_to_double(uint16_t h);

/* scores[row_off[u] + j] = mean over the W*G window rows of softmax_j(scale <q,k_j>). */
int cask_ref_score(const cask_ref_params* p, int32_t n_units, const int64_t* row_off,
                   const void* K, const void* Q, float* scores, int n_threads);

/* role[0,P_u) := PREFIX_KEEP for the top P_keep by (score desc, index asc), else PREFIX_DROP. */
int cask_ref_prefix_evict(const cask_ref_params* p, int32_t n_units, const int64_t* row_off,
                          const int32_t* prefix_len, const float* scores, uint8_t* role,
                          int32_t* status);

/* role[P_u,N_u) := CORE / SEED / DONOR / RECENT (or DECODE_EVICT when exhausted). */
int cask_ref_partition(const cask_ref_params* p, int32_t n_units, const int64_t* row_off,
                       const int32_t* prefix_len, const float* scores, uint8_t* role,
                       int32_t* status);

/* cask_ref_partition followed by de-duplicated seeding when p->seed_dedup > 0 (needs the keys).
 * min_gap[u] (optional) = the smallest |cosine - sim_threshold| over the (row, earlier seed)
 * pairs the walk compared, +inf when it compared none: how close the unit came to another
 * seed set. */
int cask_ref_partition_keys(const cask_ref_params* p, int32_t n_units, const int64_t* row_off,
                            const int32_t* prefix_len, const void* K, const float* scores,
                            uint8_t* role, int32_t* status, double* min_gap);

/* assign[row] = unit-local row of the seed a donor folds into, own row if kept, -1 if evicted.
 * best_sim / second_sim (either may be NULL): per row, the largest and second largest cosine
 * over the seeds for donors (NaN elsewhere); used by tests to excuse near-ties. */
int cask_ref_consolidate(const cask_ref_params* p, int32_t n_units, const int64_t* row_off,
                         const int32_t* prefix_len, const void* K, const float* scores,
                         const uint8_t* role, int32_t* assign, double* best_sim,
                         double* second_sim);

/* The whole event.  scores_given != 0: `scores` is an input; else it is written.
 * K_out, V_out: [n_units, B, d] in the cache dtype, rows >= out_len[u] untouched.
 * out_src: [n_units, B] unit-local source row (the seed's row for a representative).
 * out_mass: [n_units, B] (may be NULL) mass m of each output row.
 * assign: [total_rows] (may be NULL) output slot of every input row, -1 if evicted.
 * role: [total_rows] (may be NULL) final roles. */
int cask_ref_compress(const cask_ref_params* p, int32_t n_units, const int64_t* row_off,
                      const int32_t* prefix_len, const void* K, const void* V, const void* Q,
                      int scores_given, float* scores, void* K_out, void* V_out,
                      int32_t* out_len, int32_t* out_src, float* out_mass, int32_t* assign,
                      uint8_t* role, int32_t* status, int n_threads);

/* One event of a decode loop (the paper's runs compress a trace several times, Tables 3 and
 * the bridge table count the events; it states no trigger or carry rule, so these are readings):
 *   - a unit is compressed when it holds B + delta rows (delta = the number of tokens decoded
 *     between events; the caller decides when to call);
 *   - every cache row stands for in_count[row] >= 1 original tokens (NULL: all 1); a fold adds
 *     the counts of its members into out_count, and a group whose score mass is zero is
 *     averaged with the counts as weights.  Scores are always fresh: the mass a representative
 *     receives from the current window already is the mass of what it stands for;
 *   - the output of unit u starts at row u * out_stride_rows of K_out / V_out
 *     (out_stride_rows >= B), so that a caller can keep appending decoded tokens behind it;
 *     out_src, out_mass, out_count stay [n_units, B];
 *   - the prefix of the next event is the surviving prefix: p_keep of this event's plan.
 * With in_count == NULL and out_stride_rows == B this is cask_ref_compress. */
int cask_ref_compress_step(const cask_ref_params* p, int32_t n_units, const int64_t* row_off,
                           const int32_t* prefix_len, const void* K, const void* V, const void* Q,
                           int scores_given, float* scores, const int32_t* in_count, void* K_out,
                           void* V_out, int32_t out_stride_rows, int32_t* out_len,
                           int32_t* out_src, float* out_mass, int32_t* out_count,
                           int32_t* assign, uint8_t* role_out, int32_t* status, int n_threads);

/* Representative-set mass diagnostics of Section 2.6 (see the definition in the source for the
 * readings of TopK, C and R).  role, out_mass, out_len as produced by cask_ref_compress.
 * rho: [n_units][2] = {rho_core, rho_rep}. */
int cask_ref_mass_diagnostics(const cask_ref_params* p, int32_t n_units, const int64_t* row_off,
                              const float* scores, const uint8_t* role, const float* out_mass,
                              const int32_t* out_len, float* rho);

/* Perturbation diagnostics of a finished event (Section 2.6, Appendix B): the bound on a
 * representative's error splits into within-group kappa-dispersion and lost mass.
 * Readings taken here:
 *   - the weights a_i are the event's scores, not renormalised inside a group;
 *   - ||x||_kappa is the band norm of Section 2.5, sum_f w_f * ||x_f||_2 over the rotary bands
 *     (channels f and f + d/2), w = p->band_weight, all ones when that is NULL;
 *   - k~_G is the representative as stored: row assign[i] of K_out (cache dtype);
 *   - dispersion[u] = sum over rows with assign[i] >= 0 of s_i * ||k_i - k~||_kappa (rows
 *     kept verbatim add exact zeros);
 *   - a fold hands its group's whole mass to the representative, so the mass that is lost is
 *     that of the rows that leave without one: lost_mass[u] = sum of s_i over assign[i] < 0.
 * assign as written by cask_ref_compress(_step); K_out rows of unit u start at row
 * u * out_stride_rows. */
int cask_ref_group_diagnostics(const cask_ref_params* p, int32_t n_units, const int64_t* row_off,
                               const void* K, const float* scores, const int32_t* assign,
                               const void* K_out, int32_t out_stride_rows, float* dispersion,
                               float* lost_mass);

/* Consumer side: one decode step's attention over a compressed cache.  A fold keeps the mass of its
 * group (Section 2.4); what a consumer does with it the paper leaves open; the reading
 * taken here is proportional attention: a row that stands for n original tokens enters the
 * softmax with n times its weight,
 *     p_t = softmax_t( scale * <q, k_t> + ln(count_t) ),   o = sum_t p_t v_t,
 * which is exact when the n tokens it replaced had the same key and value (attention over a
 * cache with a row repeated n times equals attention over the cache with that row once and
 * count n), and reduces to plain attention when count is NULL or all ones.
 *   Q   [n_units, G, d]            the step's queries of the G heads that share the KV head
 *   K_c, V_c [n_units, stride_rows, d]  rows [0, len[u]) in use
 *   count [n_units, count_pitch] or NULL (count_pitch >= max len)
 *   out [n_units, G, d] double (not rounded to the cache dtype)
 * scale = softmax_scale, or 1/sqrt(d) when that is <= 0 (the one rule of every scorer here). */
int cask_ref_attend(const cask_ref_params* p, int32_t n_units, const void* Q, const void* K_c,
                    const void* V_c, int32_t stride_rows, const int32_t* len, const int32_t* count,
                    int32_t count_pitch, double* out);

#ifdef __cplusplus
}
#endif
#endif
