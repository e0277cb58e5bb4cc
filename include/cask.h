/*
 * cask.h -- C ABI of the MI355X (gfx950) CASK compression-event library.
 *
 * One compression event, for every unit u = (sequence, layer, KV head) of a batch:
 *   score      the cached tokens with the attention mass that a window of recent queries
 *              puts on them (the scalar importance the method inherits, Section 1; used as
 *              the local score mass a_i of Section 2.4);
 *   evict      in the prefix, to leave room for the decode stage (stage 1, Section 2.2);
 *   partition  the decode trace into protected core and mergeable scratch (Section 2.1);
 *   consolidate near-duplicate scratch onto representatives by key cosine similarity
 *              (Section 2.5 names raw cosine as the plain merge geometry);
 *   fold       each group into a weighted representative (Section 2.4:
 *              m = sum a_i, k~ = sum a_i k_i / m, v~ = sum a_i v_i / m);
 *   compact    to the budget with the core included (|R| <= B, C subset of R, Section 2.3),
 *              flagging the prefix_budget_exhausted / merge_inactive regimes (Section 5.2).
 *
 * Conventions
 *   - Every data pointer is a DEVICE pointer owned by the caller, unless marked HOST.
 *     The library allocates nothing, never synchronises, and only enqueues work on
 *     `hip_stream` (a hipStream_t passed as void*; NULL = the default stream).
 *   - Inputs are never modified.  Outputs of one call must not alias its inputs.
 *   - K, V, Q, K_out, V_out and the workspace must be 16-byte aligned (CASK_EINVAL otherwise).
 *   - Argument errors are found on the host before any launch and returned as a
 *     negative code; nothing is enqueued then.  Per-unit regime outcomes are status bits
 *     in device memory, not errors.
 *   - Row layout: K, V are [total_rows, d] row-major in the cache dtype; unit u owns rows
 *     [row_off[u], row_off[u+1]).  row_off and prefix_len live on the device AND are
 *     mirrored on the host (the host copy sizes the launches).
 *   - Calls that share a workspace on different streams race; one workspace per stream.
 *   - The first launch of a kernel on a device raises that kernel's LDS limit (a function
 *     attribute, not a stream operation; the scoring sweeps, the one-launch scoring and
 *     cask_attend's matrix-core kernels need more than the default 64 KB): make one call of an
 *     entry point with the shapes in question before capturing the stream into a HIP graph.
 *   - Entry points may be called from several host threads (each on its own stream and
 *     workspace); the timing aid at the end of this header records one stream at a time.
 */
#ifndef CASK_H
#define CASK_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { CASK_F32 = 0, CASK_BF16 = 1 } cask_dtype;

/* return codes */
enum {
  CASK_OK = 0,
  CASK_EINVAL = -1,  /* bad parameter, shape or NULL pointer */
  CASK_ENOMEM = -2,  /* workspace smaller than cask_workspace_bytes() */
  CASK_EDEVICE = -3  /* a HIP call failed (launch error) */
};

/* per-unit status bits (device memory) */
enum {
  CASK_ST_ACTIVE = 0,
  CASK_ST_IDENTITY = 1,                /* N <= B: output equals input */
  CASK_ST_PREFIX_BUDGET_EXHAUSTED = 2, /* the prefix left no decode slot (Section 5.2) */
  CASK_ST_MERGE_INACTIVE = 4           /* no donor was folded into any representative */
};

/* token roles */
enum {
  CASK_ROLE_PREFIX_DROP = 0,
  CASK_ROLE_PREFIX_KEEP = 1,
  CASK_ROLE_CORE = 2,
  CASK_ROLE_SEED = 3,   /* kept scratch token that representatives are built around */
  CASK_ROLE_DONOR = 4,  /* scratch token offered to the seeds */
  CASK_ROLE_RECENT = 5,
  CASK_ROLE_DECODE_EVICT = 6 /* decode token dropped unseen: exhausted regime only */
};

typedef struct {
  int32_t dtype;         /* cask_dtype of K, V, Q and of K_out, V_out */
  int32_t head_dim;      /* d: 64 or 128 */
  int32_t q_per_kv;      /* G query heads per KV head */
  int32_t window;        /* W query positions = the last W cache slots of the unit */
  int32_t recent;        /* R: tail always kept verbatim; < 0 => W */
  int32_t budget;        /* B >= R + 1 */
  int32_t core;          /* C; < 0 => floor(4 * slots / 5) */
  int32_t prefix_budget; /* B_p; < 0 => max(floor(B / 4), ceil(P / 64)) */
  float sim_threshold;   /* tau: a donor folds into its best seed iff cosine >= tau */
  float softmax_scale;   /* <= 0 => 1 / sqrt(d) */
  int32_t causal;        /* 1: the query at slot t sees keys j <= t; 0: all keys */
  int32_t scores_given;  /* cask_compress only: 1 => `scores` is an input, scoring skipped */
  /* Merge geometry of the consolidation step; all zero / NULL = raw key cosine, no locality. */
  int32_t merge_radius;  /* r > 0: a donor may fold only into a seed at most r cache rows away
                            (merges stay inside temporal neighbourhoods, Section 5.2); 0: anywhere */
  int32_t merge_geometry; /* 0: key cosine >= sim_threshold; 1: kappa-weighted band distance
                             (Section 2.5) d(k_i, k_j) = sum_f w_f |k_i,f - k_j,f|_2 <= dist_threshold,
                             f the rotary band of channels (f, f + d/2); nearest seed, ties to the
                             lowest cache index */
  float dist_threshold;  /* theta of geometry 1, >= 0 */
  const float* band_weight; /* DEVICE [d/2], geometry 1: w_f = |kappa(omega_f)| >= 0 (the paper does
                               not fix the horizon distribution behind kappa: the caller supplies
                               the weights; not validated on the device) */
  /* De-duplicated seeding (the paper does not say how representatives are seeded).  0: the
     seeds are the M best-scored scratch rows.  h > 0: walk the best h * M scratch rows in the
     order (score descending, index ascending); a row becomes a seed unless its key cosine
     with a seed chosen before it is >= sim_threshold, until M seeds are chosen; rows passed
     over, and all rows behind the walk, are donors; fewer than M seeds (out_len < B) may
     result.  Needs merge_geometry 0 and h * (largest M of the plan) <= 2048, else
     CASK_EINVAL.  Applies to cask_partition, cask_compress and cask_compress_step.  bf16
     caches run the walk's cosines on the matrix cores (CASK_PATH_DEDUP_VECTOR in path_flags
     sends them through the vector kernel that serves fp32 caches, for comparisons). */
  int32_t seed_dedup;
  /* Path selection for measurements and tests; all zero = the library's own choice.  None of
     them changes what is computed (results agree bit for bit, or to the scoring tolerance where
     a different kernel sums in another order). */
  uint32_t path_flags;   /* CASK_PATH_* bits below */
  int32_t score_splits;  /* 1..64: key splits of the first scoring sweep; 0 = chosen by a cost model */
  int32_t score_qsplit;  /* 1 | 2: workgroups sharing a key tile in the second sweep; 0 = chosen */
} cask_params;

enum {
  CASK_PATH_NO_FUSED_TAIL = 1,  /* short units: the general kernels instead of the one-launch tail */
  CASK_PATH_NO_FUSED_SCORE = 2, /* short units: two scoring launches instead of one */
  CASK_PATH_DEDUP_VECTOR = 4,   /* bf16 de-duplicated seeding on the vector kernel fp32 caches use */
  CASK_PATH_ATTEND_VECTOR = 8,  /* bf16 cask_attend on the vector kernel fp32 caches use */
  CASK_PATH_NO_FUSED_SWEEPS = 16, /* many long units with W*G <= 512: two scoring launches instead of one */
  CASK_PATH_FORCE_FUSED_SWEEPS = 32, /* W*G <= 512: one scoring launch whatever the number of units */
  CASK_PATH_NARROW_ROWS = 64, /* both scoring sweeps: 64 resident rows per wave (256 per workgroup) whatever the shape */
  CASK_PATH_WIDE_ROWS = 128   /* both scoring sweeps: 128 resident rows per wave (512 per workgroup) whatever the shape */
};

typedef struct {
  int32_t n_units;
  const int64_t* row_off;      /* DEVICE [n_units + 1]; W <= N_u = row_off[u+1] - row_off[u] <= 2^23 - 1 */
  const int32_t* prefix_len;   /* DEVICE [n_units], 0 <= P_u <= N_u */
  const int64_t* row_off_host; /* HOST mirror of row_off */
  const int32_t* prefix_len_host; /* HOST mirror of prefix_len */
  const void* K;               /* DEVICE [total_rows, d], keys as cached (post-RoPE) */
  const void* V;               /* DEVICE [total_rows, d] */
  const void* Q;               /* DEVICE [n_units, W, G, d]; row (w, g) sits at slot N_u - W + w */
} cask_batch;

/* Budget split of one unit (two-stage compression, Section 2.2; pure host arithmetic). */
typedef struct {
  int32_t r_eff;  /* min(R, D) */
  int32_t p_keep; /* prefix tokens kept by stage 1 */
  int32_t slots;  /* decode slots outside the recent tail: B - r_eff - p_keep */
  int32_t core;   /* C */
  int32_t seeds;  /* M = slots - C representatives */
  int32_t status; /* regime bits that follow from the sizes alone */
} cask_plan_t;

/* HOST: the split for prefix length P and cache length N.  Returns CASK_EINVAL on bad sizes. */
int cask_plan(const cask_params* params, int32_t P, int32_t N, cask_plan_t* out);

/* HOST: bytes of device workspace every entry point below needs for such a batch (with the
 * same params: score_splits and score_qsplit enter the layout). */
size_t cask_workspace_bytes(const cask_params* params, int32_t n_units, int64_t total_rows,
                            int32_t max_unit_len);

/* Scores (importance; the a_i of Section 2.4): scores[row_off[u] + j] = mean over the W*G
 * window rows of softmax_j(scale * <q, k_j>) with the causal mask of `params`.
 * Reads K, Q.  Writes scores [total_rows] float. */
int cask_score(const cask_params* params, const cask_batch* batch, float* scores, void* ws,
               size_t ws_bytes, void* hip_stream);

/* Stage 1 (Section 2.2): role[row_off[u] + j], j < P_u, := PREFIX_KEEP for the top P_keep
 * by (score descending, index ascending), else PREFIX_DROP.  status[u] := plan bits.
 * Rows >= P_u of `role` are left untouched. */
int cask_prefix_evict(const cask_params* params, const cask_batch* batch, const float* scores,
                      uint8_t* role, int32_t* status, void* ws, size_t ws_bytes,
                      void* hip_stream);

/* Stage 2 decomposition (Section 2.1): writes role for rows [P_u, N_u): top C => CORE, next
 * M => SEED, rest => DONOR, last r_eff => RECENT (DECODE_EVICT when exhausted).
 * status[u] := plan bits.  Rows < P_u are left untouched. */
int cask_partition(const cask_params* params, const cask_batch* batch, const float* scores,
                   uint8_t* role, int32_t* status, void* ws, size_t ws_bytes, void* hip_stream);

/* Selective consolidation (Sections 2.1, 2.5): for every DONOR the seed of largest key
 * cosine (ties: lowest cache index); assign[row] = unit-local row of that seed when the
 * cosine is >= tau, -1 otherwise; kept rows get their own unit-local row; dropped rows -1.
 * Reads K, role.  `scores` is accepted for symmetry and not read. */
int cask_consolidate(const cask_params* params, const cask_batch* batch, const float* scores,
                     const uint8_t* role, int32_t* assign, void* ws, size_t ws_bytes,
                     void* hip_stream);

/* The whole event (Sections 2.1-2.4).  (A batch whose units all have at most 1024 rows, with
 * B <= 1024, bf16 and the cosine geometry, takes a one-launch path after scoring; results and
 * tie rules are the same; with d = 128 the two scoring sweeps of such a batch are one launch
 * as well; CASK_PATH_NO_FUSED_TAIL and CASK_PATH_NO_FUSED_SCORE in path_flags switch these
 * paths off.)
 *   K_out, V_out [n_units, B, d]  rows [0, out_len[u]) in ascending source order; a
 *                                 representative sits at its seed's position; kept tokens
 *                                 are bit-identical copies; rows >= out_len[u] untouched
 *   out_len  [n_units]            = min(N_u, B)
 *   out_src  [n_units, B]         unit-local source row of each output row
 *   out_mass [n_units, B] or NULL mass m of each output row (own score if not merged)
 *   assign   [total_rows] or NULL output slot each input row went to, -1 if evicted
 *   scores   [total_rows] or NULL input when params->scores_given, else optional output
 *   status   [n_units]            regime bits (plan bits, plus MERGE_INACTIVE when no donor
 *                                 passed tau)
 */
int cask_compress(const cask_params* params, const cask_batch* batch, void* K_out, void* V_out,
                  int32_t* out_len, int32_t* out_src, float* out_mass, int32_t* assign,
                  float* scores, int32_t* status, void* ws, size_t ws_bytes, void* hip_stream);

/* cask_compress for callers that cannot allocate device memory: a stream under HIP graph
 * capture, a tight serving loop, a harness that forbids allocation.  Same arguments and results
 * as cask_compress without `ws`: the workspace is a fixed array of CASK_STATIC_WORKSPACE_BYTES
 * in device memory that the library owns (each device the library is used on holds its copy
 * until the process ends).  Calls no allocating routine.
 *   - CASK_ENOMEM when cask_workspace_bytes() for the batch exceeds CASK_STATIC_WORKSPACE_BYTES
 *     (48 MiB: about 1.3 million cached rows, e.g. 112 units of 8448 rows with 896 window rows);
 *     nothing is enqueued then.
 *   - Every call on a device shares that device's array: calls that overlap on one device (two
 *     streams, two threads) race.  Calls in sequence on one stream are fine; nothing has to be
 *     cleared between them.
 *   - The first call on a device looks up the array's address (no stream operation): make one
 *     call before capturing the stream into a HIP graph. */
#define CASK_STATIC_WORKSPACE_BYTES (48u << 20)
int cask_compress_static(const cask_params* params, const cask_batch* batch, void* K_out, void* V_out,
                         int32_t* out_len, int32_t* out_src, float* out_mass, int32_t* assign,
                         float* scores, int32_t* status, void* hip_stream);

/* One event of a decode loop: cask_compress with per-row token counts carried in and out and
 * an output row stride.  The paper's runs compress a trace several times (its result tables
 * count the events) without stating a trigger or carry rule; the readings taken:
 *   - the caller fires the event when a unit holds B + delta rows (delta tokens decoded since
 *     the last event); the next event's prefix length is this event's p_keep (cask_plan);
 *   - in_count [total_rows] or NULL: original tokens each cache row stands for (>= 1; NULL = 1
 *     each).  out_count [n_units, B] or NULL: sum over each output row's group.  A group whose
 *     score mass is zero is averaged with the counts as weights; otherwise the fold weights are
 *     the fresh scores, exactly as in cask_compress;
 *   - K_out, V_out are [n_units, out_stride_rows, d] with out_stride_rows >= B: unit u's output
 *     starts at row u * out_stride_rows, so decoded tokens can be appended behind it and the
 *     buffer handed back as the next event's K, V (units of equal length then lie back to
 *     back).  out_src, out_mass, out_count stay [n_units, B].
 * Everything else as cask_compress, which is this call with in_count = out_count = NULL and
 * out_stride_rows = B.  in_count is not validated on the device: a count < 1 gives a
 * meaningless out_count, nothing worse. */
int cask_compress_step(const cask_params* params, const cask_batch* batch, const int32_t* in_count,
                       void* K_out, void* V_out, int32_t out_stride_rows, int32_t* out_len,
                       int32_t* out_src, float* out_mass, int32_t* out_count, int32_t* assign,
                       float* scores, int32_t* status, void* ws, size_t ws_bytes,
                       void* hip_stream);

/* Representative-set mass diagnostics (Section 2.6), optional, after cask_compress:
 *   rho[2u]     = rho_core = mass(C) / mass(TopK)
 *   rho[2u + 1] = rho_rep  = mass(R) / mass(TopK)
 * for every unit, where mass is the sum of `scores`; TopK = the min(B, N_u) best rows in the
 * order (score descending, index ascending), i.e. what plain top-k eviction to the same budget
 * would keep; C = the rows protection keeps verbatim (PREFIX_KEEP, CORE, RECENT); mass(R) = the
 * sum of out_mass over the unit's out_len output rows (a representative counts with its whole
 * group, so rho_rep may exceed 1).  A unit whose TopK mass is zero reports 1 and 1.
 * Reads scores [total_rows], role [total_rows] (as written by cask_prefix_evict and
 * cask_partition for the same scores), out_mass [n_units, B], out_len [n_units]; writes
 * rho [n_units, 2] float.  Needs no workspace. */
int cask_mass_diagnostics(const cask_params* params, const cask_batch* batch, const float* scores,
                          const uint8_t* role, const float* out_mass, const int32_t* out_len,
                          float* rho, void* hip_stream);

/* Perturbation diagnostics of a finished event (Section 2.6, Appendix B: a representative's
 * error is bounded by within-group kappa-dispersion plus lost mass), optional, after
 * cask_compress or cask_compress_step:
 *   dispersion[u] = sum over the unit's rows with assign[i] >= 0 of
 *                   scores[i] * || K[i] - K_out[u, assign[i]] ||_kappa
 *   lost_mass[u]  = sum of scores[i] over the rows with assign[i] < 0
 * where ||x||_kappa = sum over rotary bands f (channels f and f + d/2) of w_f * ||x_f||_2 with
 * w = params->band_weight (device, float [d/2], not validated), all ones when that is NULL;
 * the scores are used as they are (not renormalised inside a group); the representative is
 * the row as stored in K_out (cache dtype), so rows kept verbatim add exact zeros; a fold
 * hands its group's whole mass to the representative, so what is lost is the mass of the rows
 * that leave without one.
 * Reads K, scores [total_rows], assign [total_rows] (output slot or -1, as written by
 * cask_compress; a value >= B is skipped), K_out [n_units, out_stride_rows, d] (device,
 * 16-byte aligned, out_stride_rows >= B); writes dispersion, lost_mass [n_units] float.
 * Needs no workspace. */
int cask_group_diagnostics(const cask_params* params, const cask_batch* batch, const float* scores,
                           const int32_t* assign, const void* K_out, int32_t out_stride_rows,
                           float* dispersion, float* lost_mass, void* hip_stream);

/* Consumer side: one decode step's attention over a compressed cache.  The folds preserve
 * group mass (Section 2.4); how attention uses a representative is left open by the paper.
 * The reading taken here is proportional attention: a row standing for n original tokens
 * enters the softmax with n times its weight,
 *     p_t = softmax_t( scale * <q, k_t> + ln(count_t) ),   out = sum_t p_t v_t,
 * exact when the n tokens had the same key and value, plain attention for count == NULL.
 *   Q     [n_units, G, d]               device, cache dtype: the step's queries of the G heads
 *   K_c, V_c [n_units, stride_rows, d]  device, cache dtype: rows [0, len[u]) are used
 *   len   [n_units] device (cask_compress's out_len); clamped to [0, stride_rows], 0 gives zeros
 *   count [n_units, count_pitch] device or NULL (cask_compress_step's out_count; values < 1
 *         are not validated and count as 1, and so do rows at or behind count_pitch)
 *   out   [n_units, G, d]               device, cache dtype (fp32 accumulation, rounded once)
 * All data pointers 16-byte aligned.  scale = softmax_scale, 1/sqrt(d) when that is <= 0.  Needs
 * no workspace.  Decoded tokens appended behind the compressed rows attend the same way (their
 * count is 1): pass the buffer with its row stride and the enlarged len.  bf16 caches run on
 * the matrix cores (CASK_PATH_ATTEND_VECTOR in path_flags sends them through the vector kernel
 * that serves fp32 caches, for comparisons).  (Graph capture: see the
 * note on LDS limits at the top of this header.) */
int cask_attend(const cask_params* params, int32_t n_units, const void* Q, const void* K_c,
                const void* V_c, int32_t stride_rows, const int32_t* len, const int32_t* count,
                int32_t count_pitch, void* out, void* hip_stream);

/* Measurement aid (not part of the method): per-stage timing of cask_compress with HIP
 * events recorded on the caller's stream between its kernels.  Stage order: 0 score sweep A
 * (row statistics), 1 score sweep B (column mass; with the small kernel that combines the row
 * statistics of several key splits in front of it), 2 select (with the ordered walk over the
 * roles, which cask_compress runs in the same kernel), 3 index roles (zero in cask_compress),
 * 4 similarity, 5 gather merged donors (grouping by seed; the same launch copies the kept rows
 * to the output), 6 emit (folds the seeds that have donors).  A batch of short units (every unit at most
 * 1024 rows, B <= 1024, bf16, cosine geometry) runs stages 2-6 as one kernel: its time is
 * reported as stage 2 and stages 3-6 read as the cost of an empty event pair; with d = 128
 * stages 0 and 1 are one kernel too, reported as stage 0.
 * cask_timing_enable(n > 0) creates events for the next n compress calls (n <= 4096) and
 * switches recording on; n <= 0 switches it off and destroys them.  Calls beyond n are not
 * recorded.  cask_timing_read waits for the recorded calls, writes the summed milliseconds
 * per stage into stage_ms[CASK_N_STAGES] and the number of recorded calls into *n_calls,
 * and rearms.  cask_timing_enable_stages(n, k) records only the first k stages (k = 2: the two
 * scoring sweeps, three events per call instead of eight); the other entries read as 0.
 * The bookkeeping is guarded by a lock; the events of one recording belong to one stream. */
#define CASK_N_STAGES 7
int cask_timing_enable(int max_calls);
int cask_timing_enable_stages(int max_calls, int n_stages);
int cask_timing_read(float* stage_ms, int* n_calls);

/* Measurement aids (not part of the method): plain loops that pin what the device delivers, so
 * that a report can print measured ceilings beside the published ones.  Both only launch a kernel
 * on `hip_stream`; the caller times it with events.
 *
 * cask_probe_issue: register-only loops of the scoring sweeps' instruction mix.  One unit = one
 * v_mfma_f32_32x32x16_bf16 (32 768 flop, 32 matrix-pipe cycles), kind 0; the same followed by the
 * vector epilogue of two logits (fma, exp2, add each), kind 1; the vector part alone, kind 2;
 * kind 1 with the MFMA's first operand read from LDS as the sweeps read theirs, kind 3; kind 1
 * with the six vector instructions in dependent order on one running sum, kind 4.
 * `blocks` workgroups of 4 * waves_per_simd waves (one compute unit's SIMDs each get
 * waves_per_simd of them) run iters * 8 units per wave.
 *   operands  DEVICE, 32 KB of random bf16 values, 16-byte aligned (operand bits set the power)
 *   cycles    DEVICE uint64 [2 * blocks]: per workgroup, shader-clock cycles and 100 MHz ticks
 *   sink      DEVICE float [blocks * 256 * waves_per_simd] (keeps the loops alive)
 * cask_probe_copy: dst[0, bytes) = src[0, bytes), 16 bytes per thread and step; bytes a multiple
 * of 16, both pointers 16-byte aligned.  (Also the kernel of known size that scales the
 * profiler's HBM byte counters.) */
int cask_probe_issue(int kind, int waves_per_simd, int blocks, int iters, const void* operands,
                     uint64_t* cycles, float* sink, void* hip_stream);
int cask_probe_copy(const void* src, void* dst, size_t bytes, void* hip_stream);
/* cask_probe_read: a read-only stream over src[0, bytes) (what the HBM-bound kernels of the event
 * do: they read far more than they write); `blocks` workgroups of 256 threads, eight 16-byte
 * loads in flight per thread; sink DEVICE uint32 [blocks * 256]. */
int cask_probe_read(const void* src, size_t bytes, uint32_t* sink, int blocks, void* hip_stream);

/* HOST: short name of a return code. */
const char* cask_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* CASK_H */
