// Shared declarations of the gfx950 CASK kernels: kernel-side parameter block, the budget
// split (two-stage compression, Section 2.2 of the paper), workspace layout and the
// launchers each translation unit exports to the C-ABI layer.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>

#include "cask.h"

namespace cask {

constexpr int kWave = 64;

// Kernel-side copy of cask_params with defaults resolved.
struct KParams {
  int dtype;
  int d;
  int G;
  int W;
  int R;             // resolved recent
  int B;
  int core;          // < 0 => default share
  int prefix_budget; // < 0 => default
  float tau;
  float scale_log2;  // softmax scale * log2(e): logits are handled in base-2 units
  int causal;
  int Mq;            // W * G window rows
  int radius;        // merge radius in cache rows, 0 = unlimited
  int geometry;      // 0 cosine, 1 kappa-weighted band distance
  float theta;       // distance threshold of geometry 1
  const float* band_w;  // device [d / 2] band weights of geometry 1
  int dedup;         // h > 0: de-duplicated seeding over the best h * M scratch rows
  unsigned path_flags;  // CASK_PATH_* bits (host-side path selection only)
  int score_splits;  // forced key splits of sweep A, 0 = cost model
  int score_qsplit;  // forced window-row halves of sweep B, 0 = chosen
};

constexpr int kSeedWalkMax = 2048;  // rows the de-duplicating walk of a unit can cover

struct UnitPlan {
  int r_eff, p_keep, slots, core, seeds, status;
};

// Budget split of one unit.  Stage 1 evicts in the prefix only to leave room for the decode
// stage; the decode trace outside the always-kept recent tail gets the remaining slots, split
// into a protected core and representative seeds (Sections 2.1-2.3); a unit whose prefix
// leaves no slot is flagged prefix_budget_exhausted (Section 5.2).
__host__ __device__ inline UnitPlan make_plan(int R, int B, int core_param, int prefix_budget,
                                              int P, int N) {
  UnitPlan pl;
  const int D = N - P;
  const int r_eff = R < D ? R : D;
  const int dnr = D - r_eff;
  pl.r_eff = r_eff;
  if (N <= B) {
    pl.p_keep = P;
    pl.slots = dnr;
    pl.core = dnr;
    pl.seeds = 0;
    pl.status = CASK_ST_IDENTITY;
    return pl;
  }
  int bp = prefix_budget;
  if (bp < 0) {
    const int quarter = B / 4, floor64 = (P + 63) / 64;
    bp = quarter > floor64 ? quarter : floor64;
  }
  const int room = B - r_eff;
  const int unused = room - dnr;
  const int want = bp > unused ? bp : unused;
  int p_keep = P;
  if (room < p_keep) p_keep = room;
  if (want < p_keep) p_keep = want;
  pl.p_keep = p_keep;
  pl.slots = room - p_keep;
  if (dnr <= pl.slots) {
    pl.core = dnr;
    pl.seeds = 0;
    pl.status = CASK_ST_MERGE_INACTIVE;
  } else if (pl.slots == 0) {
    pl.core = 0;
    pl.seeds = 0;
    pl.status = CASK_ST_PREFIX_BUDGET_EXHAUSTED;
  } else {
    int c = core_param >= 0 ? (core_param < pl.slots ? core_param : pl.slots)
                            : (int)((4LL * pl.slots) / 5);
    pl.core = c;
    pl.seeds = pl.slots - c;
    pl.status = pl.seeds == 0 ? CASK_ST_MERGE_INACTIVE : CASK_ST_ACTIVE;
  }
  return pl;
}

__host__ __device__ inline UnitPlan make_plan(const KParams& kp, int P, int N) {
  return make_plan(kp.R, kp.B, kp.core, kp.prefix_budget, P, N);
}

// Seeds a unit can have when its roles come from the plan: seeds = slots - core with
// slots <= B, so at most B - core for an explicit core size and at most ceil(B / 5) for the
// default four-fifths core share.
// Rows of the scratch (n of them outside the recent tail, C of them core) that the selection
// marks as seeds: the M best, or with de-duplicated seeding the best h * M (the walk's range),
// when the unit has donors at all.
__host__ __device__ inline int seed_range(const KParams& kp, const UnitPlan& pl, int n) {
  if (kp.dedup <= 0 || pl.seeds <= 0 || n <= pl.core + pl.seeds) return pl.seeds;
  const long long want = (long long)kp.dedup * pl.seeds;
  return (int)(want < n - pl.core ? want : n - pl.core);
}

inline int plan_seed_bound(const KParams& kp) {
  const int sb = kp.core >= 0 ? (kp.B - kp.core > 0 ? kp.B - kp.core : 0) : (kp.B + 4) / 5;
  return sb < kp.B ? sb : kp.B;
}

// ---------------------------------------------------------------- element helpers

__device__ inline float bf16_bits_to_float(uint16_t h) {
  return __uint_as_float(((uint32_t)h) << 16);
}

// round-to-nearest-even float -> bf16 bit pattern
__device__ inline uint16_t float_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);  // NaN
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

template <typename T>
struct Elem;
template <>
struct Elem<float> {
  __device__ static float load(const float* p) { return *p; }
  __device__ static void store(float* p, float x) { *p = x; }
};
template <>
struct Elem<uint16_t> {
  __device__ static float load(const uint16_t* p) { return bf16_bits_to_float(*p); }
  __device__ static void store(uint16_t* p, float x) { *p = float_to_bf16_bits(x); }
};

// Order-preserving 32-bit key of a float score: larger score <=> larger key; -0 == +0.
__device__ inline uint32_t score_key(float s) {
  uint32_t u = __float_as_uint(s);
  if ((u << 1) == 0u) u = 0u;
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// Raises a kernel's dynamic-LDS limit the first time the kernel is launched on a device (a
// function attribute, not a stream operation).  One instance per kernel; safe to call from
// several threads.
class LdsLimitOnce {
 public:
  hipError_t ensure(const void* kernel, int bytes) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(mu_);
    if (done_ & (1ull << dev)) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess) done_ |= 1ull << dev;
    return e;
  }

 private:
  std::mutex mu_;
  uint64_t done_ = 0;
};

// ---------------------------------------------------------------- workspace layout

struct Workspace {
  // all offsets in bytes from the workspace base, 256-byte aligned
  size_t rowstat;    // float2 [n_units][n_splits][mq_pad]: per-split running (max, sum) per window row
  size_t bias;       // float  [n_units][mq_pad]: -L_row of every window row (base-2 log-sum-exp over all keys)
  size_t scores;     // float  [total_rows] (used when the caller passes no score buffer)
  size_t role;       // uint8  [total_rows]
  size_t slot_of;    // int32  [total_rows] output slot of kept rows, -1 otherwise
  size_t assign_ord; // int32  [total_rows] seed ordinal a donor folds into, -1 otherwise
  size_t merged_row; // int32  [total_rows] per unit: rows of merged donors, ascending
  size_t merged_ord; // int32  [total_rows] their seed ordinals
  size_t seg_row;    // int32  [total_rows] per unit: the same rows grouped by seed ordinal, ascending inside a group
  size_t seg_start;  // int32  [n_units][B + 1] where each seed's group starts in seg_row
  size_t seed_rows;  // int32  [n_units][B] unit-local rows of the seeds, ascending
  size_t n_merged;   // int32  [n_units]
  size_t n_seeds;    // int32  [n_units]
  size_t total;
  int n_splits;
  int split_len;     // keys per split (multiple of the key tile)
  int q_splits;      // sweep B: window-row halves taken by separate workgroups (1 or 2)
  int wide_rows;     // sweep A: 1 = 128 resident window rows per wave (512 per workgroup), 0 = 64 (256)
  int wide_cols;     // sweep B: 1 = 128 resident keys per wave (512 per workgroup), 0 = 64 (256)
  size_t parts;      // float  [n_units][ceil(Mq / 64)][parts_pitch]: partial column sums of the one-launch scoring
  int parts_pitch;   // 0: not laid out (units too long for that path)
  int mq_pad;
};

Workspace layout_workspace(const KParams& kp, int n_units, int64_t total_rows, int max_unit_len);

// ---------------------------------------------------------------- launchers

struct Batch {
  int n_units;
  const int64_t* row_off;
  const int32_t* prefix_len;
  const void* K;
  const void* V;
  const void* Q;
  int max_unit_len;
  int max_decode_len;  // longest decode trace N - P of the batch
  int64_t total_rows;
};

// `between`, when not null, is recorded on the stream between the two scoring sweeps.
hipError_t launch_score(const KParams& kp, const Batch& b, const Workspace& wl, char* ws,
                        float* scores, hipStream_t st, hipEvent_t between = nullptr);
// Both sweeps in one launch for long units with W*G <= 512 (bf16, d = 128), results in `scores`
// (must be 16-byte aligned when W*G > 256).
bool score_fused_fits(const KParams& kp, const Batch& b);
hipError_t launch_score_fused(const KParams& kp, const Batch& b, const Workspace& wl, float* scores,
                              hipStream_t st);
// Short units (at most Workspace::parts_pitch rows, one key split, bf16 d = 128): both scoring
// sweeps in one launch, leaving partial column sums for the consumer to add.
bool score_parts_fits(const KParams& kp, const Batch& b, const Workspace& wl);
hipError_t launch_score_parts(const KParams& kp, const Batch& b, const Workspace& wl, char* ws,
                              hipStream_t st);
hipError_t launch_select(const KParams& kp, const Batch& b, const float* scores, uint8_t* role,
                         int32_t* status, bool do_prefix, bool do_decode, hipStream_t st);
// de-duplicated seeding: turns the provisional seeds launch_select marked into seeds and donors
hipError_t launch_dedup_seeds(const KParams& kp, const Batch& b, const float* scores, uint8_t* role,
                              hipStream_t st);
// both stages of the selection and the ordered walk in one launch (whole-event path)
hipError_t launch_select_index(const KParams& kp, const Batch& b, const float* scores,
                               uint8_t* role, int32_t* status, int32_t* slot_of, int32_t* out_src,
                               int32_t* out_len, int32_t* seed_rows, int32_t* n_seeds,
                               hipStream_t st);
hipError_t launch_index_roles(const KParams& kp, const Batch& b, const uint8_t* role,
                              int32_t* slot_of, int32_t* out_src, int32_t* out_len,
                              int32_t* seed_rows, int32_t* n_seeds, hipStream_t st);
hipError_t launch_mass_diag(const KParams& kp, const Batch& b, const float* scores,
                            const uint8_t* role, const float* out_mass, const int32_t* out_len,
                            float* rho, hipStream_t st);
// roles_follow_plan: the roles were written by launch_select for these parameters, so the
// seeds per unit are bounded by the plan (lets the kernel keep all of them in LDS)
hipError_t launch_similarity(const KParams& kp, const Batch& b, const uint8_t* role,
                             const int32_t* seed_rows, const int32_t* n_seeds,
                             int32_t* assign_ord, bool roles_follow_plan, hipStream_t st);
// Copy of the kept rows that rides in the launch that groups the donors (`n_units` and
// `lane_bytes` are filled in by the launcher).
struct CopyJob {
  const unsigned char* K;
  const unsigned char* V;
  unsigned char* K_out;
  unsigned char* V_out;
  const float* scores;
  const int32_t* in_count;
  const int32_t* out_src;
  const int32_t* out_len;
  float* out_mass;
  int32_t* out_count;
  int out_stride;
  int n_units;
  int lane_bytes;
};
hipError_t launch_gather_merged(const KParams& kp, const Batch& b, const uint8_t* role,
                                const int32_t* assign_ord, const int32_t* slot_of,
                                const int32_t* seed_rows, int32_t* merged_row, int32_t* merged_ord,
                                int32_t* n_merged, int32_t* assign_out, int assign_mode,
                                int32_t* status, const int32_t* n_seeds, int32_t* seg_row,
                                int32_t* seg_start, const CopyJob* copy, hipStream_t st);
// Everything after scoring in one launch, for batches whose units all fit a workgroup (a row per
// thread), bf16, cosine geometry; `tail_small_fits` says whether a batch qualifies.
bool tail_small_fits(const KParams& kp, const Batch& b);
// `parts` not null: the scores come as `n_parts` partial sums per key (row pitch
// `parts_pitch`); the kernel adds them, writes the scores to `scores` and goes on from there.
hipError_t launch_tail_small(const KParams& kp, const Batch& b, float* scores, const float* parts,
                             int n_parts, int parts_pitch, const int32_t* in_count, void* K_out, void* V_out, int out_stride,
                             int32_t* out_len, int32_t* out_src, float* out_mass,
                             int32_t* out_count, int32_t* assign, int32_t* status,
                             hipStream_t st);
hipError_t launch_attend(const KParams& kp, int n_units, const void* Q, const void* Kc, const void* Vc,
                         int stride, const int32_t* len, const int32_t* count, int count_pitch,
                         void* out, hipStream_t st);
hipError_t launch_group_diag(const KParams& kp, const Batch& b, const float* scores,
                             const int32_t* assign, const void* K_out, int out_stride,
                             float* dispersion, float* lost_mass, hipStream_t st);
// Folds every seed that has donors into its output slot; the kept rows (the seeds' own among
// them) were copied by the launch that grouped the donors (`launch_gather_merged` with a copy).
hipError_t launch_emit(const KParams& kp, const Batch& b, const float* scores,
                       const int32_t* seed_rows, const int32_t* n_seeds, const int32_t* slot_of,
                       const int32_t* seg_row, const int32_t* seg_start,
                       const int32_t* n_merged, void* K_out, void* V_out, float* out_mass,
                       const int32_t* in_count, int32_t* out_count, int out_stride,
                       hipStream_t st);

}  // namespace cask
