// C-ABI layer: argument checks on the host, workspace carving, and the launch sequence of
// one compression event (two-stage compression, Section 2.2 of the paper):
//   score -> select (stage-1 prefix eviction + stage-2 core/seed/donor split) -> index roles
//   -> similarity -> gather merged donors -> emit (copy kept rows, fold representatives).
// Nothing here allocates or synchronises; everything is enqueued on the caller's stream.
#include <cmath>
#include <cstring>
#include <mutex>
#include <vector>

#include "cask_common.h"

namespace cask {

static size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

Workspace layout_workspace(const KParams& kp, int n_units, int64_t total_rows, int max_unit_len) {
  Workspace w;
  std::memset(&w, 0, sizeof(w));
  // Key splits of the row-statistics sweep: more splits mean more, shorter workgroups (better
  // balance over the 512 workgroup slots, two per compute unit) but a fixed cost per workgroup.
  // Measured on this kernel, a launch takes about (rounds of 512 workgroups, rounded up to a
  // half) x (stages per workgroup + 4), a stage of the wide form counting 1.85 narrow ones (twice
  // the products, less LDS traffic per product); take the split count that minimises it.
  auto best_splits = [&](bool wide, double* cost_out) {
    const int block_rows = wide ? 512 : 256;
    const int64_t pairs = (int64_t)n_units * ((kp.Mq + block_rows - 1) / block_rows);
    int best = 1;
    double best_cost = 0.0;
    for (int sp = 1; sp <= 64; ++sp) {
      const int len = (int)align_up((size_t)(max_unit_len + sp - 1) / sp, 64);
      if (sp > 1 && len < 1024) break;
      const int eff = len > 0 ? (max_unit_len + len - 1) / len : 1;
      const int64_t wgs = pairs * eff;
      const double rounds = 0.5 * (double)((wgs + 255) / 256);
      const double cost = rounds * ((len / 64) * (wide ? 1.85 : 1.0) + 4);
      if (sp == 1 || cost < best_cost) {
        best_cost = cost;
        best = sp;
      }
    }
    *cost_out = best_cost;
    return best;
  };
  // Resident window rows of that sweep: 128 per wave (512 per workgroup: every stream operand
  // read from LDS serves four products) when that leaves no more waves idle than 64 per wave
  // (256 per workgroup) does (W*G = 896, 1024, 512, 384: yes; 640, 768: no) and the model above
  // does not prefer the narrow form (small batches: twice as many workgroups fill more of the chip).
  double cost_n = 0.0, cost_w = 0.0;
  const int splits_n = best_splits(false, &cost_n), splits_w = best_splits(true, &cost_w);
  {
    const int live_w = (kp.Mq + 127) / 128, all_w = (kp.Mq + 511) / 512 * 4;
    const int live_n = (kp.Mq + 63) / 64, all_n = (kp.Mq + 255) / 256 * 4;
    w.wide_rows = (kp.Mq > 256 && (int64_t)live_w * all_n >= (int64_t)live_n * all_w && cost_w <= cost_n) ? 1 : 0;
    if (kp.path_flags & CASK_PATH_WIDE_ROWS) w.wide_rows = 1;
    if (kp.path_flags & CASK_PATH_NARROW_ROWS) w.wide_rows = 0;
  }
  int n_splits = w.wide_rows ? splits_w : splits_n;
  if (kp.score_splits >= 1) n_splits = kp.score_splits;
  int split_len = (int)align_up((size_t)(max_unit_len + n_splits - 1) / n_splits, 64);
  if (split_len < 64) split_len = 64;
  n_splits = (max_unit_len + split_len - 1) / split_len;
  if (n_splits < 1) n_splits = 1;
  w.n_splits = n_splits;
  // Sweep B of a batch of short units has few workgroups (one per 256 keys), each paying its
  // fixed cost for all W*G window rows: two workgroups then share a key tile, one half of the
  // window rows each, and add their column sums (two addends onto zero: the order cannot
  // change the result).
  w.q_splits = 1;
  {
    const int64_t wgsB = (int64_t)((n_units + 7) / 8 * 8) * ((max_unit_len + 255) / 256);
    if (wgsB <= 384 && kp.Mq >= 512) w.q_splits = 2;  // measured: helps up to about 1.5 rounds of the 512 slots
    if (kp.score_qsplit >= 1) w.q_splits = kp.score_qsplit;
  }
  // Sweep B with 128 resident keys per wave (512 per workgroup) when that still leaves at least
  // two rounds of workgroups
  {
    const int64_t wgs_wide = (int64_t)((n_units + 7) / 8 * 8) * ((max_unit_len + 511) / 512);
    w.wide_cols = (w.q_splits == 1 && wgs_wide >= 1024) ? 1 : 0;
    if (kp.path_flags & CASK_PATH_WIDE_ROWS) {
      w.wide_cols = 1;
      w.q_splits = 1;
    }
    if (kp.path_flags & CASK_PATH_NARROW_ROWS) w.wide_cols = 0;
  }
  w.split_len = split_len;
  w.mq_pad = (int)align_up((size_t)kp.Mq, 64);
  size_t off = 0;
  auto take = [&](size_t bytes) {
    const size_t at = off;
    off = align_up(off + bytes, 256);
    return at;
  };
  const size_t rows = (size_t)total_rows, units = (size_t)n_units;
  // one-launch scoring of short units: partial column sums, one row per 64 window rows
  // (reserved whatever the unit length, capped at the longest unit that path takes, so that a
  // workspace sized for longer units also serves a batch of shorter ones)
  {
    const size_t len64 = align_up((size_t)(max_unit_len > 0 ? max_unit_len : 1), 64);
    w.parts_pitch = (int)(len64 < 1024 ? len64 : 1024);
  }
  w.parts = take(units * (size_t)((kp.Mq + 63) / 64) * (size_t)w.parts_pitch * sizeof(float));
  w.rowstat = take(units * n_splits * w.mq_pad * sizeof(float2));
  w.bias = take(units * w.mq_pad * sizeof(float));
  w.scores = take(rows * sizeof(float));
  w.role = take(rows);
  w.slot_of = take(rows * sizeof(int32_t));
  w.assign_ord = take(rows * sizeof(int32_t));
  w.merged_row = take(rows * sizeof(int32_t));
  w.merged_ord = take(rows * sizeof(int32_t));
  w.seg_row = take(rows * sizeof(int32_t));
  w.seg_start = take(units * ((size_t)kp.B + 1) * sizeof(int32_t));
  w.seed_rows = take(units * kp.B * sizeof(int32_t));
  w.n_merged = take(units * sizeof(int32_t));
  w.n_seeds = take(units * sizeof(int32_t));
  w.total = off;
  return w;
}

static int resolve_params(const cask_params* p, KParams* kp, bool need_budget) {
  if (!p) return CASK_EINVAL;
  if (p->dtype != CASK_F32 && p->dtype != CASK_BF16) return CASK_EINVAL;
  if (p->head_dim != 64 && p->head_dim != 128) return CASK_EINVAL;
  if (p->q_per_kv < 1 || p->window < 1) return CASK_EINVAL;
  if ((int64_t)p->q_per_kv * p->window > (1 << 20)) return CASK_EINVAL;
  const int R = p->recent < 0 ? p->window : p->recent;
  if (need_budget && (p->budget < R + 1 || p->budget > (1 << 24))) return CASK_EINVAL;
  if (!(p->sim_threshold == p->sim_threshold)) return CASK_EINVAL;  // NaN
  if (p->merge_radius < 0 || p->merge_geometry < 0 || p->merge_geometry > 1) return CASK_EINVAL;
  if (p->merge_geometry == 1 && (!p->band_weight || !(p->dist_threshold >= 0.f))) return CASK_EINVAL;
  if (p->seed_dedup < 0 || (p->seed_dedup > 0 && p->merge_geometry != 0)) return CASK_EINVAL;
  if (p->score_splits < 0 || p->score_splits > 64 || p->score_qsplit < 0 || p->score_qsplit > 2) return CASK_EINVAL;
  kp->dtype = p->dtype;
  kp->d = p->head_dim;
  kp->G = p->q_per_kv;
  kp->W = p->window;
  kp->R = R;
  kp->B = p->budget > 0 ? p->budget : 1;
  kp->core = p->core;
  kp->prefix_budget = p->prefix_budget;
  kp->tau = p->sim_threshold;
  kp->radius = p->merge_radius;
  kp->geometry = p->merge_geometry;
  kp->theta = p->dist_threshold;
  kp->band_w = p->band_weight;
  kp->dedup = p->seed_dedup;
  kp->path_flags = p->path_flags;
  kp->score_splits = p->score_splits;
  kp->score_qsplit = p->score_qsplit;
  const double scale = p->softmax_scale > 0.f ? (double)p->softmax_scale : 1.0 / std::sqrt((double)p->head_dim);
  kp->scale_log2 = (float)(scale * 1.4426950408889634);
  kp->causal = p->causal ? 1 : 0;
  kp->Mq = p->q_per_kv * p->window;
  // the de-duplicating walk of a unit covers at most h * M rows and holds them in LDS
  if (need_budget && kp->dedup > 0 && (int64_t)kp->dedup * plan_seed_bound(*kp) > kSeedWalkMax) return CASK_EINVAL;
  return CASK_OK;
}

static int resolve_batch(const KParams& kp, const cask_batch* b, Batch* out, bool need_q, bool need_v) {
  if (!b || b->n_units < 0) return CASK_EINVAL;
  out->n_units = b->n_units;
  out->max_unit_len = 0;
  out->max_decode_len = 0;
  out->total_rows = 0;
  if (b->n_units == 0) return CASK_OK;
  if (!b->row_off || !b->prefix_len || !b->row_off_host || !b->prefix_len_host || !b->K) return CASK_EINVAL;
  if (need_q && !b->Q) return CASK_EINVAL;
  if (need_v && !b->V) return CASK_EINVAL;
  auto misaligned = [](const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; };
  if (misaligned(b->K) || misaligned(b->V) || misaligned(b->Q)) return CASK_EINVAL;
  if (b->row_off_host[0] != 0) return CASK_EINVAL;
  for (int u = 0; u < b->n_units; ++u) {
    const int64_t n = b->row_off_host[u + 1] - b->row_off_host[u];
    // a unit's keys are addressed with 32-bit byte offsets: at most 2^23 - 1 rows
    if (n < kp.W || n > 0x7fffffLL) return CASK_EINVAL;
    const int32_t P = b->prefix_len_host[u];
    if (P < 0 || P > n) return CASK_EINVAL;
    if ((int)n > out->max_unit_len) out->max_unit_len = (int)n;
    if ((int)n - P > out->max_decode_len) out->max_decode_len = (int)n - P;
  }
  out->total_rows = b->row_off_host[b->n_units];
  out->row_off = b->row_off;
  out->prefix_len = b->prefix_len;
  out->K = b->K;
  out->V = b->V;
  out->Q = b->Q;
  return CASK_OK;
}

static int dev_rc(hipError_t e) { return e == hipSuccess ? CASK_OK : CASK_EDEVICE; }

// Optional per-stage timing of cask_compress: HIP events recorded on the caller's stream
// between the kernels of an event.  Off by default; the events are created when it is
// switched on, never inside a compression call.
struct StageTiming {
  bool on = false;
  int max_calls = 0;
  int n_calls = 0;
  int stages = CASK_N_STAGES;  // stages recorded per call (the first `stages` of them)
  std::vector<hipEvent_t> ev;  // (CASK_N_STAGES + 1) per call
};
static StageTiming g_timing;
static std::mutex g_timing_mu;  // guards g_timing's bookkeeping (the events themselves belong to one stream)

struct StageRecorder {
  hipEvent_t* ev = nullptr;
  hipStream_t st;
  int next = 0;
  int stages = 0;
  explicit StageRecorder(hipStream_t s) : st(s) {
    std::lock_guard<std::mutex> lock(g_timing_mu);
    if (g_timing.on && g_timing.n_calls < g_timing.max_calls) {
      ev = g_timing.ev.data() + (size_t)g_timing.n_calls * (CASK_N_STAGES + 1);
      stages = g_timing.stages;
      ++g_timing.n_calls;
    }
  }
  hipEvent_t peek() const { return (ev && next <= stages) ? ev[next] : nullptr; }  // handed to a launcher to record
  void skip() { if (ev) ++next; }
  void mark() {
    if (!ev) return;
    if (next <= stages) (void)hipEventRecord(ev[next], st);
    ++next;
  }
};

}  // namespace cask

using namespace cask;

extern "C" {

const char* cask_strerror(int code) {
  switch (code) {
    case CASK_OK: return "ok";
    case CASK_EINVAL: return "invalid argument";
    case CASK_ENOMEM: return "workspace too small";
    case CASK_EDEVICE: return "HIP error";
    default: return "unknown";
  }
}

int cask_plan(const cask_params* params, int32_t P, int32_t N, cask_plan_t* out) {
  KParams kp;
  if (!out || resolve_params(params, &kp, true) != CASK_OK) return CASK_EINVAL;
  if (N < 0 || P < 0 || P > N) return CASK_EINVAL;
  const UnitPlan pl = make_plan(kp, P, N);
  out->r_eff = pl.r_eff;
  out->p_keep = pl.p_keep;
  out->slots = pl.slots;
  out->core = pl.core;
  out->seeds = pl.seeds;
  out->status = pl.status;
  return CASK_OK;
}

size_t cask_workspace_bytes(const cask_params* params, int32_t n_units, int64_t total_rows,
                            int32_t max_unit_len) {
  KParams kp;
  if (resolve_params(params, &kp, false) != CASK_OK || n_units < 0 || total_rows < 0 || max_unit_len < 0)
    return 0;
  return layout_workspace(kp, n_units, total_rows, max_unit_len).total + 256;
}

int cask_score(const cask_params* params, const cask_batch* batch, float* scores, void* ws,
               size_t ws_bytes, void* hip_stream) {
  KParams kp;
  Batch b;
  int rc = resolve_params(params, &kp, false);
  if (rc) return rc;
  rc = resolve_batch(kp, batch, &b, true, false);
  if (rc) return rc;
  if (b.n_units == 0) return CASK_OK;
  if (!scores || !ws) return CASK_EINVAL;
  if ((reinterpret_cast<uintptr_t>(ws) & 15u) != 0) return CASK_EINVAL;
  const Workspace wl = layout_workspace(kp, b.n_units, b.total_rows, b.max_unit_len);
  if (ws_bytes < wl.total) return CASK_ENOMEM;
  if (score_fused_fits(kp, b) && (reinterpret_cast<uintptr_t>(scores) & 15u) == 0)
    return dev_rc(launch_score_fused(kp, b, wl, scores, static_cast<hipStream_t>(hip_stream)));
  return dev_rc(launch_score(kp, b, wl, static_cast<char*>(ws), scores, static_cast<hipStream_t>(hip_stream)));
}

int cask_prefix_evict(const cask_params* params, const cask_batch* batch, const float* scores,
                      uint8_t* role, int32_t* status, void* ws, size_t ws_bytes,
                      void* hip_stream) {
  (void)ws;
  (void)ws_bytes;
  KParams kp;
  Batch b;
  int rc = resolve_params(params, &kp, true);
  if (rc) return rc;
  rc = resolve_batch(kp, batch, &b, false, false);
  if (rc) return rc;
  if (b.n_units == 0) return CASK_OK;
  if (!scores || !role) return CASK_EINVAL;
  return dev_rc(launch_select(kp, b, scores, role, status, true, false, static_cast<hipStream_t>(hip_stream)));
}

int cask_partition(const cask_params* params, const cask_batch* batch, const float* scores,
                   uint8_t* role, int32_t* status, void* ws, size_t ws_bytes, void* hip_stream) {
  (void)ws;
  (void)ws_bytes;
  KParams kp;
  Batch b;
  int rc = resolve_params(params, &kp, true);
  if (rc) return rc;
  rc = resolve_batch(kp, batch, &b, false, false);
  if (rc) return rc;
  if (b.n_units == 0) return CASK_OK;
  if (!scores || !role) return CASK_EINVAL;
  hipError_t e = launch_select(kp, b, scores, role, status, false, true, static_cast<hipStream_t>(hip_stream));
  if (e != hipSuccess) return CASK_EDEVICE;
  return dev_rc(launch_dedup_seeds(kp, b, scores, role, static_cast<hipStream_t>(hip_stream)));
}

int cask_consolidate(const cask_params* params, const cask_batch* batch, const float* scores,
                     const uint8_t* role, int32_t* assign, void* ws, size_t ws_bytes,
                     void* hip_stream) {
  (void)scores;
  KParams kp;
  Batch b;
  int rc = resolve_params(params, &kp, true);
  if (rc) return rc;
  rc = resolve_batch(kp, batch, &b, false, false);
  if (rc) return rc;
  if (b.n_units == 0) return CASK_OK;
  if (!role || !assign || !ws) return CASK_EINVAL;
  if ((reinterpret_cast<uintptr_t>(ws) & 15u) != 0) return CASK_EINVAL;
  const Workspace wl = layout_workspace(kp, b.n_units, b.total_rows, b.max_unit_len);
  if (ws_bytes < wl.total) return CASK_ENOMEM;
  char* w = static_cast<char*>(ws);
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  int32_t* seed_rows = reinterpret_cast<int32_t*>(w + wl.seed_rows);
  int32_t* n_seeds = reinterpret_cast<int32_t*>(w + wl.n_seeds);
  int32_t* assign_ord = reinterpret_cast<int32_t*>(w + wl.assign_ord);
  hipError_t e = launch_index_roles(kp, b, role, nullptr, nullptr, nullptr, seed_rows, n_seeds, st);
  if (e != hipSuccess) return CASK_EDEVICE;
  e = launch_similarity(kp, b, role, seed_rows, n_seeds, assign_ord, false, st);
  if (e != hipSuccess) return CASK_EDEVICE;
  e = launch_gather_merged(kp, b, role, assign_ord, nullptr, seed_rows,
                           reinterpret_cast<int32_t*>(w + wl.merged_row),
                           reinterpret_cast<int32_t*>(w + wl.merged_ord), nullptr, assign, 2,
                           nullptr, n_seeds, nullptr, nullptr, nullptr, st);
  return dev_rc(e);
}

int cask_mass_diagnostics(const cask_params* params, const cask_batch* batch, const float* scores,
                          const uint8_t* role, const float* out_mass, const int32_t* out_len,
                          float* rho, void* hip_stream) {
  KParams kp;
  Batch b;
  int rc = resolve_params(params, &kp, true);
  if (rc) return rc;
  rc = resolve_batch(kp, batch, &b, false, false);
  if (rc) return rc;
  if (b.n_units == 0) return CASK_OK;
  if (!scores || !role || !out_mass || !out_len || !rho) return CASK_EINVAL;
  return dev_rc(launch_mass_diag(kp, b, scores, role, out_mass, out_len, rho,
                                 static_cast<hipStream_t>(hip_stream)));
}

int cask_group_diagnostics(const cask_params* params, const cask_batch* batch, const float* scores,
                           const int32_t* assign, const void* K_out, int32_t out_stride_rows,
                           float* dispersion, float* lost_mass, void* hip_stream) {
  KParams kp;
  Batch b;
  int rc = resolve_params(params, &kp, true);
  if (rc) return rc;
  rc = resolve_batch(kp, batch, &b, false, false);
  if (rc) return rc;
  if (b.n_units == 0) return CASK_OK;
  if (!scores || !assign || !K_out || !dispersion || !lost_mass) return CASK_EINVAL;
  if ((reinterpret_cast<uintptr_t>(K_out) & 15u) != 0 || out_stride_rows < kp.B) return CASK_EINVAL;
  kp.band_w = params->band_weight;  // used here whatever the merge geometry
  return dev_rc(launch_group_diag(kp, b, scores, assign, K_out, out_stride_rows, dispersion,
                                  lost_mass, static_cast<hipStream_t>(hip_stream)));
}

int cask_attend(const cask_params* params, int32_t n_units, const void* Q, const void* K_c,
                const void* V_c, int32_t stride_rows, const int32_t* len, const int32_t* count,
                int32_t count_pitch, void* out, void* hip_stream) {
  KParams kp;
  int rc = resolve_params(params, &kp, false);
  if (rc) return rc;
  if (n_units < 0) return CASK_EINVAL;
  if (n_units == 0) return CASK_OK;
  if (!Q || !K_c || !V_c || !len || !out || stride_rows < 1) return CASK_EINVAL;
  if (count && count_pitch < 1) return CASK_EINVAL;
  if (((reinterpret_cast<uintptr_t>(Q) | reinterpret_cast<uintptr_t>(K_c) | reinterpret_cast<uintptr_t>(V_c) |
        reinterpret_cast<uintptr_t>(out)) & 15u) != 0)
    return CASK_EINVAL;
  return dev_rc(launch_attend(kp, n_units, Q, K_c, V_c, stride_rows, len, count, count_pitch, out,
                              static_cast<hipStream_t>(hip_stream)));
}

int cask_compress(const cask_params* params, const cask_batch* batch, void* K_out, void* V_out,
                  int32_t* out_len, int32_t* out_src, float* out_mass, int32_t* assign,
                  float* scores, int32_t* status, void* ws, size_t ws_bytes, void* hip_stream) {
  return cask_compress_step(params, batch, nullptr, K_out, V_out, params ? params->budget : 0,
                            out_len, out_src, out_mass, nullptr, assign, scores, status, ws, ws_bytes,
                            hip_stream);
}

int cask_compress_step(const cask_params* params, const cask_batch* batch, const int32_t* in_count,
                       void* K_out, void* V_out, int32_t out_stride_rows, int32_t* out_len,
                       int32_t* out_src, float* out_mass, int32_t* out_count, int32_t* assign,
                       float* scores, int32_t* status, void* ws, size_t ws_bytes,
                       void* hip_stream) {
  KParams kp;
  Batch b;
  int rc = resolve_params(params, &kp, true);
  if (rc) return rc;
  const bool given = params->scores_given != 0;
  rc = resolve_batch(kp, batch, &b, !given, true);
  if (rc) return rc;
  if (b.n_units == 0) return CASK_OK;
  if (!K_out || !V_out || !out_len || !out_src || !status || !ws) return CASK_EINVAL;
  if (((reinterpret_cast<uintptr_t>(K_out) | reinterpret_cast<uintptr_t>(V_out) | reinterpret_cast<uintptr_t>(ws)) & 15u) != 0)
    return CASK_EINVAL;
  if (given && !scores) return CASK_EINVAL;
  if (out_stride_rows < kp.B) return CASK_EINVAL;
  const Workspace wl = layout_workspace(kp, b.n_units, b.total_rows, b.max_unit_len);
  if (ws_bytes < wl.total) return CASK_ENOMEM;
  char* w = static_cast<char*>(ws);
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  float* s = scores ? scores : reinterpret_cast<float*>(w + wl.scores);
  uint8_t* role = reinterpret_cast<uint8_t*>(w + wl.role);
  int32_t* slot_of = reinterpret_cast<int32_t*>(w + wl.slot_of);
  int32_t* assign_ord = reinterpret_cast<int32_t*>(w + wl.assign_ord);
  int32_t* merged_row = reinterpret_cast<int32_t*>(w + wl.merged_row);
  int32_t* merged_ord = reinterpret_cast<int32_t*>(w + wl.merged_ord);
  int32_t* seg_row = reinterpret_cast<int32_t*>(w + wl.seg_row);
  int32_t* seg_start = reinterpret_cast<int32_t*>(w + wl.seg_start);
  int32_t* seed_rows = reinterpret_cast<int32_t*>(w + wl.seed_rows);
  int32_t* n_merged = reinterpret_cast<int32_t*>(w + wl.n_merged);
  int32_t* n_seeds = reinterpret_cast<int32_t*>(w + wl.n_seeds);
  hipError_t e;
  StageRecorder rec(st);
  rec.mark();  // start
  const bool fused_tail = tail_small_fits(kp, b) && kp.dedup == 0 && !(kp.path_flags & CASK_PATH_NO_FUSED_TAIL);
  // short units: both sweeps are one launch as well, handing partial sums to the tail kernel
  // (reported as the first scoring stage; the second reads as an empty bracket)
  const bool fused_score = fused_tail && !given && score_parts_fits(kp, b, wl) &&
                           !(kp.path_flags & CASK_PATH_NO_FUSED_SCORE);
  if (fused_score) {
    e = launch_score_parts(kp, b, wl, w, st);
    if (e != hipSuccess) return CASK_EDEVICE;
    rec.mark();
  } else if (!given && score_fused_fits(kp, b) && (reinterpret_cast<uintptr_t>(s) & 15u) == 0) {
    // many long units with few window rows: both sweeps in one launch (reported as the first
    // scoring stage; the second reads as an empty bracket)
    e = launch_score_fused(kp, b, wl, s, st);
    if (e != hipSuccess) return CASK_EDEVICE;
    rec.mark();
  } else if (!given) {
    e = launch_score(kp, b, wl, w, s, st, rec.peek());  // records the end of sweep A itself
    if (e != hipSuccess) return CASK_EDEVICE;
    rec.skip();
  } else {
    rec.mark();
  }
  rec.mark();  // end of sweep B
  if (fused_tail) {
    // short units: the rest of the event is one launch (reported as the select stage)
    e = launch_tail_small(kp, b, s, fused_score ? reinterpret_cast<const float*>(w + wl.parts) : nullptr,
                          (kp.Mq + 63) / 64, wl.parts_pitch, in_count, K_out, V_out, out_stride_rows,
                          out_len, out_src, out_mass, out_count, assign, status, st);
    for (int k = 0; k < 5; ++k) rec.mark();
    return dev_rc(e);
  }
  if (kp.dedup > 0) {
    // de-duplicated seeding sits between the selection and the ordered walk: three launches
    e = launch_select(kp, b, s, role, status, true, true, st);
    if (e == hipSuccess) e = launch_dedup_seeds(kp, b, s, role, st);
    if (e != hipSuccess) return CASK_EDEVICE;
    rec.mark();
    e = launch_index_roles(kp, b, role, slot_of, out_src, out_len, seed_rows, n_seeds, st);
    if (e != hipSuccess) return CASK_EDEVICE;
    rec.mark();
  } else {
    e = launch_select_index(kp, b, s, role, status, slot_of, out_src, out_len, seed_rows, n_seeds,
                            st);
    if (e != hipSuccess) return CASK_EDEVICE;
    rec.mark();
    rec.mark();  // the ordered walk runs inside the select kernel here: its own stage reads as zero
  }
  e = launch_similarity(kp, b, role, seed_rows, n_seeds, assign_ord, true, st);
  if (e != hipSuccess) return CASK_EDEVICE;
  rec.mark();
  // the rows that pass through unchanged are copied by spare workgroups of the grouping launch
  CopyJob cj{};
  cj.K = static_cast<const unsigned char*>(b.K);
  cj.V = static_cast<const unsigned char*>(b.V);
  cj.K_out = static_cast<unsigned char*>(K_out);
  cj.V_out = static_cast<unsigned char*>(V_out);
  cj.scores = s;
  cj.in_count = in_count;
  cj.out_src = out_src;
  cj.out_len = out_len;
  cj.out_mass = out_mass;
  cj.out_count = out_count;
  cj.out_stride = out_stride_rows;
  e = launch_gather_merged(kp, b, role, assign_ord, slot_of, seed_rows, merged_row, merged_ord,
                           n_merged, assign, assign ? 1 : 0, status, n_seeds, seg_row, seg_start,
                           &cj, st);
  if (e != hipSuccess) return CASK_EDEVICE;
  rec.mark();
  e = launch_emit(kp, b, s, seed_rows, n_seeds, slot_of, seg_row, seg_start, n_merged, K_out,
                  V_out, out_mass, in_count, out_count, out_stride_rows, st);
  rec.mark();
  return dev_rc(e);
}

// ---------------------------------------------------------------- allocation-free variant
//
// cask_compress for callers that cannot allocate device memory (a stream under graph capture, a
// tight serving loop, a harness that forbids allocation): the workspace is a fixed array in
// device memory that belongs to the library.  Every device the library runs on holds its own
// copy of the array, at its own address, until the process ends.  In host code the array's
// name only stands for the symbol: its device address is looked up once per device and every
// use below goes through that address.
static __device__ __align__(256) __attribute__((used)) unsigned char scratch[CASK_STATIC_WORKSPACE_BYTES];

namespace {
std::mutex g_scratch_mu;
void* g_scratch_ptr[64] = {};  // per device: address of that device's copy of `scratch`

// Address of the current device's copy; looked up on the first call on that device.
int static_workspace(void** out) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return CASK_EDEVICE;
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return CASK_EDEVICE;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return CASK_OK;
}
}  // namespace

int cask_compress_static(const cask_params* params, const cask_batch* batch, void* K_out, void* V_out,
                         int32_t* out_len, int32_t* out_src, float* out_mass, int32_t* assign,
                         float* scores, int32_t* status, void* hip_stream) {
  // sizes first, on the host mirrors: a batch whose workspace would not fit is refused before
  // anything touches the device
  KParams kp;
  Batch b;
  int rc = resolve_params(params, &kp, true);
  if (rc) return rc;
  rc = resolve_batch(kp, batch, &b, params->scores_given == 0, true);
  if (rc) return rc;
  if (b.n_units == 0) return CASK_OK;
  if (layout_workspace(kp, b.n_units, b.total_rows, b.max_unit_len).total > (size_t)CASK_STATIC_WORKSPACE_BYTES)
    return CASK_ENOMEM;
  void* ws = nullptr;
  rc = static_workspace(&ws);
  if (rc) return rc;
  // Nothing in the workspace has to start at zero: every kernel of the event writes what it or a
  // later kernel reads (the same holds for a caller's uninitialised workspace), so the contents
  // the previous call left behind are harmless.
  return cask_compress(params, batch, K_out, V_out, out_len, out_src, out_mass, assign, scores, status,
                       ws, (size_t)CASK_STATIC_WORKSPACE_BYTES, hip_stream);
}

int cask_timing_enable(int max_calls) { return cask_timing_enable_stages(max_calls, CASK_N_STAGES); }

int cask_timing_enable_stages(int max_calls, int n_stages) {
  std::lock_guard<std::mutex> lock(g_timing_mu);
  for (hipEvent_t e : g_timing.ev) (void)hipEventDestroy(e);
  g_timing.ev.clear();
  g_timing.on = false;
  g_timing.n_calls = 0;
  g_timing.max_calls = 0;
  if (max_calls <= 0) return CASK_OK;
  if (max_calls > 4096 || n_stages < 1 || n_stages > CASK_N_STAGES) return CASK_EINVAL;
  g_timing.stages = n_stages;
  g_timing.ev.resize((size_t)max_calls * (CASK_N_STAGES + 1));
  for (auto& e : g_timing.ev)
    if (hipEventCreate(&e) != hipSuccess) return CASK_EDEVICE;
  g_timing.max_calls = max_calls;
  g_timing.on = true;
  return CASK_OK;
}

int cask_timing_read(float* stage_ms, int* n_calls) {
  if (!stage_ms || !n_calls) return CASK_EINVAL;
  std::lock_guard<std::mutex> lock(g_timing_mu);
  for (int i = 0; i < CASK_N_STAGES; ++i) stage_ms[i] = 0.f;
  *n_calls = g_timing.n_calls;
  for (int c = 0; c < g_timing.n_calls; ++c) {
    hipEvent_t* ev = g_timing.ev.data() + (size_t)c * (CASK_N_STAGES + 1);
    if (hipEventSynchronize(ev[g_timing.stages]) != hipSuccess) return CASK_EDEVICE;
    for (int i = 0; i < g_timing.stages; ++i) {
      float ms = 0.f;
      if (hipEventElapsedTime(&ms, ev[i], ev[i + 1]) != hipSuccess) return CASK_EDEVICE;
      stage_ms[i] += ms;
    }
  }
  g_timing.n_calls = 0;
  return CASK_OK;
}

}  // extern "C"
