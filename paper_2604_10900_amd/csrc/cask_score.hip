// Scoring: s_j = mean over the W*G window rows of softmax_j(scale <q, k_j>), the scalar
// importance used as local score mass a_i (Sections 1 and 2.4 of the paper).
//
// The softmax normaliser of a row needs all keys before any column can be summed, so the
// score takes two sweeps of Q.K^T:
//   sweep A (row statistics)  per window row and key split: a reference logit and the sum of
//                             exp2 against it (pairs of splits combine exactly);
//   sweep B (column mass)     per key: sum over window rows of exp2(logit - L_row).
// Logits are never stored: recomputing the contraction on the matrix cores is cheaper than
// writing and re-reading a W*G x N fp32 matrix through HBM.
//
// bf16, d = 128: both sweeps use one MFMA kernel (32x32x16 bf16 tiles, fp32 accumulation).
// One operand ("resident") stays in registers for the whole loop, the other ("stream") is
// staged through LDS.  The product tile is stream x resident^T, so each lane owns ONE
// resident column and 16 stream rows: the reduction over the stream dimension (keys in
// sweep A, window rows in sweep B) stays inside a lane until the very end.
// Other dtypes/head sizes take a plain FMA kernel with the same two-sweep structure.
#include "cask_common.h"

namespace cask {

namespace {

constexpr float kNegInf = -__builtin_inff();

__device__ inline float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// (m, l) <- combination of two partial softmax statistics in base-2 units
__device__ inline void ml_combine(float& m, float& l, float m2, float l2) {
  const float M = fmaxf(m, m2);
  const float a = (m == kNegInf) ? 0.f : fast_exp2(m - M);
  const float b = (m2 == kNegInf) ? 0.f : fast_exp2(m2 - M);
  l = l * a + l2 * b;
  m = M;
}

// -L_row (base-2) of every window row from the per-split partials; -inf for padding rows.
// Fills negL[0, n_fill); rows >= Mq get -inf.  `pitch` is the row pitch of the partials.
__device__ inline void fill_neg_lse(const float2* __restrict__ part, int n_splits, int n_fill,
                                    int Mq, float* negL, int tid, int nthreads, int pitch) {
  for (int r = tid; r < n_fill; r += nthreads) {
    float v = kNegInf;
    if (r < Mq) {
      float m = kNegInf, l = 0.f;
      for (int s = 0; s < n_splits; ++s) {
        const float2 p = part[(size_t)s * pitch + r];
        ml_combine(m, l, p.x, p.y);
      }
      v = -(m + log2f(l));
    }
    negL[r] = v;
  }
}

// XCD-aware block -> (unit, tile): consecutive workgroups go round-robin over the 8 XCDs, so
// unit u is pinned to XCD (u % 8) and its tiles are consecutive on that XCD: the unit's K
// (sweep A) or Q (sweep B) stays in one L2 while its tiles run.
__device__ inline bool map_block(int n_units, int tiles_per_unit, int& unit, int& tile) {
  const int bid = blockIdx.x;
  const int xcd = bid & 7;
  const int k = bid >> 3;
  unit = (k / tiles_per_unit) * 8 + xcd;
  tile = k % tiles_per_unit;
  return unit < n_units;
}

// ------------------------------------------------------------------ MFMA path (bf16, d=128)

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kD = 128;
constexpr int kRowBytes = kD * 2;
constexpr int kWaves = 4;                    // waves per workgroup, 1 per SIMD; two workgroups share a CU
constexpr int kThreads = kWaves * 64;
constexpr int kResRows = kWaves * 64;        // resident rows per workgroup (64 per wave)
constexpr int kStageRows = 64;               // stream rows per ring slot
constexpr int kGroupPitch = 1024 + 64;       // LDS pitch of a 4-row group (see stage layout)
constexpr int kDataBytes = (kStageRows / 4) * kGroupPitch;
constexpr int kStageBytes = kDataBytes + kStageRows * 4;   // + one float per row: -L_row (sweep B)
constexpr int kDepth = 4;                    // ring slots: loads run kDepth - 1 stages ahead
constexpr int kLoadsPerThread = kStageRows * 16 / kThreads;  // 16-byte pieces per thread per stage

// Pad value of -L for window rows past W*G: far enough down that exp2 flushes to zero.
constexpr float kPadNegL = -1.0e30f;

// Per window row of a unit: -L_row, L_row the base-2 log-sum-exp combined over the key splits
// of sweep A.  Sweep B adds it to every logit of the row inside the exponent's fma.
constexpr int kBiasThreads = 1024;  // a thread per window row at W*G <= 1024: every partial of the unit in flight at once
__global__ __launch_bounds__(kBiasThreads) void score_bias_kernel(KParams kp, int n_splits, int mq_pad,
                                                         const float2* __restrict__ rowstat,
                                                         float* __restrict__ bias) {
  const int unit = blockIdx.x;
  const float2* part = rowstat + (size_t)unit * n_splits * mq_pad;
  for (int r = threadIdx.x; r < mq_pad; r += kBiasThreads) {
    float nl = kPadNegL;
    if (r < kp.Mq) {
      float m = kNegInf, l = 0.f;
      for (int s0 = 0; s0 < n_splits; s0 += 8) {  // eight partials in flight, combined in order
        float2 pr[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) pr[e] = part[(size_t)min(s0 + e, n_splits - 1) * mq_pad + r];
#pragma unroll
        for (int e = 0; e < 8; ++e)
          if (s0 + e < n_splits) ml_combine(m, l, pr[e].x, pr[e].y);
      }
      nl = -(m + log2f(l));
    }
    bias[(size_t)unit * mq_pad + r] = nl;
  }
}

// Both scoring sweeps.  MODE 0 = sweep A (resident: window rows, stream: keys),
// MODE 1 = sweep B (resident: keys, stream: window rows).
//
// Workgroup: 4 waves, one per SIMD, and two workgroups per compute unit, so a SIMD always has a
// second wave from an independent workgroup to run while the first sits in its prologue or at
// a barrier.  Wave w keeps CT resident tiles of 32 rows (rows [32 CT w, 32 CT (w + 1)) of the
// workgroup's 128 CT) as MFMA B-operands in registers: CT = 2 in the narrow form, CT = 4 in the
// wide form that the two separate sweeps take where the shape fills such blocks (every stream
// operand read from LDS then serves four products instead of two; see pipelined_wide below).
// Stream rows arrive 64 at a time in a ring of LDS slots,
// written by direct global->LDS loads (no register staging, no LDS stores) that run
// kDepth - 1 stages ahead of the stage being consumed; one barrier per stage both publishes a
// slot and frees the one consumed before it.
//
// Stage layout in LDS: each load instruction of a wave lands 1 KB = four 256-byte rows; lane s
// fetches 16-byte piece s / 4 of row s % 4, so the group holds piece-major data
// (piece g of row r at g * 64 + r * 16).  A wave reading A-operands (lane = row) then touches
// 16 consecutive bytes per row and groups 1088 bytes apart: conflict-free, and the eight
// k-steps are plain immediate offsets (128 bytes apart).
//
// Per stage a wave runs 2 CT tiles of 32x32, (rt0,ct0) ... (rt0,ct CT-1) (rt1,ct0) ...,
// software-pipelined: the MFMA chain of a tile is issued interleaved, two logits per MFMA, with
// the exp2 epilogue of the tile before it, so the matrix cores and the vector ALU of a wave
// run at the same time; the epilogue of a stage's last tile rides on the next stage's first
// chain.  The epilogue is exactly three vector instructions per logit:
//   sweep A  fma, exp2, add: no running maximum in the loop -- exp2 is taken against a per-lane
//            reference (the first logit of the lane's row), which is exact as long as the sum
//            stays finite, because (reference, sum) pairs combine exactly.  A sum that left the
//            fp32 range (a logit more than ~128 binary orders above the reference) shows as
//            inf at the end; the wave then recomputes its share with a true running maximum,
//            operands straight from memory (rare, slow, exact);
//   sweep B  fma, exp2, add: the fma adds -L_row, read from LDS next to the stage's rows (a lane's
//            16 rows of a tile are four float4 reads).
// Stages that touch masked entries (causal tail, ragged end, keys inside the window) run the same
// pipeline with two more instructions per logit (a compare of the logit's constant row offset
// with a per-lane limit, a select); only a sweep-A workgroup without a single clean stage, which
// has no reference logit yet, takes a plain unpipelined path with a true running maximum.
template <int MODE, int CT = 2, bool RING_RES = false>
__global__ __launch_bounds__(kThreads, 2) void score_mfma_kernel(
    KParams kp, int n_units, int tiles_per_unit, int n_splits, int split_len, int q_splits, int mq_pad,
    const int64_t* __restrict__ row_off, const uint16_t* __restrict__ K,
    const uint16_t* __restrict__ Q, float2* __restrict__ rowstat,
    const float* __restrict__ bias, float* __restrict__ bias_out, float* __restrict__ scores,
    float* __restrict__ parts, int part_pitch) {
  constexpr int NK = 8;  // k-steps per tile
  // MODE 2 = both sweeps in one launch for short units (one key split): the first pass is
  // MODE 0; the second keeps the same resident window rows and streams the keys again, leaving
  // one partial column sum per wave.  MODE 3 = the same for units of any length when W*G <= 512
  // (at most two row blocks per unit): the four waves' column sums are added in LDS in wave
  // order and leave the workgroup as one addend per key -- stored when the unit has one row
  // block, added atomically onto scores cleared beforehand when it has two (two addends onto
  // zero: the order cannot change the bits).
  // CT = resident 32-row tiles per wave: 2 (64 rows a wave, 256 a workgroup) or 4 (128 / 512:
  // every stream operand read from LDS then serves four products instead of two)
  constexpr int kWaveRows = CT * 32;
  constexpr int kResRowsT = kWaves * kWaveRows;
  // RING_RES: the resident rows come through the ring as well, in kResStages ring stages ahead
  // of the stream (else they are loaded straight into registers and the ring starts with the stream)
  constexpr int kResStages = RING_RES ? kResRowsT / kStageRows : 0;
  constexpr bool kRowPass = MODE != 1;
  constexpr bool kTwoPass = MODE >= 2;
  constexpr bool kWgReduce = MODE == 3;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  unsigned char* ring = smem;

  int unit, tile;
  if (!map_block(n_units, tiles_per_unit, unit, tile)) return;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int c32 = lane & 31, h = lane >> 5;
  const int64_t row0 = row_off[unit];
  const int N = (int)(row_off[unit + 1] - row0);
  const int Mq = kp.Mq, W = kp.W, Gq = kp.G;
  const float c = kp.scale_log2;
  const uint16_t* Ku = K + (size_t)row0 * kD;
  const uint16_t* Qu = Q + (size_t)unit * Mq * kD;

  // ---- what this workgroup covers
  const uint16_t* res_ptr;
  const uint16_t* str_ptr;
  int res_base, res_limit, s_begin, s_end;  // resident rows [res_base, ..), stream rows [s_begin, s_end)
  int split = 0;
  if (kRowPass) {
    const int qb = tile / n_splits;
    split = tile % n_splits;
    res_base = qb * kResRowsT;
    if (res_base >= Mq) return;
    res_ptr = Qu;
    res_limit = Mq;
    str_ptr = Ku;
    s_begin = split * split_len;
    s_end = min(N, s_begin + split_len);
    if (kp.causal) {  // (MODE 2: the keys cut here get zeros as their partial sums at the end)
      const int last_row = min(Mq, res_base + kResRowsT) - 1;
      s_end = min(s_end, N - W + last_row / Gq + 1);
    }
  } else {
    // a unit's last tile first: its waves run the masked path and take longest
    const int key_tiles = tiles_per_unit / q_splits;
    res_base = (key_tiles - 1 - tile / q_splits) * kResRowsT;
    if (res_base >= N) return;
    res_ptr = Ku;
    res_limit = N;
    str_ptr = Qu;
    s_begin = 0;
    s_end = Mq;
    if (q_splits == 2) {  // this workgroup's half of the window rows, whole stages
      const int half = ((Mq + 2 * kStageRows - 1) / (2 * kStageRows)) * kStageRows;
      if (tile & 1) s_begin = half; else s_end = min(Mq, half);
    }
    if (kp.causal && res_base > N - W)
      s_begin = max(s_begin, (((res_base - (N - W)) * Gq) / kStageRows) * kStageRows);
  }
  const int n_stages = s_end > s_begin ? (s_end - s_begin + kStageRows - 1) / kStageRows : 0;
  if (MODE == 0 && q_splits == 2 && tile == 0) {
    // sweep B will add two partial sums per key: clear the unit's scores here
    for (int i = tid; i < N; i += kThreads) scores[row0 + i] = 0.f;
  }

  // ---- ring loads: thread t, piece j covers 16-byte LDS slot t + kThreads * j of the stage:
  //      row = 4 * (slot / 64) + slot % 4, 16-byte piece = (slot % 64) / 4
  const __amdgpu_buffer_rsrc_t rsrc =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(str_ptr), 0,
                                        max(s_end, 0) * kRowBytes, 0x00020000);
  // (load j of a wave fills 4-row group wv + kWaves * j: the same lane offset, 4 * kWaves rows on)
  const int ld_voff = (wv * 4 + (lane & 3)) * kRowBytes + (lane >> 2) * 16;
  // sweep B: the -L_row of a stage's 64 rows is one more 256-byte load, taken in turn by the
  // waves (stage % kWaves), so every wave has at most one extra load in flight
  const __amdgpu_buffer_rsrc_t brsrc = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<float*>(bias + (size_t)unit * mq_pad), 0, mq_pad * 4, 0x00020000);
  // RING_RES: ring stages [0, kResStages) hold resident rows [res_base + 64 s, ...), each read out
  // of LDS by the wave that owns those rows; ring stage kResStages + s is stream stage s.  Loaded
  // straight into registers, a lane per row, every load instruction touches 32 rows at 32 bytes
  // each: a workgroup of the wide sweep B spends 8 us on its resident keys.  Through the ring the
  // loads are whole rows, but the stream waits behind them: it pays where workgroups are short
  // (W*G <= 512: eight stream stages in sweep B) and costs elsewhere (measured both ways).
  const __amdgpu_buffer_rsrc_t res_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint16_t*>(res_ptr), 0, res_limit * kRowBytes, 0x00020000);
  // (two functions, and the resident phase below unrolled: where one call site could take
  // either descriptor the compiler kept both in scratch memory and fetched one per call)
  auto issue_resident = [&](int stage) {  // rows past the end read as zero through the descriptor
    unsigned char* slot = ring + (stage % kDepth) * kStageBytes;
    const int roff = (res_base + stage * kStageRows) * kRowBytes;
#pragma unroll
    for (int j = 0; j < kLoadsPerThread; ++j) {
      const int grp = wv + kWaves * j;
      __builtin_amdgcn_raw_ptr_buffer_load_lds(
          res_rsrc, (__attribute__((address_space(3))) void*)(slot + grp * kGroupPitch),
          16, ld_voff, roff + j * (4 * kWaves * kRowBytes), 0, 0);
    }
  };
  auto issue_stage = [&](int stage) {  // ring stage >= kResStages; rows past s_end read as zero
    unsigned char* slot = ring + (stage % kDepth) * kStageBytes;
    const int sstage = stage - kResStages;
    // MODE 2: the stages of the second pass follow those of the first and read the same keys
    const int src_stage = (kTwoPass && sstage >= n_stages) ? sstage - n_stages : sstage;
    const int soff = (s_begin + src_stage * kStageRows) * kRowBytes;
    if (MODE == 1 && (stage & (kWaves - 1)) == wv)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(
          brsrc, (__attribute__((address_space(3))) void*)(slot + kDataBytes), 4, lane * 4,
          (s_begin + sstage * kStageRows) * 4, 0, 0);
#pragma unroll
    for (int j = 0; j < kLoadsPerThread; ++j) {
      const int grp = wv + kWaves * j;
      __builtin_amdgcn_raw_ptr_buffer_load_lds(
          rsrc, (__attribute__((address_space(3))) void*)(slot + grp * kGroupPitch),
          16, ld_voff, soff + j * (4 * kWaves * kRowBytes), 0, 0);
    }
  };
  // Once per ring stage g: this thread's pieces of stages g and g + 1 have landed when at most
  // (kDepth - 3) later stages of its loads are still in flight; the barrier extends that to
  // every thread's pieces and tells everyone that the slot consumed before is free, so the next
  // load can go there.  The barrier is bare: a fence here would drain the whole ring.
  auto ring_wait = [&]() {
    __builtin_amdgcn_s_waitcnt(0x0F70 | (((kDepth - 3) * kLoadsPerThread) & 0xF) |
                               ((((kDepth - 3) * kLoadsPerThread) >> 4) << 14));
    __builtin_amdgcn_s_barrier();
  };
  auto ring_sync = [&](int g) {  // g + kDepth - 1 >= kResStages
    ring_wait();
    issue_stage(g + kDepth - 1);
  };

  static_assert(!RING_RES || kResStages >= kDepth - 1, "the ring's first loads are resident rows");
  if (n_stages > 0) {
#pragma unroll
    for (int s = 0; s < kDepth - 1; ++s) {
      if (RING_RES) issue_resident(s);
      else issue_stage(s);
    }
  }

  // Operand rows of this lane inside a stage: row rt * 32 + c32 -> group, row-in-group
  // (lane (c32, h) holds row c32 of a 32-row tile, k-chunk h: the same layout for both operands)
  const int a_off = (c32 >> 2) * kGroupPitch + (c32 & 3) * 16 + h * 64;
  auto load_a = [&](bf16x8(&a)[NK], const unsigned char* slot, int rt) {
    const unsigned char* p = slot + rt * 8 * kGroupPitch + a_off;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) a[ks] = *reinterpret_cast<const bf16x8*>(p + ks * 128);
  };

  // ---- resident fragments: wave w owns ring stages [w CT / 2, (w + 1) CT / 2) of the resident
  // phase, two 32-row tiles each
  bf16x8 bres[CT][NK];
  auto res_row_of = [&](int ct) { return res_base + wv * kWaveRows + ct * 32 + c32; };
  if (!RING_RES) {
    // straight into registers through a bounds-checked descriptor (rows past the end read as
    // zero), after the ring's first loads are on their way so that the two latencies overlap
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) {
      const int r = res_row_of(ct);
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(res_rsrc, r * kRowBytes + h * 16, ks * 32, 0);
        bres[ct][ks] = __builtin_bit_cast(bf16x8, v);
      }
    }
  } else if (n_stages > 0) {
#pragma unroll
    for (int g = 0; g < kResStages; ++g) {
      ring_wait();
      if (g + kDepth - 1 < kResStages) issue_resident(g + kDepth - 1);
      else issue_stage(g + kDepth - 1);
      const unsigned char* slot = ring + (g % kDepth) * kStageBytes;
#pragma unroll
      for (int q = 0; q < CT / 2; ++q)
        if (g == wv * (CT / 2) + q) {
          load_a(bres[2 * q], slot, 0);
          load_a(bres[2 * q + 1], slot, 1);
          // the rows are in registers before the wave lets the slot go at the next barrier
          __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0) alone
        }
    }
  } else {
#pragma unroll
    for (int ct = 0; ct < CT; ++ct)
#pragma unroll
      for (int ks = 0; ks < NK; ++ks) bres[ct][ks] = bf16x8{0};
  }
  // a wave whose resident rows are all past the end only helps with loads and barriers
  const bool wave_live = res_base + wv * kWaveRows < res_limit;
  // sweep B: -L of the lane's 16 rows of tile row rt (accumulator order)
  auto load_nl = [&](float (&nl)[16], const unsigned char* slot, int rt) {
    if (MODE == 1) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        // read with the operands' vector type: a differently typed LDS read is taken to alias
        // the ring's loads still in flight and would wait for all of them
        const bf16x8 raw = *reinterpret_cast<const bf16x8*>(slot + kDataBytes + (rt * 32 + g * 8 + h * 4) * 4);
        const f32x4 v = __builtin_bit_cast(f32x4, raw);
        nl[g * 4 + 0] = v[0]; nl[g * 4 + 1] = v[1]; nl[g * 4 + 2] = v[2]; nl[g * 4 + 3] = v[3];
      }
    }
  };

  // per-lane reduction state
  // (vector values, not arrays: an array the optimiser cannot split ends up in scratch memory)
  typedef float fxCT __attribute__((ext_vector_type(CT)));
  fxCT m_ref, l_run;  // sweep A
  fxCT colsum;                 // sweep B
#pragma unroll
  for (int ct = 0; ct < CT; ++ct) {
    m_ref[ct] = kNegInf;
    l_run[ct] = 0.f;
    colsum[ct] = 0.f;
  }
  // sweep A: last key the lane's window row sees; sweep B: the lane's key
  auto vis_limit_of = [&](int ct) {
    return (kRowPass) ? (kp.causal ? N - W + res_row_of(ct) / Gq : N - 1) : res_row_of(ct);
  };
  const int tail_start = kp.causal ? N - W : N;  // keys > tail_start are hidden from some row
  typedef int ixCT __attribute__((ext_vector_type(CT)));
  ixCT first_row;  // sweep B: first window row that sees the lane's key
#pragma unroll
  for (int ct = 0; ct < CT; ++ct)
    first_row[ct] = (MODE == 1 && kp.causal) ? max(0, (res_row_of(ct) - (N - W)) * Gq) : 0;

  // ---- epilogues
  // sweep A: a tile's 16 terms are summed on their own and banked into the lane's running sum
  // once per tile, so the long sum over a unit's keys has N / 32 addends, not N / 2 (the rounding
  // error of a single fp32 running sum would grow with the unit's length)
  float tsum = 0.f;
  auto bank_tile = [&](int ct) {
    if (kRowPass) {
      // (static indices only: an index the optimiser does not see through would move the
      // array into scratch memory)
#pragma unroll
      for (int k = 0; k < CT; ++k)
        if (k == ct) l_run[k] += tsum;
      tsum = 0.f;
    }
  };
  // Masked variant (tag true): a logit is dropped by one comparison of its stream-row offset
  // inside the tile (a constant) with `d`, the lane's limit relative to the tile:
  //   sweep A: hidden iff offset > d, d = (last key the lane's row sees) - first row of the tile - 4 h
  //   sweep B: hidden iff offset < d, d = (first row that sees the lane's key) - first row of the tile - 4 h
  // sweep A: last stream row (key) that counts for the lane's window row.  Only masked stages
  // look at it: set_limits() runs in front of them, so the clean stages do not carry the values.
  int lim_a[CT];
  auto set_limits = [&]() {
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) lim_a[ct] = min(s_end - 1, vis_limit_of(ct));
  };
  auto mask_d = [&](int ct, int trow0) { return (kRowPass ? lim_a[ct] : first_row[ct]) - trow0 - h * 4; };
  auto piece = [&](auto masked, const f32x16& acc, const float (&nl)[16], int ct, int i, int d) {  // two logits of the fast epilogue
    constexpr bool kMasked = decltype(masked)::value;
    const int o0 = ((2 * i) >> 2) * 8 + ((2 * i) & 3), o1 = o0 + 1;  // row offsets of logits 2i, 2i + 1
    if (kRowPass) {
      const float nm = -m_ref[ct];
      float x0 = acc[2 * i], x1 = acc[2 * i + 1];
      if (kMasked) {
        x0 = o0 > d ? kNegInf : x0;
        x1 = o1 > d ? kNegInf : x1;
      }
      tsum += fast_exp2(__builtin_fmaf(x0, c, nm));
      tsum += fast_exp2(__builtin_fmaf(x1, c, nm));
      // pin the partial sum here: without it the optimiser is free to sink these pieces out
      // of the MFMA chain they are meant to overlap with
      asm volatile("" : "+v"(tsum));
    } else {
      float y0 = __builtin_fmaf(acc[2 * i], c, nl[2 * i]), y1 = __builtin_fmaf(acc[2 * i + 1], c, nl[2 * i + 1]);
      if (kMasked) {
        y0 = o0 < d ? kNegInf : y0;
        y1 = o1 < d ? kNegInf : y1;
      }
      colsum[ct] += fast_exp2(y0);
      colsum[ct] += fast_exp2(y1);
      asm volatile("" : "+v"(colsum[ct]));
    }
  };
  // exact online-softmax update of (m_ref, l_run) with the 16 logits of `acc` (masked = -inf)
  auto exact_update = [&](const f32x16& acc, int ct) {
    float xm = acc[0];
#pragma unroll
    for (int r = 1; r < 16; ++r) xm = fmaxf(xm, acc[r]);
    const float m_new = fmaxf(m_ref[ct], xm * c);
    const float nm = (m_new == kNegInf) ? 0.f : -m_new;
    float sum = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) sum += fast_exp2(__builtin_fmaf(acc[r], c, nm));
    l_run[ct] = l_run[ct] * fast_exp2(m_ref[ct] + nm) + sum;
    m_ref[ct] = m_new;
  };
  auto slow_tile = [&](f32x16& acc, const float (&nl)[16], int ct, int trow0) {
    if (kRowPass) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int key = trow0 + (r >> 2) * 8 + h * 4 + (r & 3);
        if (!(key <= lim_a[ct])) acc[r] = kNegInf;  // (the limit is already cut at the end of the stream)
      }
      exact_update(acc, ct);
    } else {
      // window row r sits at slot N - W + r / G, so key j is visible to it iff
      // r >= (j - (N - W)) * G: one comparison against a per-lane constant
      float sum = 0.f;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = trow0 + (r >> 2) * 8 + h * 4 + (r & 3);
        const float y = (row < first_row[ct]) ? kNegInf : __builtin_fmaf(acc[r], c, nl[r]);
        sum += fast_exp2(y);
      }
      colsum[ct] += sum;
    }
  };
  auto chain = [&](f32x16& acc, const bf16x8(&a)[NK], int ct) {
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[0], bres[ct][0], f32x16{0}, 0, 0, 0);
#pragma unroll
    for (int ks = 1; ks < NK; ++ks)
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ks], bres[ct][ks], acc, 0, 0, 0);
  };
  // chain of the new tile interleaved with the fast epilogue of the old one
  // (`trow_old`: first stream row of the old tile; only the masked variant looks at it)
  auto fused = [&](auto masked, f32x16& acc_new, const bf16x8(&a)[NK], int ct_new, const f32x16& acc_old,
                   const float (&nl_old)[16], int ct_old, int trow_old) {
    const int d = mask_d(ct_old, trow_old);
#pragma unroll
    for (int ks = 0; ks < NK; ++ks) {
      piece(masked, acc_old, nl_old, ct_old, ks, d);
      acc_new = (ks == 0)
                    ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[0], bres[ct_new][0], f32x16{0}, 0, 0, 0)
                    : __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ks], bres[ct_new][ks], acc_new, 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
    bank_tile(ct_old);
  };
  auto drain = [&](auto masked, const f32x16& acc_old, const float (&nl_old)[16], int ct_old, int trow_old) {
    const int d = mask_d(ct_old, trow_old);
#pragma unroll
    for (int i = 0; i < 8; ++i) piece(masked, acc_old, nl_old, ct_old, i, d);
    bank_tile(ct_old);
  };

  // ---- main loop over ring stages
  // Take the wait for the resident operands here, before the first barrier issues more loads:
  // left to the compiler it lands inside the loop prologue as a wait for every load in flight,
  // the ring's newest stage included.
#pragma unroll
  for (int ct = 0; ct < CT; ++ct)
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) asm volatile("" ::"v"(bres[ct][ks]));
  // Stream stage `it` is ring stage kResStages + it.  Being one stage ahead (see ring_sync) lets
  // a wave fetch the next stage's first operands from LDS while it is still busy with this one.
  auto stage_sync = [&](int it) { ring_sync(kResStages + it); };
  auto slot_of = [&](int it) -> const unsigned char* {
    return ring + ((kResStages + it) % kDepth) * kStageBytes;
  };
  f32x16 acc0, acc1;
  bf16x8 a0[NK], a1[NK];
  float nl0[16], nl1[16];  // sweep B: -L of the rows of tile rows 0 and 1 of the stage in flight
  auto slow_stage = [&](int it) {
    const unsigned char* cur = slot_of(it);
    const int stage_base = s_begin + it * kStageRows;
#pragma unroll
    for (int rt = 0; rt < 2; ++rt) {
      const int trow0 = stage_base + rt * 32;
      if (trow0 >= s_end) continue;
      load_a(a0, cur, rt);
      load_nl(nl0, cur, rt);
#pragma unroll
      for (int ct = 0; ct < CT; ++ct) {
        chain(acc0, a0, ct);
        slow_tile(acc0, nl0, ct, trow0);
      }
    }
    if (kRowPass) {
      // a lane that saw nothing yet takes 0 as its reference: (0, 0) is the empty sum
#pragma unroll
      for (int ct = 0; ct < CT; ++ct)
        if (m_ref[ct] == kNegInf) m_ref[ct] = 0.f;
    }
  };

  // Stages [f0, f1) run the pipelined path, [sk, f0) and [f1, n_stages) the masked path, and
  // the wave sits out stages [0, sk).
  // Sweep A: the causal tail and the ragged end are masked.
  // Sweep B: window rows come in slot order, so a wave whose keys lie in the window sees
  // nothing in the first stages (every row is older than its oldest key), is partly masked
  // until the rows pass its youngest key, and is clean from there on.
  int sk = 0, f0 = 0, f1;
  if (kRowPass) {
    const int clean_rows = min(tail_start + 1, s_end) - s_begin;  // keys every row sees
    f1 = clean_rows > 0 ? clean_rows / kStageRows : 0;
  } else {
    if (kp.causal) {
      const int k0 = res_base + wv * kWaveRows - (N - W);  // the wave's oldest key, relative to the window
      const int fr_min = max(0, k0 * Gq), fr_max = max(0, (k0 + kWaveRows - 1) * Gq);
      sk = max(0, min(n_stages, (fr_min - s_begin) / kStageRows));
      f0 = max(sk, min(n_stages, (fr_max - s_begin + kStageRows - 1) / kStageRows));
    }
    f1 = n_stages;
  }
  f1 = max(min(f1, n_stages), f0);
  if (!wave_live) sk = f0 = f1 = n_stages;  // only loads and barriers: the first loop below

  // stages [from, to), to > from, software-pipelined; does the stage_sync of each of them
  auto pipelined = [&](auto masked, int from, int to) {
    constexpr bool kMasked = decltype(masked)::value;
    stage_sync(from);
    load_a(a0, slot_of(from), 0);
    load_nl(nl0, slot_of(from), 0);
    if (kRowPass && !kMasked && from == 0) {
      // Nothing seen yet: the first logit of the lane's own row is the reference.  Too low shows
      // as an infinite sum at the end and sends the wave through the exact recomputation; too
      // high only means every other term is negligible next to this one, which is itself part
      // of the sum.
      chain(acc1, a0, 1);
      m_ref[1] = acc1[0] * c;
      chain(acc0, a0, 0);
      m_ref[0] = acc0[0] * c;
    } else {
      chain(acc0, a0, 0);
    }
    for (int it = from;; ++it) {
      const unsigned char* cur = slot_of(it);
      const int base = s_begin + it * kStageRows;
      load_a(a1, cur, 1);
      load_nl(nl1, cur, 1);
      fused(masked, acc1, a0, 1, acc0, nl0, 0, base);
      load_a(a0, slot_of(it + 1), 0);  // a0 is free: operands of the coming stage
      fused(masked, acc0, a1, 0, acc1, nl0, 1, base);
      load_nl(nl0, slot_of(it + 1), 0);  // the last tile of tile row 0 is through its epilogue
      fused(masked, acc1, a1, 1, acc0, nl1, 0, base + 32);
      if (it + 1 >= to) break;
      stage_sync(it + 1);
      fused(masked, acc0, a0, 0, acc1, nl1, 1, base + 32);
    }
    drain(masked, acc1, nl1, 1, s_begin + (to - 1) * kStageRows + 32);
  };
  // Wide form, four resident tiles per wave (both sweeps): a wave keeps ONE tile row's stream
  // operands; while the last of the tile row's four chains consumes them k-step by k-step, each
  // is replaced in place by the next tile row's (the 32 registers that saves, with the 64 the two
  // more resident tiles cost, still fit two waves per SIMD).  Sweep B's 16 -L values of a tile
  // row change hands the same way during the chain that carries the tile row's last epilogue.
  // Tiles of a stage in the order (tile row, resident tile) = (0,0) (0,1) (0,2) (0,3) (1,0) ...
  // (1,3), accumulators alternating.
  // fused_refill: `refill_a`: the stream operands are replaced by the rows at `next_rows`;
  // `refill_nl` (sweep B): the -L values by those at `next_nl`, four at a time behind the two
  // pieces that used them.
  auto fused_refill = [&](auto masked, auto refill_a, auto refill_nl, f32x16& acc_new, bf16x8(&a)[NK],
                          int ct_new, const f32x16& acc_old, float (&nl)[16], int ct_old, int trow_old,
                          const unsigned char* next_rows, const unsigned char* next_nl) {
    constexpr bool kA = decltype(refill_a)::value, kNl = decltype(refill_nl)::value && MODE == 1;
    const int d = mask_d(ct_old, trow_old);
#pragma unroll
    for (int ks = 0; ks < NK; ++ks) {
      piece(masked, acc_old, nl, ct_old, ks, d);
      acc_new = (ks == 0)
                    ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[0], bres[ct_new][0], f32x16{0}, 0, 0, 0)
                    : __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ks], bres[ct_new][ks], acc_new, 0, 0, 0);
      if (kA) a[ks] = *reinterpret_cast<const bf16x8*>(next_rows + ks * 128);
      if (kNl && (ks & 1)) {
        const int g = ks >> 1;
        const bf16x8 raw = *reinterpret_cast<const bf16x8*>(next_nl + (g * 8 + h * 4) * 4);
        const f32x4 v = __builtin_bit_cast(f32x4, raw);
        nl[g * 4 + 0] = v[0]; nl[g * 4 + 1] = v[1]; nl[g * 4 + 2] = v[2]; nl[g * 4 + 3] = v[3];
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    bank_tile(ct_old);
  };
  auto pipelined_wide = [&](auto masked, int from, int to) {
    constexpr bool kMasked = decltype(masked)::value;
    constexpr int L = CT - 1;  // the last resident tile
    const std::integral_constant<bool, true> yes;
    const std::integral_constant<bool, false> no;
    stage_sync(from);
    load_a(a0, slot_of(from), 0);
    load_nl(nl0, slot_of(from), 0);
    if (kRowPass && !kMasked && from == 0) {
      // references: the first logit of every resident row of the lane
#pragma unroll
      for (int ct = L; ct >= 1; --ct) {
        chain(acc1, a0, ct);
        m_ref[ct] = acc1[0] * c;
      }
      chain(acc0, a0, 0);
      m_ref[0] = acc0[0] * c;
    } else {
      chain(acc0, a0, 0);
    }
    for (int it = from;; ++it) {
      const unsigned char* cur = slot_of(it);
      const int base = s_begin + it * kStageRows;
      fused(masked, acc1, a0, 1, acc0, nl0, 0, base);
      fused(masked, acc0, a0, 2, acc1, nl0, 1, base);
      // a0 <- tile row 1 behind the last chain of tile row 0
      fused_refill(masked, yes, no, acc1, a0, 3, acc0, nl0, 2, base, cur + 8 * kGroupPitch + a_off, nullptr);
      // the last epilogue of tile row 0 hands its -L registers over to tile row 1
      fused_refill(masked, no, yes, acc0, a0, 0, acc1, nl0, 3, base, nullptr, cur + kDataBytes + 32 * 4);
      fused(masked, acc1, a0, 1, acc0, nl0, 0, base + 32);
      fused(masked, acc0, a0, 2, acc1, nl0, 1, base + 32);
      if (it + 1 >= to) {
        fused(masked, acc1, a0, 3, acc0, nl0, 2, base + 32);
        break;
      }
      const unsigned char* nxt = slot_of(it + 1);
      fused_refill(masked, yes, no, acc1, a0, 3, acc0, nl0, 2, base + 32, nxt + a_off, nullptr);  // a0 <- next stage
      stage_sync(it + 1);
      fused_refill(masked, no, yes, acc0, a0, 0, acc1, nl0, 3, base + 32, nullptr, nxt + kDataBytes);
    }
    drain(masked, acc1, nl0, L, s_begin + (to - 1) * kStageRows + 32);
  };
  const std::integral_constant<bool, false> clean_tag;
  const std::integral_constant<bool, true> masked_tag;

  int it = 0;
  if (kRowPass && f0 < f1) {
    // (placeholder values while the clean stages run: nothing reads them there)
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) lim_a[ct] = 0;
  } else if (kRowPass) {
    set_limits();
  }
  for (; it < sk; ++it) stage_sync(it);
  if (MODE == 1) {
    // the partly visible stages run pipelined as well, with the mask in the epilogue
    if (f0 > sk) {
      if (CT == 4) pipelined_wide(masked_tag, sk, f0);
      else pipelined(masked_tag, sk, f0);
    }
  } else {
    for (; it < f0; ++it) {
      stage_sync(it);
      slow_stage(it);
    }
  }
  if (f1 > f0) {
    if (CT == 4) pipelined_wide(clean_tag, f0, f1);
    else pipelined(clean_tag, f0, f1);
  }
  it = f1;
  if (kRowPass) set_limits();
  if (kRowPass && f1 > 0 && n_stages > f1) {
    // the tail (causal, ragged end) after at least one clean stage: the reference is set, so
    // the masked epilogue can take it
    if (CT == 4) pipelined_wide(masked_tag, f1, n_stages);
    else pipelined(masked_tag, f1, n_stages);
    it = n_stages;
  }
  for (; it < n_stages; ++it) {
    stage_sync(it);
    slow_stage(it);
  }
  if (kRowPass && wave_live) {
    // Range check of the fast epilogue, once per wave: a finite sum is exact.
    bool bad = false;
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) bad = bad || !(l_run[ct] < __builtin_inff());
    if (__builtin_amdgcn_ballot_w64(bad) != 0ull) {
      // Recompute this wave's statistics with a true running maximum.  The ring belongs to the
      // whole workgroup, so the stream rows come straight from memory (same bounds-checked
      // descriptor: rows past the end read as zero and are masked).
#pragma unroll
      for (int ct = 0; ct < CT; ++ct) {
        m_ref[ct] = kNegInf;
        l_run[ct] = 0.f;
      }
      for (int stg = 0; stg < n_stages; ++stg) {
        for (int rt = 0; rt < 2; ++rt) {
          const int trow0 = s_begin + stg * kStageRows + rt * 32;
          if (trow0 >= s_end) continue;
#pragma unroll
          for (int ks = 0; ks < 8; ++ks) {
            const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (trow0 + c32) * kRowBytes + h * 16, ks * 32, 0);
            a0[ks] = __builtin_bit_cast(bf16x8, v);
          }
#pragma unroll
          for (int ct = 0; ct < CT; ++ct) {
            chain(acc0, a0, ct);
            slow_tile(acc0, nl0, ct, trow0);
          }
        }
      }
#pragma unroll
      for (int ct = 0; ct < CT; ++ct)
        if (m_ref[ct] == kNegInf) m_ref[ct] = 0.f;
    }
  }
  // loads issued past the last stage may still be landing in LDS: let them finish before the
  // workgroup's LDS can be handed to another one
  if (!kTwoPass) __builtin_amdgcn_s_waitcnt(0x0F70);

  // ---- finish
  if (kTwoPass) {
    // ---- second pass: the same resident window rows are now the A operand and the keys
    // stream through the ring once more (their stages were requested while the first pass
    // finished), so a lane owns one key column of a tile and 16 window rows.  exp2(c x - L_row)
    // summed over the rows of this wave is one partial column sum per key; the waves write
    // theirs side by side (`parts[unit][16-row-block wave][key]`) and whoever reads the scores
    // adds them in wave order: no atomics, the same bits every run.
    float* negl_s = reinterpret_cast<float*>(smem + kDepth * kStageBytes);  // -L of the workgroup's 256 rows
#pragma unroll
    for (int ct = 0; ct < 2; ++ct) {
      const float m2 = __shfl_xor(m_ref[ct], 32, 64);
      const float l2 = __shfl_xor(l_run[ct], 32, 64);
      float mc = m_ref[ct], lc = l_run[ct];
      ml_combine(mc, lc, m2, l2);
      m_ref[ct] = mc;
      l_run[ct] = lc;
      if (h == 0)
        negl_s[wv * 64 + ct * 32 + c32] = res_row_of(ct) < Mq ? -(m_ref[ct] + log2f(l_run[ct])) : kPadNegL;
    }
    // the wave reads back only what it wrote itself (LDS operations of a wave stay in order);
    // the empty asm keeps the compiler from moving the differently typed reads above the writes
    asm volatile("" ::: "memory");
    float nlq[2][16];
#pragma unroll
    for (int ct = 0; ct < 2; ++ct)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const bf16x8 raw = *reinterpret_cast<const bf16x8*>(
            reinterpret_cast<const unsigned char*>(negl_s) + (wv * 64 + ct * 32 + g * 8 + h * 4) * 4);
        const f32x4 v = __builtin_bit_cast(f32x4, raw);
        nlq[ct][g * 4 + 0] = v[0]; nlq[ct][g * 4 + 1] = v[1]; nlq[ct][g * 4 + 2] = v[2]; nlq[ct][g * 4 + 3] = v[3];
      }
    float* part_out = parts + ((size_t)unit * ((Mq + 63) / 64) + (res_base >> 6) + wv) * part_pitch;
    float ksum = 0.f;
    auto chain2 = [&](f32x16& acc, const bf16x8(&a)[NK], int ct) {
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bres[ct][0], a[0], f32x16{0}, 0, 0, 0);
#pragma unroll
      for (int ks = 1; ks < NK; ++ks)
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bres[ct][ks], a[ks], acc, 0, 0, 0);
    };
    // hidden iff the row's offset inside the resident tile is < d,
    // d = (first window row that sees the lane's key) - first row of the tile - 4 h
    auto mask_d2 = [&](int ct, int key) {
      const int first = kp.causal ? max(0, (key - (N - W)) * Gq) : 0;
      return first - (res_base + wv * 64 + ct * 32 + h * 4);
    };
    auto piece2 = [&](auto masked, const f32x16& acc, int ct, int i, int d) {
      constexpr bool kMasked = decltype(masked)::value;
      const int o0 = ((2 * i) >> 2) * 8 + ((2 * i) & 3), o1 = o0 + 1;
      float y0 = __builtin_fmaf(acc[2 * i], c, nlq[ct][2 * i]), y1 = __builtin_fmaf(acc[2 * i + 1], c, nlq[ct][2 * i + 1]);
      if (kMasked) {
        y0 = o0 < d ? kNegInf : y0;
        y1 = o1 < d ? kNegInf : y1;
      }
      ksum += fast_exp2(y0);
      ksum += fast_exp2(y1);
      asm volatile("" : "+v"(ksum));
    };
    auto fused2 = [&](auto masked, f32x16& acc_new, const bf16x8(&a)[NK], int ct_new, const f32x16& acc_old,
                      int ct_old, int key_old) {
      const int d = mask_d2(ct_old, key_old);
#pragma unroll
      for (int ks = 0; ks < NK; ++ks) {
        piece2(masked, acc_old, ct_old, ks, d);
        acc_new = (ks == 0)
                      ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(bres[ct_new][0], a[0], f32x16{0}, 0, 0, 0)
                      : __builtin_amdgcn_mfma_f32_32x32x16_bf16(bres[ct_new][ks], a[ks], acc_new, 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
      }
    };
    // MODE 3: per stage and wave 64 partial column sums go to LDS (a ring of four stages behind
    // the -L table), and two barriers later the wave whose turn it is adds the four waves' sums
    // in wave order.  The LDS traffic is written out as instructions: accesses the compiler
    // generates here would be taken to alias the ring's loads in flight and wait for all of them.
    const unsigned xs_base = (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)(
        smem + kDepth * kStageBytes + kResRows * sizeof(float));
    const int two_blocks = Mq > kResRows;
    const float inv_mq = 1.0f / (float)Mq;
    auto reduce_stage = [&](int st) {  // all four waves' sums of pass-2 stage `st` are in LDS
      float v0, v1, v2, v3;
      const unsigned addr = xs_base + (unsigned)(((st & 3) * kWaves * 64 + lane) * 4);
      asm volatile(
          "ds_read_b32 %0, %4\n\tds_read_b32 %1, %4 offset:256\n\tds_read_b32 %2, %4 offset:512\n\t"
          "ds_read_b32 %3, %4 offset:768\n\ts_waitcnt lgkmcnt(0)"
          : "=&v"(v0), "=&v"(v1), "=&v"(v2), "=&v"(v3)
          : "v"(addr));
      float v = v0;  // wave 0 always has rows
      if (res_base + 64 < res_limit) v += v1;
      if (res_base + 128 < res_limit) v += v2;
      if (res_base + 192 < res_limit) v += v3;
      const int key = s_begin + st * kStageRows + lane;
      if (key < N) {
        if (two_blocks) atomicAdd(&scores[row0 + key], v * inv_mq);
        else scores[row0 + key] = v * inv_mq;
      }
    };
    auto flush = [&](int key, int st, int kt) {  // both resident tiles of this key tile are through their epilogue
      const float tot = ksum + __shfl_xor(ksum, 32, 64);
      if (kWgReduce) {
        if (h == 0) {
          const unsigned addr = xs_base + (unsigned)((((st & 3) * kWaves + wv) * 64 + kt * 32 + c32) * 4);
          asm volatile("ds_write_b32 %0, %1" ::"v"(addr), "v"(tot));
        }
      } else {
        if (h == 0 && key < N) part_out[key] = tot;
      }
      ksum = 0.f;
    };
    // barrier of pass-2 stage it2; MODE 3: the waves' LDS writes are complete before it, and the
    // sums of stage it2 - 2 (complete since the barrier before this one) are added by one wave
    auto sync2 = [&](int it2) {
      if (kWgReduce) __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0) alone; vmcnt is stage_sync's business
      stage_sync(n_stages + it2);
      if (kWgReduce && it2 >= 2 && ((it2 - 2) & 3) == wv) reduce_stage(it2 - 2);
    };
    // stages [from, to) of the second pass (ring stages n_stages + from ...), software-pipelined
    auto pipelined2 = [&](auto masked, int from, int to) {
      sync2(from);
      load_a(a0, slot_of(n_stages + from), 0);
      chain2(acc0, a0, 0);
      for (int it = from;; ++it) {
        const unsigned char* cur = slot_of(n_stages + it);
        const int key0 = s_begin + it * kStageRows + c32;  // the lane's key in key tile 0 of the stage
        load_a(a1, cur, 1);
        fused2(masked, acc1, a0, 1, acc0, 0, key0);
        load_a(a0, slot_of(n_stages + it + 1), 0);
        fused2(masked, acc0, a1, 0, acc1, 1, key0);
        flush(key0, it, 0);
        fused2(masked, acc1, a1, 1, acc0, 0, key0 + 32);
        if (it + 1 >= to) break;
        sync2(it + 1);
        fused2(masked, acc0, a0, 0, acc1, 1, key0 + 32);
        flush(key0 + 32, it, 1);
      }
      const int key1 = s_begin + (to - 1) * kStageRows + 32 + c32;
      const int d = mask_d2(1, key1);
#pragma unroll
      for (int i = 0; i < 8; ++i) piece2(masked, acc1, 1, i, d);
      flush(key1, to - 1, 1);
    };
    if (wave_live) {
      const int clean = min(f1, n_stages);  // stages whose keys every window row sees
      if (clean > 0) pipelined2(clean_tag, 0, clean);
      if (n_stages > clean) pipelined2(masked_tag, clean, n_stages);
      // keys past the stages that ran are hidden from every row of this workgroup
      if (!kWgReduce)
        for (int key = s_begin + n_stages * kStageRows + lane; key < N; key += 64) part_out[key] = 0.f;
    } else {
      for (int it2 = 0; it2 < n_stages; ++it2) sync2(it2);
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);
    if (kWgReduce) {
      // the last two stages' sums: complete once every wave is here
      __builtin_amdgcn_s_waitcnt(0xC07F);
      __builtin_amdgcn_s_barrier();
      if (n_stages >= 2 && ((n_stages - 2) & 3) == wv) reduce_stage(n_stages - 2);
      if (n_stages >= 1 && ((n_stages - 1) & 3) == wv) reduce_stage(n_stages - 1);
      // a single row block stores its scores: keys past its stages are hidden from every row
      if (!two_blocks && wv == 0)
        for (int key = s_begin + n_stages * kStageRows + lane; key < N; key += 64) scores[row0 + key] = 0.f;
    }
  } else if (MODE == 0) {
    float2* part = rowstat + (size_t)unit * n_splits * mq_pad;
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) {
      const float m2 = __shfl_xor(m_ref[ct], 32, 64);
      const float l2 = __shfl_xor(l_run[ct], 32, 64);
      float mc = m_ref[ct], lc = l_run[ct];
      ml_combine(mc, lc, m2, l2);
      m_ref[ct] = mc;
      l_run[ct] = lc;
      if (h == 0 && res_row_of(ct) < Mq)
        part[(size_t)split * mq_pad + res_row_of(ct)] = make_float2(m_ref[ct], l_run[ct]);
      // a single split is the whole row: -L goes out here and no combining kernel runs
      if (n_splits == 1 && h == 0 && res_row_of(ct) < mq_pad)
        bias_out[(size_t)unit * mq_pad + res_row_of(ct)] =
            res_row_of(ct) < Mq ? -(m_ref[ct] + log2f(l_run[ct])) : kPadNegL;
    }
  } else if (MODE == 1) {
    const float inv = 1.0f / (float)Mq;
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) {
      const float tot = colsum[ct] + __shfl_xor(colsum[ct], 32, 64);
      if (h == 0 && res_row_of(ct) < N) {
        if (q_splits == 2) atomicAdd(&scores[row0 + res_row_of(ct)], tot * inv);
        else scores[row0 + res_row_of(ct)] = tot * inv;
      }
    }
  }
}

// ------------------------------------------------------------------ plain FMA path

// Sweep A: thread = (window row, key sub-range); q row in registers, keys read by the whole
// wave at the same address (broadcast).
template <typename T, int D>
__global__ __launch_bounds__(256) void score_rows_fma_kernel(
    KParams kp, int n_units, int tiles_per_unit, int n_splits, int split_len, int mq_pad,
    const int64_t* __restrict__ row_off, const T* __restrict__ K, const T* __restrict__ Q,
    float2* __restrict__ rowstat) {
  __shared__ float2 xch[256];
  int unit, tile;
  if (!map_block(n_units, tiles_per_unit, unit, tile)) return;
  const int tid = threadIdx.x, lane = tid & 63, sub = tid >> 6;
  const int qb = tile / n_splits, split = tile % n_splits;
  const int row = qb * 64 + lane;
  const int Mq = kp.Mq;
  if (qb * 64 >= Mq) return;
  const int64_t row0 = row_off[unit];
  const int N = (int)(row_off[unit + 1] - row0);
  const bool ok = row < Mq;
  float q[D];
  const T* qp = Q + ((size_t)unit * Mq + (ok ? row : 0)) * D;
#pragma unroll
  for (int i = 0; i < D; ++i) q[i] = Elem<T>::load(qp + i);
  int k_begin = split * split_len;
  int k_end = min(N, k_begin + split_len);
  const int quarter = (split_len + 3) / 4;
  k_begin += sub * quarter;
  k_end = min(k_end, k_begin + quarter);
  const int last_vis = kp.causal ? N - kp.W + (ok ? row : 0) / kp.G : N - 1;
  k_end = min(k_end, last_vis + 1);
  float m = kNegInf, l = 0.f;
  for (int j = k_begin; j < k_end; ++j) {
    const T* kr = K + (size_t)(row0 + j) * D;
    float dot = 0.f;
#pragma unroll
    for (int i = 0; i < D; ++i) dot = __builtin_fmaf(q[i], Elem<T>::load(kr + i), dot);
    const float y = dot * kp.scale_log2;
    const float m_new = fmaxf(m, y);
    l = l * fast_exp2(m - m_new) + fast_exp2(y - m_new);
    m = m_new;
  }
  xch[tid] = make_float2(m, l);
  __syncthreads();
  if (sub == 0) {
    for (int s = 1; s < 4; ++s) ml_combine(m, l, xch[s * 64 + lane].x, xch[s * 64 + lane].y);
    if (ok) rowstat[((size_t)unit * n_splits + split) * mq_pad + row] = make_float2(m, l);
  }
}

// Sweep B: thread = key; key row in registers, window rows read at a wave-uniform address.
template <typename T, int D>
__global__ __launch_bounds__(256) void score_cols_fma_kernel(
    KParams kp, int n_units, int tiles_per_unit, int n_splits, int mq_pad,
    const int64_t* __restrict__ row_off, const T* __restrict__ K, const T* __restrict__ Q,
    const float2* __restrict__ rowstat, float* __restrict__ scores) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  float* negL = reinterpret_cast<float*>(smem);
  int unit, tile;
  if (!map_block(n_units, tiles_per_unit, unit, tile)) return;
  const int tid = threadIdx.x;
  const int64_t row0 = row_off[unit];
  const int N = (int)(row_off[unit + 1] - row0);
  if (tile * 256 >= N) return;
  const int Mq = kp.Mq;
  fill_neg_lse(rowstat + (size_t)unit * n_splits * mq_pad, n_splits, mq_pad, Mq, negL, tid, 256, mq_pad);
  __syncthreads();
  const int j = tile * 256 + tid;
  const bool ok = j < N;
  float k[D];
  const T* kr = K + (size_t)(row0 + (ok ? j : 0)) * D;
#pragma unroll
  for (int i = 0; i < D; ++i) k[i] = Elem<T>::load(kr + i);
  float sum = 0.f;
  for (int r = 0; r < Mq; ++r) {
    const int tw = kp.causal ? N - kp.W + r / kp.G : N - 1;
    if (j > tw) continue;
    const T* qp = Q + ((size_t)unit * Mq + r) * D;
    float dot = 0.f;
#pragma unroll
    for (int i = 0; i < D; ++i) dot = __builtin_fmaf(k[i], Elem<T>::load(qp + i), dot);
    sum += fast_exp2(__builtin_fmaf(dot, kp.scale_log2, negL[r]));
  }
  if (ok) scores[row0 + j] = sum * (1.0f / (float)Mq);
}

template <typename T, int D>
hipError_t launch_fma(const KParams& kp, const Batch& b, const Workspace& wl, char* ws,
                      float* scores, hipStream_t st, hipEvent_t between) {
  float2* rowstat = reinterpret_cast<float2*>(ws + wl.rowstat);
  const int units8 = (b.n_units + 7) / 8 * 8;
  const int qblocks = (kp.Mq + 63) / 64;
  const int tilesA = qblocks * wl.n_splits;
  score_rows_fma_kernel<T, D><<<dim3(units8 * tilesA), dim3(256), 0, st>>>(
      kp, b.n_units, tilesA, wl.n_splits, wl.split_len, wl.mq_pad, b.row_off,
      static_cast<const T*>(b.K), static_cast<const T*>(b.Q), rowstat);
  if (between) (void)hipEventRecord(between, st);
  const int tilesB = (b.max_unit_len + 255) / 256;
  score_cols_fma_kernel<T, D><<<dim3(units8 * tilesB), dim3(256), wl.mq_pad * sizeof(float), st>>>(
      kp, b.n_units, tilesB, wl.n_splits, wl.mq_pad, b.row_off, static_cast<const T*>(b.K),
      static_cast<const T*>(b.Q), rowstat, scores);
  return hipGetLastError();
}

}  // namespace

bool score_uses_mfma(const KParams& kp) {
  return kp.dtype == CASK_BF16 && kp.d == 128;
}

hipError_t launch_score(const KParams& kp, const Batch& b, const Workspace& wl, char* ws,
                        float* scores, hipStream_t st, hipEvent_t between) {
  if (!score_uses_mfma(kp)) {
    if (kp.dtype == CASK_F32)
      return kp.d == 64 ? launch_fma<float, 64>(kp, b, wl, ws, scores, st, between)
                        : launch_fma<float, 128>(kp, b, wl, ws, scores, st, between);
    return kp.d == 64 ? launch_fma<uint16_t, 64>(kp, b, wl, ws, scores, st, between)
                      : launch_fma<uint16_t, 128>(kp, b, wl, ws, scores, st, between);
  }
  float2* rowstat = reinterpret_cast<float2*>(ws + wl.rowstat);
  float* bias = reinterpret_cast<float*>(ws + wl.bias);
  const int units8 = (b.n_units + 7) / 8 * 8;
  const uint16_t* K = static_cast<const uint16_t*>(b.K);
  const uint16_t* Q = static_cast<const uint16_t*>(b.Q);
  const size_t ldsA = (size_t)kDepth * kStageBytes;
  const size_t ldsB = ldsA;
  static LdsLimitOnce limA, limB;
  hipError_t e = limA.ensure(reinterpret_cast<const void*>(&score_mfma_kernel<0>), 160 * 1024);
  if (e == hipSuccess) e = limB.ensure(reinterpret_cast<const void*>(&score_mfma_kernel<1>), 160 * 1024);
  if (e != hipSuccess) return e;
  const int qblocks = (kp.Mq + kResRows - 1) / kResRows;
  // W*G <= 512 (one wide row block per unit, eight stream stages per workgroup of sweep B): the
  // resident rows come through the ring (measured: both sweeps 3 - 4 % faster on the Llama-shaped
  // batch, up to 4 % slower at W*G = 896)
  const bool ring_res = kp.Mq <= 2 * kResRows;
  if (wl.wide_rows) {
    static LdsLimitOnce limAw, limAr;
    e = ring_res ? limAr.ensure(reinterpret_cast<const void*>(&score_mfma_kernel<0, 4, true>), 160 * 1024)
                 : limAw.ensure(reinterpret_cast<const void*>(&score_mfma_kernel<0, 4>), 160 * 1024);
    if (e != hipSuccess) return e;
    const int tilesAw = (kp.Mq + 2 * kResRows - 1) / (2 * kResRows) * wl.n_splits;
    auto kern = ring_res ? &score_mfma_kernel<0, 4, true> : &score_mfma_kernel<0, 4>;
    kern<<<dim3(units8 * tilesAw), dim3(kThreads), ldsA, st>>>(
        kp, b.n_units, tilesAw, wl.n_splits, wl.split_len, wl.q_splits, wl.mq_pad, b.row_off, K, Q, rowstat,
        nullptr, bias, scores, nullptr, 0);
  } else {
    const int tilesA = qblocks * wl.n_splits;
    score_mfma_kernel<0><<<dim3(units8 * tilesA), dim3(kThreads), ldsA, st>>>(
        kp, b.n_units, tilesA, wl.n_splits, wl.split_len, wl.q_splits, wl.mq_pad, b.row_off, K, Q, rowstat,
        nullptr, bias, scores, nullptr, 0);
  }
  if (between) (void)hipEventRecord(between, st);  // right behind sweep A: the stage is that kernel alone
  if (wl.n_splits > 1)  // with one split sweep A has written -L itself
    score_bias_kernel<<<dim3(b.n_units), dim3(kBiasThreads), 0, st>>>(kp, wl.n_splits, wl.mq_pad, rowstat, bias);
  if (wl.wide_cols) {
    static LdsLimitOnce limBw, limBr;
    e = ring_res ? limBr.ensure(reinterpret_cast<const void*>(&score_mfma_kernel<1, 4, true>), 160 * 1024)
                 : limBw.ensure(reinterpret_cast<const void*>(&score_mfma_kernel<1, 4>), 160 * 1024);
    if (e != hipSuccess) return e;
    const int tilesBw = (b.max_unit_len + 2 * kResRows - 1) / (2 * kResRows) * wl.q_splits;
    auto kern = ring_res ? &score_mfma_kernel<1, 4, true> : &score_mfma_kernel<1, 4>;
    kern<<<dim3(units8 * tilesBw), dim3(kThreads), ldsB, st>>>(
        kp, b.n_units, tilesBw, wl.n_splits, wl.split_len, wl.q_splits, wl.mq_pad, b.row_off, K, Q, rowstat,
        bias, nullptr, scores, nullptr, 0);
  } else {
    const int tilesB = (b.max_unit_len + kResRows - 1) / kResRows * wl.q_splits;
    score_mfma_kernel<1><<<dim3(units8 * tilesB), dim3(kThreads), ldsB, st>>>(
        kp, b.n_units, tilesB, wl.n_splits, wl.split_len, wl.q_splits, wl.mq_pad, b.row_off, K, Q, rowstat,
        bias, nullptr, scores, nullptr, 0);
  }
  return hipGetLastError();
}

namespace {
__global__ __launch_bounds__(256) void clear_scores_kernel(float* __restrict__ scores, int64_t n) {
  const int64_t stride = (int64_t)gridDim.x * 256 * 4;
  for (int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4; i < n; i += stride) {
    if (i + 3 < n) {
      *reinterpret_cast<float4*>(scores + i) = make_float4(0.f, 0.f, 0.f, 0.f);
    } else {
      for (int64_t j = i; j < n; ++j) scores[j] = 0.f;
    }
  }
}
}  // namespace

// Both sweeps in one launch for units of any length: pays when a workgroup of the second sweep
// would stream few window rows (at most eight stages behind a full prologue) and there are
// enough (unit, row block) pairs to fill the chip several times over.  Its waves hold 64 window
// rows each; with 256 < W*G <= 512 the two separate sweeps in their wide form (128 resident rows
// per wave) are faster (a Llama-shaped ragged batch: 10.7 against 11.4 ms), so the one launch is
// left to W*G <= 256 unless the caller asks for it.
bool score_fused_fits(const KParams& kp, const Batch& b) {
  const int row_blocks = (kp.Mq + kResRows - 1) / kResRows;
  if (!score_uses_mfma(kp) || kp.Mq > 2 * kResRows || (kp.path_flags & CASK_PATH_NO_FUSED_SWEEPS)) return false;
  if (kp.path_flags & CASK_PATH_FORCE_FUSED_SWEEPS) return true;
  if (kp.Mq > kResRows && !(kp.path_flags & CASK_PATH_NARROW_ROWS)) return false;
  return (int64_t)b.n_units * row_blocks >= 1024;
}

hipError_t launch_score_fused(const KParams& kp, const Batch& b, const Workspace& wl, float* scores,
                              hipStream_t st) {
  if (!score_fused_fits(kp, b)) return hipErrorInvalidValue;
  const size_t lds = (size_t)kDepth * kStageBytes + kResRows * sizeof(float) + 4 * kWaves * 64 * sizeof(float);
  static LdsLimitOnce lim;
  const hipError_t e = lim.ensure(reinterpret_cast<const void*>(&score_mfma_kernel<3>), 160 * 1024);
  if (e != hipSuccess) return e;
  const int units8 = (b.n_units + 7) / 8 * 8;
  const int qblocks = (kp.Mq + kResRows - 1) / kResRows;
  if (qblocks == 2) {
    // two workgroups add onto each key's score; scores is 4-byte aligned only: float4 stores need 16
    const bool al16 = (reinterpret_cast<uintptr_t>(scores) & 15u) == 0;
    if (al16) {
      const int64_t n = b.total_rows;
      const int blocks = (int)((n / 4 + 255) / 256 < 8192 ? (n / 4 + 255) / 256 + 1 : 8192);
      clear_scores_kernel<<<dim3(blocks), dim3(256), 0, st>>>(scores, n);
    } else {
      return hipErrorInvalidValue;
    }
  }
  const int whole = (b.max_unit_len + kStageRows - 1) / kStageRows * kStageRows;
  score_mfma_kernel<3><<<dim3(units8 * qblocks), dim3(kThreads), lds, st>>>(
      kp, b.n_units, qblocks, 1, whole, 1, wl.mq_pad, b.row_off, static_cast<const uint16_t*>(b.K),
      static_cast<const uint16_t*>(b.Q), nullptr, nullptr, nullptr, scores, nullptr, 0);
  return hipGetLastError();
}

bool score_parts_fits(const KParams& kp, const Batch& b, const Workspace& wl) {
  return score_uses_mfma(kp) && wl.n_splits == 1 && wl.parts_pitch > 0 && b.max_unit_len <= wl.parts_pitch;
}

// Both scoring sweeps in one launch (short units, one key split): writes, for every unit,
// ceil(W*G / 64) partial column sums per key, `parts[unit][part][key]` with row pitch
// wl.parts_pitch; score[key] = (sum of the parts in order) / (W*G).
hipError_t launch_score_parts(const KParams& kp, const Batch& b, const Workspace& wl, char* ws,
                              hipStream_t st) {
  if (!score_parts_fits(kp, b, wl)) return hipErrorInvalidValue;
  const size_t lds = (size_t)kDepth * kStageBytes + kResRows * sizeof(float);
  static LdsLimitOnce lim;
  const hipError_t e = lim.ensure(reinterpret_cast<const void*>(&score_mfma_kernel<2>), 160 * 1024);
  if (e != hipSuccess) return e;
  const int units8 = (b.n_units + 7) / 8 * 8;
  const int qblocks = (kp.Mq + kResRows - 1) / kResRows;
  score_mfma_kernel<2><<<dim3(units8 * qblocks), dim3(kThreads), lds, st>>>(
      kp, b.n_units, qblocks, 1, wl.split_len, 1, wl.mq_pad, b.row_off,
      static_cast<const uint16_t*>(b.K), static_cast<const uint16_t*>(b.Q), nullptr, nullptr, nullptr,
      nullptr, reinterpret_cast<float*>(ws + wl.parts), wl.parts_pitch);
  return hipGetLastError();
}

}  // namespace cask
