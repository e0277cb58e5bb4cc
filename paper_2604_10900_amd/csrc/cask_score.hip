// Scoring: s_j = mean over the W*G window rows of softmax_j(scale <q, k_j>), the scalar
// importance used as local score mass a_i (Sections 1 and 2.4 of the paper).
//
// The softmax normaliser of a row needs all keys before any column can be summed, so the
// score takes two sweeps of Q.K^T:
//   sweep A (row statistics)  per window row: running max and sum of exp2 over key splits;
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
__device__ inline void fill_neg_lse(const float2* __restrict__ part, int n_splits, int mq_pad,
                                    int Mq, float* negL, int tid, int nthreads) {
  for (int r = tid; r < mq_pad; r += nthreads) {
    float v = kNegInf;
    if (r < Mq) {
      float m = kNegInf, l = 0.f;
      for (int s = 0; s < n_splits; ++s) {
        const float2 p = part[(size_t)s * mq_pad + r];
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

constexpr int kD = 128;
constexpr int kPitch = 272;  // LDS row pitch in bytes: 256 + 16 keeps b128 reads conflict-free

template <int MODE>
struct Geo;
template <>
struct Geo<0> {  // sweep A: resident = window rows (Q), stream = keys (K)
  static constexpr int RES_ROWS = 128, STAGE_ROWS = 128;  // 2 resident x 2 stream wave groups
};
template <>
struct Geo<1> {  // sweep B: resident = keys (K), stream = window rows (Q)
  static constexpr int RES_ROWS = 256, STAGE_ROWS = 64;   // 4 resident wave groups
};

template <int MODE>
__global__ __launch_bounds__(256) void score_mfma_kernel(
    KParams kp, int n_units, int tiles_per_unit, int n_splits, int split_len, int mq_pad,
    const int64_t* __restrict__ row_off, const uint16_t* __restrict__ K,
    const uint16_t* __restrict__ Q, float2* __restrict__ rowstat, float* __restrict__ scores) {
  using G_ = Geo<MODE>;
  constexpr int STAGE_ROWS = G_::STAGE_ROWS;
  constexpr int CHUNKS = STAGE_ROWS * 16 / 256;  // 16-byte chunks per thread per stage
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  unsigned char* stage0 = smem;
  unsigned char* stage1 = smem + STAGE_ROWS * kPitch;
  float* negL = reinterpret_cast<float*>(smem + 2 * STAGE_ROWS * kPitch);  // MODE 1 only
  float* xchg = negL;                                                     // MODE 0 only

  int unit, tile;
  if (!map_block(n_units, tiles_per_unit, unit, tile)) return;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int c32 = lane & 31, h = lane >> 5;
  const int rgrp = (MODE == 0) ? (wv & 1) : wv;
  const int sgrp = (MODE == 0) ? (wv >> 1) : 0;
  const int64_t row0 = row_off[unit];
  const int N = (int)(row_off[unit + 1] - row0);
  const int Mq = kp.Mq, W = kp.W, Gq = kp.G;
  const float c = kp.scale_log2;
  const uint16_t* Ku = K + (size_t)row0 * kD;
  const uint16_t* Qu = Q + (size_t)unit * Mq * kD;
  float2* part = rowstat + (size_t)unit * n_splits * mq_pad;

  // ---- what this workgroup covers
  const uint16_t* res_ptr;
  const uint16_t* str_ptr;
  int res_base, res_limit, s_begin, s_end;  // resident rows [res_base, ..), stream rows [s_begin, s_end)
  int split = 0;
  if (MODE == 0) {
    const int qb = tile / n_splits;
    split = tile % n_splits;
    res_base = qb * G_::RES_ROWS;
    if (res_base >= Mq) return;
    res_ptr = Qu;
    res_limit = Mq;
    str_ptr = Ku;
    s_begin = split * split_len;
    s_end = min(N, s_begin + split_len);
    if (kp.causal) {
      const int last_row = min(Mq, res_base + G_::RES_ROWS) - 1;
      s_end = min(s_end, N - W + last_row / Gq + 1);
    }
  } else {
    res_base = tile * G_::RES_ROWS;
    if (res_base >= N) return;
    res_ptr = Ku;
    res_limit = N;
    str_ptr = Qu;
    s_begin = 0;
    s_end = Mq;
    if (kp.causal && res_base > N - W) s_begin = (((res_base - (N - W)) * Gq) / STAGE_ROWS) * STAGE_ROWS;
    fill_neg_lse(part, n_splits, mq_pad, Mq, negL, tid, 256);
  }

  // ---- resident fragments: lane (c32, h) holds row c32 of each 32-row tile, k-chunk h
  bf16x8 bres[2][8];
  int res_row[2];
#pragma unroll
  for (int ct = 0; ct < 2; ++ct) {
    const int r = res_base + rgrp * 64 + ct * 32 + c32;
    res_row[ct] = r;
    const bool ok = r < res_limit;
    const uint4* src = reinterpret_cast<const uint4*>(res_ptr + (size_t)(ok ? r : 0) * kD) + h;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      uint4 v = ok ? src[ks * 2] : make_uint4(0, 0, 0, 0);
      bres[ct][ks] = *reinterpret_cast<bf16x8*>(&v);
    }
  }

  // per-lane reduction state
  float m_run[2] = {kNegInf, kNegInf}, l_run[2] = {0.f, 0.f};  // sweep A
  float colsum[2] = {0.f, 0.f};                                  // sweep B
  int vis_limit[2];  // sweep A: last key the lane's window row sees; sweep B: the lane's key
#pragma unroll
  for (int ct = 0; ct < 2; ++ct)
    vis_limit[ct] = (MODE == 0) ? (kp.causal ? N - W + res_row[ct] / Gq : N - 1) : res_row[ct];
  const int tail_start = kp.causal ? N - W : N;  // keys > tail_start are hidden from some row

  const int n_stages = (s_end - s_begin + STAGE_ROWS - 1) / STAGE_ROWS;
  uint4 pre[CHUNKS];
  auto fetch = [&](int stage) {
    const int base = s_begin + stage * STAGE_ROWS;
#pragma unroll
    for (int i = 0; i < CHUNKS; ++i) {
      const int q = tid + 256 * i;
      const int r = base + (q >> 4);
      pre[i] = (r < s_end) ? reinterpret_cast<const uint4*>(str_ptr + (size_t)r * kD)[q & 15]
                           : make_uint4(0, 0, 0, 0);
    }
  };
  auto stash = [&](unsigned char* buf) {
#pragma unroll
    for (int i = 0; i < CHUNKS; ++i) {
      const int q = tid + 256 * i;
      *reinterpret_cast<uint4*>(buf + (q >> 4) * kPitch + (q & 15) * 16) = pre[i];
    }
  };

  if (n_stages > 0) {
    fetch(0);
    stash(stage0);
  }
  __syncthreads();

  for (int it = 0; it < n_stages; ++it) {
    unsigned char* cur = (it & 1) ? stage1 : stage0;
    unsigned char* nxt = (it & 1) ? stage0 : stage1;
    if (it + 1 < n_stages) fetch(it + 1);
    const int stage_row0 = s_begin + it * STAGE_ROWS + sgrp * 64;
#pragma unroll
    for (int rt = 0; rt < 2; ++rt) {
      const int trow0 = stage_row0 + rt * 32;  // stream index of this tile's row 0
      if (trow0 >= s_end) continue;
      bf16x8 a[8];
      const unsigned char* ap = cur + (sgrp * 64 + rt * 32 + c32) * kPitch + h * 16;
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) a[ks] = *reinterpret_cast<const bf16x8*>(ap + ks * 32);
#pragma unroll
      for (int ct = 0; ct < 2; ++ct) {
        f32x16 acc = {0};
#pragma unroll
        for (int ks = 0; ks < 8; ++ks)
          acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ks], bres[ct][ks], acc, 0, 0, 0);
        if (MODE == 0) {
          // stream rows are keys; the lane's column is one window row
          const bool slow = (trow0 + 31 > tail_start) || (trow0 + 32 > s_end);
          if (slow) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              const int key = trow0 + (r >> 2) * 8 + h * 4 + (r & 3);
              if (!(key < s_end && key <= vis_limit[ct])) acc[r] = kNegInf;
            }
          }
          float xm = acc[0];
#pragma unroll
          for (int r = 1; r < 16; ++r) xm = fmaxf(xm, acc[r]);
          const float m_new = fmaxf(m_run[ct], xm * c);
          const float nm = (m_new == kNegInf) ? 0.f : -m_new;
          float sum = 0.f;
#pragma unroll
          for (int r = 0; r < 16; ++r) sum += fast_exp2(__builtin_fmaf(acc[r], c, nm));
          l_run[ct] = l_run[ct] * fast_exp2(m_run[ct] + nm) + sum;
          m_run[ct] = m_new;
        } else {
          // stream rows are window rows; the lane's column is one key
          const bool slow = kp.causal && (res_base + G_::RES_ROWS - 1 > tail_start);
          float sum = 0.f;
#pragma unroll
          for (int g4 = 0; g4 < 4; ++g4) {
            const int rowb = trow0 + g4 * 8 + h * 4;
            const float4 nl = *reinterpret_cast<const float4*>(negL + rowb);
            const float nls[4] = {nl.x, nl.y, nl.z, nl.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              float y = __builtin_fmaf(acc[g4 * 4 + e], c, nls[e]);
              if (slow) {
                const int tw = N - W + (rowb + e) / Gq;
                if (vis_limit[ct] > tw) y = kNegInf;
              }
              sum += fast_exp2(y);
            }
          }
          colsum[ct] += sum;
        }
      }
    }
    if (it + 1 < n_stages) stash(nxt);
    __syncthreads();
  }

  // ---- finish
  if (MODE == 0) {
#pragma unroll
    for (int ct = 0; ct < 2; ++ct) {
      const float m2 = __shfl_xor(m_run[ct], 32, 64);
      const float l2 = __shfl_xor(l_run[ct], 32, 64);
      ml_combine(m_run[ct], l_run[ct], m2, l2);
    }
    float2* x2 = reinterpret_cast<float2*>(xchg);
    if (sgrp == 1 && h == 0) {
#pragma unroll
      for (int ct = 0; ct < 2; ++ct) x2[rgrp * 64 + ct * 32 + c32] = make_float2(m_run[ct], l_run[ct]);
    }
    __syncthreads();
    if (sgrp == 0 && h == 0) {
#pragma unroll
      for (int ct = 0; ct < 2; ++ct) {
        const float2 o = x2[rgrp * 64 + ct * 32 + c32];
        ml_combine(m_run[ct], l_run[ct], o.x, o.y);
        if (res_row[ct] < Mq) part[(size_t)split * mq_pad + res_row[ct]] = make_float2(m_run[ct], l_run[ct]);
      }
    }
  } else {
    const float inv = 1.0f / (float)Mq;
#pragma unroll
    for (int ct = 0; ct < 2; ++ct) {
      const float tot = colsum[ct] + __shfl_xor(colsum[ct], 32, 64);
      if (h == 0 && res_row[ct] < N) scores[row0 + res_row[ct]] = tot * inv;
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
  fill_neg_lse(rowstat + (size_t)unit * n_splits * mq_pad, n_splits, mq_pad, Mq, negL, tid, 256);
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
                      float* scores, hipStream_t st) {
  float2* rowstat = reinterpret_cast<float2*>(ws + wl.rowstat);
  const int units8 = (b.n_units + 7) / 8 * 8;
  const int qblocks = (kp.Mq + 63) / 64;
  const int tilesA = qblocks * wl.n_splits;
  score_rows_fma_kernel<T, D><<<dim3(units8 * tilesA), dim3(256), 0, st>>>(
      kp, b.n_units, tilesA, wl.n_splits, wl.split_len, wl.mq_pad, b.row_off,
      static_cast<const T*>(b.K), static_cast<const T*>(b.Q), rowstat);
  const int tilesB = (b.max_unit_len + 255) / 256;
  score_cols_fma_kernel<T, D><<<dim3(units8 * tilesB), dim3(256), wl.mq_pad * sizeof(float), st>>>(
      kp, b.n_units, tilesB, wl.n_splits, wl.mq_pad, b.row_off, static_cast<const T*>(b.K),
      static_cast<const T*>(b.Q), rowstat, scores);
  return hipGetLastError();
}

}  // namespace

bool score_uses_mfma(const KParams& kp) {
  return kp.dtype == CASK_BF16 && kp.d == 128 && kp.Mq <= 8192;
}

hipError_t launch_score(const KParams& kp, const Batch& b, const Workspace& wl, char* ws,
                        float* scores, hipStream_t st) {
  if (!score_uses_mfma(kp)) {
    if (kp.dtype == CASK_F32)
      return kp.d == 64 ? launch_fma<float, 64>(kp, b, wl, ws, scores, st)
                        : launch_fma<float, 128>(kp, b, wl, ws, scores, st);
    return kp.d == 64 ? launch_fma<uint16_t, 64>(kp, b, wl, ws, scores, st)
                      : launch_fma<uint16_t, 128>(kp, b, wl, ws, scores, st);
  }
  float2* rowstat = reinterpret_cast<float2*>(ws + wl.rowstat);
  const int units8 = (b.n_units + 7) / 8 * 8;
  const uint16_t* K = static_cast<const uint16_t*>(b.K);
  const uint16_t* Q = static_cast<const uint16_t*>(b.Q);
  static bool attr_set = false;
  const size_t ldsA = 2 * Geo<0>::STAGE_ROWS * kPitch + 128 * sizeof(float2);
  const size_t ldsB = 2 * Geo<1>::STAGE_ROWS * kPitch + (size_t)wl.mq_pad * sizeof(float);
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&score_mfma_kernel<0>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(&score_mfma_kernel<1>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const int qblocks = (kp.Mq + Geo<0>::RES_ROWS - 1) / Geo<0>::RES_ROWS;
  const int tilesA = qblocks * wl.n_splits;
  score_mfma_kernel<0><<<dim3(units8 * tilesA), dim3(256), ldsA, st>>>(
      kp, b.n_units, tilesA, wl.n_splits, wl.split_len, wl.mq_pad, b.row_off, K, Q, rowstat,
      scores);
  const int tilesB = (b.max_unit_len + Geo<1>::RES_ROWS - 1) / Geo<1>::RES_ROWS;
  score_mfma_kernel<1><<<dim3(units8 * tilesB), dim3(256), ldsB, st>>>(
      kp, b.n_units, tilesB, wl.n_splits, wl.split_len, wl.mq_pad, b.row_off, K, Q, rowstat,
      scores);
  return hipGetLastError();
}

}  // namespace cask
