// De-duplicated seeding (an option; the paper does not say how the representatives are
// seeded, Section 2.3).  The selection has marked the best h*M scratch rows of a unit as
// provisional seeds; this kernel walks them in the order (score descending, index ascending)
// and keeps a row as a seed unless its key cosine with a seed kept before it is >= tau, until
// M seeds are kept.  Every other provisional seed becomes a donor.
#include <hip/hip_runtime.h>

#include "cask.h"
#include "cask_common.h"

namespace cask {

namespace {

constexpr int kDdThreads = 512;
constexpr int kDdWaves = kDdThreads / 64;
constexpr int kDdChunk = 32;  // keys staged in LDS at a time

// One workgroup per unit.  The provisional seeds are collected into LDS as 64-bit keys
// (score image, inverted row) and sorted by a bitonic network; the walk then takes them 64 at
// a time, lane i of every wave holding candidate i's key in registers: the eight waves share
// out the seeds kept so far (staged through LDS 32 at a time) and the 64 candidates of the
// block themselves, each lane collects "resembles a kept seed" and a 64-bit mask of the block
// mates it resembles, and wave 0 resolves the block in rank order (a candidate is kept unless
// it resembles a kept seed or a block mate kept before it).  The walk is sequential by
// definition; only the cosines are parallel.
template <typename T, int D>
__global__ __launch_bounds__(kDdThreads) void dedup_seed_kernel(
    KParams kp, const int64_t* __restrict__ row_off, const int32_t* __restrict__ prefix_len,
    const T* __restrict__ K, const float* __restrict__ scores, uint8_t* __restrict__ role) {
  __shared__ uint64_t keys[kSeedWalkMax];
  __shared__ int32_t seed_rank[kSeedWalkMax];
  __shared__ float seed_inv[kSeedWalkMax];
  __shared__ __align__(16) float stage[kDdChunk * D];
  __shared__ float stage_inv[kDdChunk];
  __shared__ float blk_inv[64];
  __shared__ uint32_t blocked_w[kDdWaves * 64];
  __shared__ uint32_t mask_w[kDdWaves * 64 * 2];
  __shared__ uint8_t is_seed[kSeedWalkMax];
  __shared__ int n_cand, n_chosen_s;
  const int u = blockIdx.x, tid = threadIdx.x, wv = tid >> 6, lane = tid & 63;
  const int64_t row0 = row_off[u];
  const int N = (int)(row_off[u + 1] - row0);
  const int P = prefix_len[u];
  const UnitPlan pl = make_plan(kp, P, N);
  const int hi = N - pl.r_eff, n = hi - P, C = pl.core, M = pl.seeds;
  // the same condition under which the selection widened its seed range
  if ((pl.status & CASK_ST_PREFIX_BUDGET_EXHAUSTED) || M <= 0 || n <= C + M) return;
  const float* s = scores + row0;
  uint8_t* ro = role + row0;
  const T* Ku = K + row0 * D;

  if (tid == 0) n_cand = 0;
  __syncthreads();
  for (int i = P + tid; i < hi; i += kDdThreads)
    if (ro[i] == CASK_ROLE_SEED) {
      const int k = atomicAdd(&n_cand, 1);  // the order of arrival does not matter: sorted next
      if (k < kSeedWalkMax) keys[k] = ((uint64_t)score_key(s[i]) << 32) | (uint32_t)~(uint32_t)i;
    }
  __syncthreads();
  const int Tn = n_cand < kSeedWalkMax ? n_cand : kSeedWalkMax;
  int n_pad = 2;
  while (n_pad < Tn) n_pad <<= 1;
  for (int k = Tn + tid; k < n_pad; k += kDdThreads) keys[k] = 0ull;  // below every real key
  for (int k = tid; k < kSeedWalkMax; k += kDdThreads) is_seed[k] = 0;
  __syncthreads();
  for (int size = 2; size <= n_pad; size <<= 1)
    for (int stride = size >> 1; stride > 0; stride >>= 1) {
      for (int t = tid; t < (n_pad >> 1); t += kDdThreads) {
        const int i = ((t / stride) * 2 * stride) + (t % stride), j = i + stride;
        const bool desc = (i & size) == 0;
        const uint64_t a = keys[i], b = keys[j];
        if ((a < b) == desc) {
          keys[i] = b;
          keys[j] = a;
        }
      }
      __syncthreads();
    }
  auto row_of = [&](int rank) { return (int)(~(uint32_t)keys[rank]); };

  // rows -> LDS as floats, `cnt` of them, row index of entry j given by `which(j)`
  auto stage_rows = [&](int cnt, auto which) {
    constexpr int PPR = D * (int)sizeof(T) / 16;  // 16-byte pieces per row
    constexpr int EPP = 16 / (int)sizeof(T);      // elements per piece
    for (int q = tid; q < cnt * PPR; q += kDdThreads) {
      const int j = q / PPR, pc = q % PPR;
      const uint4 raw = *reinterpret_cast<const uint4*>(Ku + (size_t)which(j) * D + pc * EPP);
      const T* e = reinterpret_cast<const T*>(&raw);
#pragma unroll
      for (int x = 0; x < EPP; ++x) stage[j * D + pc * EPP + x] = Elem<T>::load(e + x);
    }
  };

  int n_chosen = 0;
  for (int b0 = 0; b0 < Tn && n_chosen < M; b0 += 64) {
    const int me = b0 + lane;
    const bool valid = me < Tn;
    const int my_row = row_of(valid ? me : b0);
    float c[D];
    float nn = 0.f;
    {
      constexpr int EPP = 16 / (int)sizeof(T);
#pragma unroll
      for (int pc = 0; pc < D / EPP; ++pc) {
        const uint4 raw = *reinterpret_cast<const uint4*>(Ku + (size_t)my_row * D + pc * EPP);
        const T* e = reinterpret_cast<const T*>(&raw);
#pragma unroll
        for (int x = 0; x < EPP; ++x) {
          c[pc * EPP + x] = Elem<T>::load(e + x);
          nn = __builtin_fmaf(c[pc * EPP + x], c[pc * EPP + x], nn);
        }
      }
    }
    const float inv_i = nn > 0.f ? 1.f / sqrtf(nn) : 0.f;
    if (wv == 0) blk_inv[lane] = inv_i;
    bool blocked = false;
    uint32_t m_lo = 0u, m_hi = 0u;
    auto cosine = [&](int j, float inv_j) {
      float dot = 0.f;
#pragma unroll
      for (int e4 = 0; e4 < D / 4; ++e4) {
        const float4 k4 = *reinterpret_cast<const float4*>(&stage[j * D + e4 * 4]);
        dot = __builtin_fmaf(c[e4 * 4 + 0], k4.x, dot);
        dot = __builtin_fmaf(c[e4 * 4 + 1], k4.y, dot);
        dot = __builtin_fmaf(c[e4 * 4 + 2], k4.z, dot);
        dot = __builtin_fmaf(c[e4 * 4 + 3], k4.w, dot);
      }
      return dot * inv_i * inv_j;
    };
    // the seeds kept so far
    for (int j0 = 0; j0 < n_chosen; j0 += kDdChunk) {
      const int cnt = n_chosen - j0 < kDdChunk ? n_chosen - j0 : kDdChunk;
      __syncthreads();  // the previous chunk has been read
      stage_rows(cnt, [&](int j) { return row_of(seed_rank[j0 + j]); });
      if (tid < cnt) stage_inv[tid] = seed_inv[j0 + tid];
      __syncthreads();
      for (int j = wv; j < cnt; j += kDdWaves) blocked = blocked || cosine(j, stage_inv[j]) >= kp.tau;
    }
    // the block's own candidates, 32 at a time
    for (int h = 0; h < 2; ++h) {
      const int first = b0 + h * 32;
      const int cnt = Tn - first < 32 ? (Tn - first > 0 ? Tn - first : 0) : 32;
      __syncthreads();
      stage_rows(cnt, [&](int j) { return row_of(first + j); });
      __syncthreads();
      for (int j = wv; j < cnt; j += kDdWaves)
        if (cosine(j, blk_inv[h * 32 + j]) >= kp.tau) {
          if (h == 0) m_lo |= 1u << j; else m_hi |= 1u << j;
        }
    }
    blocked_w[wv * 64 + lane] = blocked ? 1u : 0u;
    mask_w[(wv * 64 + lane) * 2] = m_lo;
    mask_w[(wv * 64 + lane) * 2 + 1] = m_hi;
    __syncthreads();
    if (wv == 0) {
      uint32_t bl = 0u, lo = 0u, hi32 = 0u;
      for (int w = 0; w < kDdWaves; ++w) {
        bl |= blocked_w[w * 64 + lane];
        lo |= mask_w[(w * 64 + lane) * 2];
        hi32 |= mask_w[(w * 64 + lane) * 2 + 1];
      }
      const uint64_t mates = ((uint64_t)hi32 << 32) | lo;
      uint64_t kept = 0ull;
      int cnt = n_chosen;
      for (int i = 0; i < 64; ++i) {  // rank order inside the block
        const int ok = (valid && !bl && (mates & kept) == 0ull) ? 1 : 0;
        if (__shfl(ok, i, 64) && cnt < M) {
          kept |= 1ull << i;
          if (lane == i) {
            seed_rank[cnt] = me;
            seed_inv[cnt] = inv_i;
            is_seed[me] = 1;
          }
          ++cnt;
        }
      }
      if (lane == 0) n_chosen_s = cnt;
    }
    __syncthreads();
    n_chosen = n_chosen_s;
  }
  // every provisional seed becomes a donor, then the kept ones are restored
  for (int i = P + tid; i < hi; i += kDdThreads)
    if (ro[i] == CASK_ROLE_SEED) ro[i] = CASK_ROLE_DONOR;
  __syncthreads();
  for (int k = tid; k < Tn; k += kDdThreads)
    if (is_seed[k]) ro[row_of(k)] = CASK_ROLE_SEED;
}

}  // namespace

hipError_t launch_dedup_seeds(const KParams& kp, const Batch& b, const float* scores, uint8_t* role,
                              hipStream_t st) {
  if (b.n_units == 0 || kp.dedup <= 0) return hipSuccess;
#define CASK_DD(T, D)                                                              \
  dedup_seed_kernel<T, D><<<dim3(b.n_units), dim3(kDdThreads), 0, st>>>(           \
      kp, b.row_off, b.prefix_len, static_cast<const T*>(b.K), scores, role)
  if (kp.dtype == CASK_F32) {
    if (kp.d == 64) CASK_DD(float, 64); else CASK_DD(float, 128);
  } else {
    if (kp.d == 64) CASK_DD(uint16_t, 64); else CASK_DD(uint16_t, 128);
  }
#undef CASK_DD
  return hipGetLastError();
}

}  // namespace cask
