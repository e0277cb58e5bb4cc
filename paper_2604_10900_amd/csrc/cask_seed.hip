// De-duplicated seeding (an option; the paper does not say how the representatives are
// seeded, Section 2.3).  The selection has marked the best h*M scratch rows of a unit as
// provisional seeds; this kernel walks them in the order (score descending, index ascending)
// and keeps a row as a seed unless its key cosine with a seed kept before it is >= tau, until
// M seeds are kept.  Every other provisional seed becomes a donor.
#include <hip/hip_runtime.h>

#include <cstdlib>

#include "cask.h"
#include "cask_common.h"

namespace cask {

namespace {

constexpr int kDdThreads = 512;
constexpr int kDdWaves = kDdThreads / 64;
constexpr int kDdStageBytes = 16 * 1024;  // keys staged in LDS at a time, in the cache's own type

// One workgroup per unit.  The provisional seeds are collected into LDS as 64-bit keys
// (score image, inverted row) and sorted by a bitonic network; the walk then takes them 64 at
// a time, lane i of every wave holding candidate i's key in registers: the eight waves share
// out the seeds kept so far (staged through LDS 16 KB at a time) and the 64 candidates of the
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
  constexpr int kChunk = kDdStageBytes / (D * (int)sizeof(T)) < 64 ? kDdStageBytes / (D * (int)sizeof(T)) : 64;
  static_assert(64 % kChunk == 0, "a block of candidates is staged in whole chunks");
  __shared__ __align__(16) T stage[kChunk * D];
  __shared__ float stage_inv[kChunk];
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

  // rows -> LDS as they are, `cnt` of them, row index of entry j given by `which(j)`
  auto stage_rows = [&](int cnt, auto which) {
    constexpr int PPR = D * (int)sizeof(T) / 16;  // 16-byte pieces per row
    constexpr int EPP = 16 / (int)sizeof(T);      // elements per piece
    for (int q = tid; q < cnt * PPR; q += kDdThreads) {
      const int j = q / PPR, pc = q % PPR;
      *reinterpret_cast<uint4*>(&stage[j * D + pc * EPP]) =
          *reinterpret_cast<const uint4*>(Ku + (size_t)which(j) * D + pc * EPP);
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
      constexpr int EPP = 16 / (int)sizeof(T);
      float dot = 0.f;
#pragma unroll
      for (int pc = 0; pc < D / EPP; ++pc) {  // the same address in every lane: a broadcast read
        const uint4 raw = *reinterpret_cast<const uint4*>(&stage[j * D + pc * EPP]);
        const T* e = reinterpret_cast<const T*>(&raw);
#pragma unroll
        for (int x = 0; x < EPP; ++x) dot = __builtin_fmaf(c[pc * EPP + x], Elem<T>::load(e + x), dot);
      }
      return dot * inv_i * inv_j;
    };
    // the seeds kept so far
    for (int j0 = 0; j0 < n_chosen; j0 += kChunk) {
      const int cnt = n_chosen - j0 < kChunk ? n_chosen - j0 : kChunk;
      __syncthreads();  // the previous chunk has been read
      stage_rows(cnt, [&](int j) { return row_of(seed_rank[j0 + j]); });
      if (tid < cnt) stage_inv[tid] = seed_inv[j0 + tid];
      __syncthreads();
      for (int j = wv; j < cnt; j += kDdWaves) blocked = blocked || cosine(j, stage_inv[j]) >= kp.tau;
    }
    // the block's own candidates
    for (int h = 0; h < 64 / kChunk; ++h) {
      const int first = b0 + h * kChunk;
      const int cnt = Tn - first < kChunk ? (Tn - first > 0 ? Tn - first : 0) : kChunk;
      __syncthreads();
      stage_rows(cnt, [&](int j) { return row_of(first + j); });
      __syncthreads();
      for (int j = wv; j < cnt; j += kDdWaves)
        if (cosine(j, blk_inv[h * kChunk + j]) >= kp.tau) {
          const int bit = h * kChunk + j;
          if (bit < 32) m_lo |= 1u << bit; else m_hi |= 1u << (bit - 32);
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


// ------------------------------------------------------------------ bf16: cosines on MFMA

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// The same walk for bf16 caches with every cosine a 32x32x16 MFMA product, and with the order
// of the work turned round so that a row is staged in LDS once: the walk takes its sorted rows
// 64 at a time; the block's rows are staged (padded pitch: operand reads are conflict-free),
// four waves form the block's own 64 x 64 cosines (a row's mask of earlier block mates it
// resembles), wave 0 resolves the block in rank order against the rows' "resembles a kept
// seed" bits, and then all waves compare the rows of the later blocks (operands straight from
// global memory, the two lane halves holding the two halves of the head dimension for both
// operands) with the seeds this block kept and set those bits for them.  Inverse norms of
// all rows are formed once up front.
template <int D>
__global__ __launch_bounds__(kDdThreads) void dedup_seed_mfma_kernel(
    KParams kp, const int64_t* __restrict__ row_off, const int32_t* __restrict__ prefix_len,
    const uint16_t* __restrict__ K, const float* __restrict__ scores, uint8_t* __restrict__ role) {
  constexpr int KS = D / 16;
  constexpr int kPitch = D * 2 + 16;  // bytes per staged row
  __shared__ uint64_t keys[kSeedWalkMax];
  __shared__ __align__(16) float inv_norm[kSeedWalkMax];
  __shared__ uint32_t blocked[kSeedWalkMax / 32];
  __shared__ uint8_t is_seed[kSeedWalkMax];
  __shared__ __align__(16) unsigned char stage[64 * kPitch];
  __shared__ uint32_t mates[64 * 2];
  __shared__ uint32_t kept_s[2];
  __shared__ int n_cand, n_chosen_s;
  const int u = blockIdx.x, tid = threadIdx.x, wv = tid >> 6, lane = tid & 63;
  const int c32 = lane & 31, hh = lane >> 5;
  const int64_t row0 = row_off[u];
  const int N = (int)(row_off[u + 1] - row0);
  const int P = prefix_len[u];
  const UnitPlan pl = make_plan(kp, P, N);
  const int hi = N - pl.r_eff, n = hi - P, C = pl.core, M = pl.seeds;
  if ((pl.status & CASK_ST_PREFIX_BUDGET_EXHAUSTED) || M <= 0 || n <= C + M) return;
  const float* s = scores + row0;
  uint8_t* ro = role + row0;
  const uint16_t* Ku = K + row0 * D;

  if (tid == 0) n_cand = 0;
  __syncthreads();
  for (int i = P + tid; i < hi; i += kDdThreads)
    if (ro[i] == CASK_ROLE_SEED) {
      const int k = atomicAdd(&n_cand, 1);
      if (k < kSeedWalkMax) keys[k] = ((uint64_t)score_key(s[i]) << 32) | (uint32_t)~(uint32_t)i;
    }
  __syncthreads();
  const int Tn = n_cand < kSeedWalkMax ? n_cand : kSeedWalkMax;
  int n_pad = 2;
  while (n_pad < Tn) n_pad <<= 1;
  for (int k = Tn + tid; k < n_pad; k += kDdThreads) keys[k] = 0ull;
  for (int k = tid; k < kSeedWalkMax; k += kDdThreads) is_seed[k] = 0;
  for (int k = tid; k < kSeedWalkMax / 32; k += kDdThreads) blocked[k] = 0u;
  if (tid < 128) mates[tid] = 0u;
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
  // inverse norms, one row per thread and turn
  for (int k = tid; k < Tn; k += kDdThreads) {
    const uint16_t* kr = Ku + (size_t)row_of(k) * D;
    float nn = 0.f;
#pragma unroll
    for (int pc = 0; pc < D / 8; ++pc) {
      const u32x4 raw = *reinterpret_cast<const u32x4*>(kr + pc * 8);
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const float a = __uint_as_float(raw[w] << 16), b = __uint_as_float(raw[w] & 0xffff0000u);
        nn = __builtin_fmaf(a, a, nn);
        nn = __builtin_fmaf(b, b, nn);
      }
    }
    inv_norm[k] = nn > 0.f ? 1.f / sqrtf(nn) : 0.f;
  }
  __syncthreads();

  // B operand: staged row `col`, k-step ks, of this lane's half of the head dimension
  auto staged = [&](int col, int ks) {
    return __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(stage + col * kPitch + hh * D + ks * 16));
  };
  const int n_blocks = (Tn + 63) >> 6;
  int n_chosen = 0;
  for (int blk = 0; blk < n_blocks && n_chosen < M; ++blk) {
    const int b0 = blk << 6;
    // the block's rows into LDS (ranks past the end repeat the last row; they are masked)
    for (int q = tid; q < 64 * (D / 8); q += kDdThreads) {
      const int j = q / (D / 8), pc = q % (D / 8);
      const int rank = b0 + j < Tn ? b0 + j : Tn - 1;
      *reinterpret_cast<u32x4*>(stage + j * kPitch + pc * 16) =
          *reinterpret_cast<const u32x4*>(Ku + (size_t)row_of(rank) * D + pc * 8);
    }
    __syncthreads();
    if (wv < 4) {  // the block's own cosines: row tile wv / 2 against column tile wv % 2
      const int rt = wv >> 1, ct = wv & 1;
      if (ct <= rt) {  // only earlier mates matter: column tile 1 never precedes row tile 0
        f32x16 acc = {0};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
          acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(staged(rt * 32 + c32, ks), staged(ct * 32 + c32, ks), acc, 0, 0, 0);
        const int j = ct * 32 + c32;  // this lane's column: the candidate mate
        const float inv_j = inv_norm[b0 + j < Tn ? b0 + j : Tn - 1];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int i = rt * 32 + (r >> 2) * 8 + hh * 4 + (r & 3);
          if (j < i && b0 + i < Tn && acc[r] * inv_norm[b0 + i] * inv_j >= kp.tau)
            atomicOr(&mates[i * 2 + (j >> 5)], 1u << (j & 31));
        }
      }
    }
    __syncthreads();
    if (wv == 0) {
      const int me = b0 + lane;
      const bool valid = me < Tn;
      const bool bl = (blocked[(me & (kSeedWalkMax - 1)) >> 5] >> (me & 31)) & 1u;
      const uint64_t mt = ((uint64_t)mates[lane * 2 + 1] << 32) | mates[lane * 2];
      uint64_t kept = 0ull;
      int cnt = n_chosen;
      for (int i = 0; i < 64; ++i) {  // rank order inside the block
        const int ok = (valid && !bl && (mt & kept) == 0ull) ? 1 : 0;
        if (__shfl(ok, i, 64) && cnt < M) {
          kept |= 1ull << i;
          if (lane == i) is_seed[me] = 1;
          ++cnt;
        }
      }
      mates[lane * 2] = 0u;
      mates[lane * 2 + 1] = 0u;
      if (lane == 0) {
        n_chosen_s = cnt;
        kept_s[0] = (uint32_t)kept;
        kept_s[1] = (uint32_t)(kept >> 32);
      }
    }
    __syncthreads();
    n_chosen = n_chosen_s;
    const uint32_t kept_lo = kept_s[0], kept_hi = kept_s[1];
    if (n_chosen < M && (kept_lo | kept_hi) != 0u) {
      // rows of the later blocks against the seeds this block kept: 32-row tiles, dealt to the waves
      const int n_tiles = (n_blocks - blk - 1) * 2;
      for (int t = wv; t < n_tiles; t += kDdWaves) {
        const int first = b0 + 64 + t * 32;
        if (first >= Tn) continue;
        const int rank = first + c32 < Tn ? first + c32 : Tn - 1;
        const uint16_t* kr = Ku + (size_t)row_of(rank) * D + hh * (D / 2);
        bf16x8 a[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
          a[ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(kr + ks * 8));
        uint32_t hit = 0u;  // bit r: row r of this lane's sixteen resembles a kept seed
#pragma unroll
        for (int ct = 0; ct < 2; ++ct) {
          const uint32_t kept_half = ct == 0 ? kept_lo : kept_hi;
          if (kept_half == 0u) continue;
          f32x16 acc = {0};
#pragma unroll
          for (int ks = 0; ks < KS; ++ks)
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ks], staged(ct * 32 + c32, ks), acc, 0, 0, 0);
          if ((kept_half >> c32) & 1u) {
            const float inv_j = inv_norm[b0 + ct * 32 + c32];
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              const int i = first + (r >> 2) * 8 + hh * 4 + (r & 3);
              if (i < Tn && acc[r] * inv_norm[i & (kSeedWalkMax - 1)] * inv_j >= kp.tau) hit |= 1u << r;
            }
          }
        }
#pragma unroll
        for (int r = 0; r < 16; ++r)
          if ((hit >> r) & 1u) {
            const int i = first + (r >> 2) * 8 + hh * 4 + (r & 3);
            atomicOr(&blocked[i >> 5], 1u << (i & 31));
          }
      }
    }
    __syncthreads();
  }
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
  } else if (kp.path_flags & CASK_PATH_DEDUP_VECTOR) {  // the vector-ALU kernel, for comparisons
    if (kp.d == 64) CASK_DD(uint16_t, 64); else CASK_DD(uint16_t, 128);
  } else if (kp.d == 64) {
    dedup_seed_mfma_kernel<64><<<dim3(b.n_units), dim3(kDdThreads), 0, st>>>(
        kp, b.row_off, b.prefix_len, static_cast<const uint16_t*>(b.K), scores, role);
  } else {
    dedup_seed_mfma_kernel<128><<<dim3(b.n_units), dim3(kDdThreads), 0, st>>>(
        kp, b.row_off, b.prefix_len, static_cast<const uint16_t*>(b.K), scores, role);
  }
#undef CASK_DD
  return hipGetLastError();
}

}  // namespace cask
