// Selective consolidation of the mergeable scratch (Sections 2.1, 2.4, 2.5 of the paper):
//   similarity   every donor against every seed of its unit by key cosine; best seed kept
//                when the cosine reaches tau (bf16 d=128: MFMA contraction seeds x donors^T,
//                each lane owns one donor and scans its seeds in ascending order);
//   gather       ordered list of the donors that merge (ascending row), per unit;
//   emit         one wavefront per output row: kept tokens are copied bit for bit, a seed
//                with donors becomes the weighted fold m = sum a_i, k~ = sum a_i k_i / m,
//                v~ = sum a_i v_i / m with a_i the token's score, accumulated in fp32 in
//                ascending row order (fixed order: reruns are bitwise identical).
#include "cask_common.h"

namespace cask {

namespace {

constexpr float kNegInf = -__builtin_inff();

__device__ inline bool better(float sim, int ord, float best, int best_ord) {
  return sim > best || (sim == best && ord < best_ord);
}

// ------------------------------------------------------------------ similarity, MFMA path

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
constexpr int kD = 128;
constexpr int kPitch = 272;
constexpr int kSeedStage = 64;    // seeds per MFMA pass (two 32-row tiles)
constexpr int kSeedBlock = 256;   // seeds held in LDS at a time
constexpr int kDonorTile = 256;   // donor rows per tile (4 waves x 64)

__device__ inline float sumsq_bf16x8(const uint4& v) {
  const uint32_t w[4] = {v.x, v.y, v.z, v.w};
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const float lo = __uint_as_float(w[i] << 16);
    const float hi = __uint_as_float(w[i] & 0xFFFF0000u);
    s = __builtin_fmaf(lo, lo, s);
    s = __builtin_fmaf(hi, hi, s);
  }
  return s;
}

// Workgroup = `tiles_per_wg` consecutive donor tiles of one unit.  The unit's seeds (up to
// kSeedBlock of them; more are taken block by block) sit in LDS with their inverse norms; the
// donors of a tile are MFMA B-operands in registers (lane = donor), and the loads of the next
// tile are issued before the current one is contracted, so the kernel streams K at memory
// speed instead of paying a round trip per tile.
__global__ __launch_bounds__(256, 2) void similarity_mfma_kernel(
    KParams kp, int n_units, int chunks_per_unit, int tiles_per_wg,
    const int64_t* __restrict__ row_off, const int32_t* __restrict__ prefix_len,
    const uint16_t* __restrict__ K, const uint8_t* __restrict__ role,
    const int32_t* __restrict__ seed_rows, const int32_t* __restrict__ n_seeds,
    int32_t* __restrict__ assign_ord) {
  __shared__ __attribute__((aligned(16))) unsigned char stage[kSeedBlock * kPitch];
  __shared__ float seed_inv[kSeedBlock];
  const int bid = blockIdx.x;
  const int xcd = bid & 7, kk = bid >> 3;
  const int u = (kk / chunks_per_unit) * 8 + xcd;
  const int chunk = kk % chunks_per_unit;
  if (u >= n_units) return;
  const int64_t row0 = row_off[u];
  const int N = (int)(row_off[u + 1] - row0);
  const int P = prefix_len[u];
  const UnitPlan pl = make_plan(kp, P, N);
  const int hi = N - pl.r_eff;
  const int first = P + chunk * tiles_per_wg * kDonorTile;
  if (first >= hi) return;
  const int n_tiles = min(tiles_per_wg, (hi - first + kDonorTile - 1) / kDonorTile);
  const int M = n_seeds[u];
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int c32 = lane & 31, h = lane >> 5;
  const uint16_t* Ku = K + (size_t)row0 * kD;
  const uint8_t* ro = role + row0;
  const int32_t* srow = seed_rows + (size_t)u * kp.B;

  // donors of a tile: lane (c32, h) holds row c32 of each 32-row half, k-chunk h
  uint4 draw[2][8];
  auto fetch_donors = [&](int t) {
#pragma unroll
    for (int ct = 0; ct < 2; ++ct) {
      const int r = first + t * kDonorTile + wv * 64 + ct * 32 + c32;
      const uint4* src = reinterpret_cast<const uint4*>(Ku + (size_t)(r < hi ? r : P) * kD) + h;
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) draw[ct][ks] = src[ks * 2];
    }
  };
  // seeds [sb, sb + kSeedBlock) -> LDS, 64 at a time (16 threads per row), with inverse norms;
  // rows past M are zero
  auto stage_seeds = [&](int sb) {
    for (int s0 = 0; s0 < kSeedBlock && sb + s0 < M; s0 += kSeedStage) {
      constexpr int kLoads = kSeedStage * 16 / 256;
      int idx[kLoads];
      uint4 v[kLoads];
#pragma unroll
      for (int i = 0; i < kLoads; ++i) {
        const int ord = sb + s0 + ((tid + 256 * i) >> 4);
        idx[i] = ord < M ? srow[ord] : -1;
      }
#pragma unroll
      for (int i = 0; i < kLoads; ++i) {
        v[i] = make_uint4(0, 0, 0, 0);
        if (idx[i] >= 0) v[i] = reinterpret_cast<const uint4*>(Ku + (size_t)idx[i] * kD)[tid & 15];
      }
#pragma unroll
      for (int i = 0; i < kLoads; ++i) {
        const int sr = s0 + ((tid + 256 * i) >> 4);
        *reinterpret_cast<uint4*>(stage + sr * kPitch + (tid & 15) * 16) = v[i];
        float ss = sumsq_bf16x8(v[i]);
#pragma unroll
        for (int o = 8; o > 0; o >>= 1) ss += __shfl_xor(ss, o, 64);
        if ((tid & 15) == 0) seed_inv[sr] = ss > 0.f ? 1.0f / sqrtf(ss) : 0.f;
      }
    }
  };

  fetch_donors(0);
  const bool one_block = M <= kSeedBlock;
  if (one_block) {
    stage_seeds(0);
    __syncthreads();
  }
  for (int t = 0; t < n_tiles; ++t) {
    bf16x8 bres[2][8];
    int drow[2];
    float dinv[2];
#pragma unroll
    for (int ct = 0; ct < 2; ++ct) {
      drow[ct] = first + t * kDonorTile + wv * 64 + ct * 32 + c32;
      const bool ok = drow[ct] < hi;
      float ss = 0.f;
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        uint4 v = ok ? draw[ct][ks] : make_uint4(0, 0, 0, 0);
        ss += sumsq_bf16x8(v);
        bres[ct][ks] = *reinterpret_cast<bf16x8*>(&v);
      }
      ss += __shfl_xor(ss, 32, 64);
      dinv[ct] = ss > 0.f ? 1.0f / sqrtf(ss) : 0.f;
    }
    if (t + 1 < n_tiles) fetch_donors(t + 1);  // in flight while this tile is contracted

    float best[2] = {kNegInf, kNegInf};
    int best_ord[2] = {-1, -1};
    for (int sb = 0; sb < M; sb += kSeedBlock) {
      if (!one_block) {
        __syncthreads();  // previous block fully consumed
        stage_seeds(sb);
        __syncthreads();
      }
      const int m_blk = min(kSeedBlock, M - sb);
      for (int s0 = 0; s0 < m_blk; s0 += 32) {
        bf16x8 a[8];
        const unsigned char* ap = stage + (s0 + c32) * kPitch + h * 16;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) a[ks] = *reinterpret_cast<const bf16x8*>(ap + ks * 32);
#pragma unroll
        for (int ct = 0; ct < 2; ++ct) {
          f32x16 acc = {0};
#pragma unroll
          for (int ks = 0; ks < 8; ++ks)
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ks], bres[ct][ks], acc, 0, 0, 0);
#pragma unroll
          for (int r = 0; r < 16; ++r) {  // ascending seed ordinal within the lane
            const int sr = s0 + (r >> 2) * 8 + h * 4 + (r & 3);
            const float sim = (acc[r] * seed_inv[sr]) * dinv[ct];
            if (sr < m_blk && sim > best[ct]) {
              best[ct] = sim;
              best_ord[ct] = sb + sr;
            }
          }
        }
      }
    }
#pragma unroll
    for (int ct = 0; ct < 2; ++ct) {
      const float ob = __shfl_xor(best[ct], 32, 64);
      const int oo = __shfl_xor(best_ord[ct], 32, 64);
      if (oo >= 0 && (best_ord[ct] < 0 || better(ob, oo, best[ct], best_ord[ct]))) {
        best[ct] = ob;
        best_ord[ct] = oo;
      }
      if (h == 0 && drow[ct] < hi) {
        const bool donor = ro[drow[ct]] == CASK_ROLE_DONOR;
        assign_ord[row0 + drow[ct]] = (donor && best_ord[ct] >= 0 && best[ct] >= kp.tau) ? best_ord[ct] : -1;
      }
    }
  }
}

// ------------------------------------------------------------------ similarity, plain path

template <typename T, int D>
__global__ __launch_bounds__(256) void similarity_fma_kernel(
    KParams kp, int n_units, int tiles_per_unit, const int64_t* __restrict__ row_off,
    const int32_t* __restrict__ prefix_len, const T* __restrict__ K,
    const uint8_t* __restrict__ role, const int32_t* __restrict__ seed_rows,
    const int32_t* __restrict__ n_seeds, int32_t* __restrict__ assign_ord) {
  constexpr int SEEDS = 32;
  __shared__ float sk[SEEDS][D + 1];
  __shared__ float sinv[SEEDS];
  const int bid = blockIdx.x;
  const int u = bid / tiles_per_unit, tile = bid % tiles_per_unit;
  if (u >= n_units) return;
  const int64_t row0 = row_off[u];
  const int N = (int)(row_off[u + 1] - row0);
  const int P = prefix_len[u];
  const UnitPlan pl = make_plan(kp, P, N);
  const int hi = N - pl.r_eff;
  const int base = P + tile * 256;
  if (base >= hi) return;
  const int M = n_seeds[u];
  const int tid = threadIdx.x;
  const int i = base + tid;
  const bool ok = i < hi;
  const T* Ku = K + (size_t)row0 * D;
  const int32_t* srow = seed_rows + (size_t)u * kp.B;
  float k[D];
  float ss = 0.f;
#pragma unroll
  for (int c = 0; c < D; ++c) {
    k[c] = Elem<T>::load(Ku + (size_t)(ok ? i : P) * D + c);
    ss = __builtin_fmaf(k[c], k[c], ss);
  }
  const float dinv = ss > 0.f ? 1.0f / sqrtf(ss) : 0.f;
  float best = kNegInf;
  int best_ord = -1;
  for (int s0 = 0; s0 < M; s0 += SEEDS) {
    __syncthreads();
    for (int q = tid; q < SEEDS * D; q += 256) {
      const int sr = q / D, c = q % D;
      sk[sr][c] = (s0 + sr < M) ? Elem<T>::load(Ku + (size_t)srow[s0 + sr] * D + c) : 0.f;
    }
    __syncthreads();
    if (tid < SEEDS) {
      float t = 0.f;
      for (int c = 0; c < D; ++c) t = __builtin_fmaf(sk[tid][c], sk[tid][c], t);
      sinv[tid] = t > 0.f ? 1.0f / sqrtf(t) : 0.f;
    }
    __syncthreads();
    const int lim = min(SEEDS, M - s0);
    for (int sr = 0; sr < lim; ++sr) {
      float dot = 0.f;
#pragma unroll
      for (int c = 0; c < D; ++c) dot = __builtin_fmaf(k[c], sk[sr][c], dot);
      const float sim = (dot * sinv[sr]) * dinv;
      if (sim > best) {
        best = sim;
        best_ord = s0 + sr;
      }
    }
  }
  if (ok) {
    const bool donor = role[row0 + i] == CASK_ROLE_DONOR;
    assign_ord[row0 + i] = (donor && best_ord >= 0 && best >= kp.tau) ? best_ord : -1;
  }
}

// ------------------------------------------------------------------ gather merged donors

constexpr int kGatherThreads = 1024;
constexpr int kGatherPer = 16;  // 64-row groups per wave and chunk

// assign_mode: 0 none, 1 output slot (whole event), 2 unit-local source row (consolidate API)
__global__ __launch_bounds__(kGatherThreads) void gather_merged_kernel(
    KParams kp, const int64_t* __restrict__ row_off, const int32_t* __restrict__ prefix_len,
    const uint8_t* __restrict__ role, const int32_t* __restrict__ assign_ord,
    const int32_t* __restrict__ slot_of, const int32_t* __restrict__ seed_rows,
    int32_t* __restrict__ merged_row, int32_t* __restrict__ merged_ord,
    int32_t* __restrict__ n_merged, int32_t* __restrict__ assign_out, int assign_mode,
    int32_t* __restrict__ status) {
  __shared__ int wsum[kGatherThreads / 64];
  const int u = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int64_t row0 = row_off[u];
  const int N = (int)(row_off[u + 1] - row0);
  const int P = prefix_len[u];
  const UnitPlan pl = make_plan(kp, P, N);
  const int hi = N - pl.r_eff;
  const int32_t* srow = seed_rows + (size_t)u * kp.B;
  // rows outside the donor range: kept rows map to themselves, the rest is dropped
  if (assign_mode != 0) {
    for (int i = tid; i < N; i += kGatherThreads) {
      if (i >= P && i < hi) continue;
      const int r = role[row0 + i];
      const bool kept = r == CASK_ROLE_PREFIX_KEEP || r == CASK_ROLE_RECENT || r == CASK_ROLE_CORE ||
                        r == CASK_ROLE_SEED;
      assign_out[row0 + i] = !kept ? -1 : (assign_mode == 1 ? slot_of[row0 + i] : i);
    }
  }
  // A wave owns kGatherPer * 64 consecutive rows, touched 64 consecutive rows at a time
  // (coalesced); positions inside the wave come from ballots with a running carry, and one
  // exchange of the wave totals per chunk orders the waves.
  const unsigned long long below = (1ull << lane) - 1ull;
  int count = 0;
  for (int cb = P; cb < hi; cb += kGatherThreads * kGatherPer) {
    const int i0 = cb + wv * (64 * kGatherPer) + lane;
    int r[kGatherPer], ord[kGatherPer], pos[kGatherPer];
#pragma unroll
    for (int e = 0; e < kGatherPer; ++e) {
      const bool in = i0 + e * 64 < hi;
      r[e] = in ? (int)role[row0 + i0 + e * 64] : (int)CASK_ROLE_PREFIX_DROP;
      ord[e] = in ? assign_ord[row0 + i0 + e * 64] : -1;
    }
    int run = 0;
#pragma unroll
    for (int e = 0; e < kGatherPer; ++e) {
      if (r[e] != CASK_ROLE_DONOR) ord[e] = -1;
      const unsigned long long b = __ballot(ord[e] >= 0);
      pos[e] = run + __popcll(b & below);
      run += __popcll(b);
    }
    if (lane == 0) wsum[wv] = run;
    __syncthreads();
    int before = 0, tot = 0;
    for (int w = 0; w < kGatherThreads / 64; ++w) {
      const int x = wsum[w];
      if (w < wv) before += x;
      tot += x;
    }
    __syncthreads();
#pragma unroll
    for (int e = 0; e < kGatherPer; ++e) {
      const int i = i0 + e * 64;
      if (i < hi) {
        if (ord[e] >= 0) {
          const int at = count + before + pos[e];
          merged_row[row0 + at] = i;
          merged_ord[row0 + at] = ord[e];
        }
        if (assign_mode != 0) {
          int v;
          if (r[e] == CASK_ROLE_DONOR) {
            v = ord[e] < 0 ? -1 : (assign_mode == 1 ? slot_of[row0 + srow[ord[e]]] : srow[ord[e]]);
          } else {
            const bool kept = r[e] == CASK_ROLE_CORE || r[e] == CASK_ROLE_SEED;
            v = !kept ? -1 : (assign_mode == 1 ? slot_of[row0 + i] : i);
          }
          assign_out[row0 + i] = v;
        }
      }
    }
    count += tot;
  }
  if (tid == 0) {
    if (n_merged) n_merged[u] = count;
    if (status && count == 0 && !(pl.status & (CASK_ST_IDENTITY | CASK_ST_PREFIX_BUDGET_EXHAUSTED)))
      status[u] = pl.status | CASK_ST_MERGE_INACTIVE;
  }
}

// ------------------------------------------------------------------ emit (copy + fold)

// Sixteen lanes per output row (D / 16 elements each), so a wave moves four rows per load
// instruction; it owns 16 consecutive slots of one unit and puts the loads of four rows of K
// and V in flight before it touches any of them.  A seed slot then folds its donors: the
// group walks the unit's merged list (ascending rows) and accumulates the matching ones in
// fp32 in that order.
template <typename T, int D>
__global__ __launch_bounds__(256) void emit_kernel(
    KParams kp, int n_units, const int64_t* __restrict__ row_off, const T* __restrict__ K,
    const T* __restrict__ V, const float* __restrict__ scores, const int32_t* __restrict__ out_src,
    const int32_t* __restrict__ out_len, const int32_t* __restrict__ ord_of_slot,
    const int32_t* __restrict__ merged_row, const int32_t* __restrict__ merged_ord,
    const int32_t* __restrict__ n_merged, T* __restrict__ K_out, T* __restrict__ V_out,
    float* __restrict__ out_mass) {
  constexpr int EPL = D / 16;                    // elements per lane
  constexpr int WORDS = EPL * sizeof(T) / 4;     // 32-bit words per lane
  constexpr int kSlotsPerWave = 16;
  struct alignas(WORDS * 4 > 16 ? 16 : WORDS * 4) Raw { uint32_t w[WORDS]; };
  const int lane = threadIdx.x & 63, grp = lane >> 4, gl = lane & 15;
  const long long wave = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
  const int B = kp.B;
  const int waves_per_unit = (B + kSlotsPerWave - 1) / kSlotsPerWave;
  const int u = (int)(wave / waves_per_unit);
  const int t_base = (int)(wave % waves_per_unit) * kSlotsPerWave;
  if (u >= n_units) return;
  const int len = out_len[u];
  if (t_base >= len) return;
  const int64_t row0 = row_off[u];
  const int nm = n_merged[u];
  const int32_t* mr = merged_row + row0;
  const int32_t* mo = merged_ord + row0;

  int slot[4], src[4], ord[4];
  float a0[4];
  Raw kraw[4], vraw[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    slot[j] = t_base + j * 4 + grp;
    const bool ok = slot[j] < len;
    src[j] = ok ? out_src[(size_t)u * B + slot[j]] : -1;
    ord[j] = ok ? ord_of_slot[(size_t)u * B + slot[j]] : -1;
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    if (src[j] >= 0) {
      kraw[j] = *reinterpret_cast<const Raw*>(K + (size_t)(row0 + src[j]) * D + gl * EPL);
      vraw[j] = *reinterpret_cast<const Raw*>(V + (size_t)(row0 + src[j]) * D + gl * EPL);
      a0[j] = scores[row0 + src[j]];
    } else {
      a0[j] = 0.f;
    }
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    int members = 1;
    float mass = a0[j];
    float ka[EPL], va[EPL], ku[EPL], vu[EPL];  // weighted and unweighted sums
    const T* kself = reinterpret_cast<const T*>(&kraw[j]);
    const T* vself = reinterpret_cast<const T*>(&vraw[j]);
    if (nm > 0 && __any(ord[j] >= 0)) {
      for (int b0 = 0; b0 < nm; b0 += 16) {
        const int idx = b0 + gl;
        const int my_ord = idx < nm ? mo[idx] : -1;
        const int my_row = idx < nm ? mr[idx] : 0;
        const unsigned long long bal = __ballot(ord[j] >= 0 && my_ord == ord[j]);
        unsigned hit = (unsigned)(bal >> (grp * 16)) & 0xFFFFu;
        while (__any(hit != 0u)) {  // every group steps through its own matches, together
          const bool have = hit != 0u;
          const int l = have ? __ffs((int)hit) - 1 : 0;
          hit &= hit - 1u;
          const int drow = __shfl(my_row, grp * 16 + l, 64);
          if (have) {
            if (members == 1) {
#pragma unroll
              for (int e = 0; e < EPL; ++e) {
                const float kf = Elem<T>::load(kself + e), vf = Elem<T>::load(vself + e);
                ka[e] = a0[j] * kf; va[e] = a0[j] * vf; ku[e] = kf; vu[e] = vf;
              }
            }
            const float a = scores[row0 + drow];
            const Raw dk = *reinterpret_cast<const Raw*>(K + (size_t)(row0 + drow) * D + gl * EPL);
            const Raw dv = *reinterpret_cast<const Raw*>(V + (size_t)(row0 + drow) * D + gl * EPL);
            const T* dkp = reinterpret_cast<const T*>(&dk);
            const T* dvp = reinterpret_cast<const T*>(&dv);
#pragma unroll
            for (int e = 0; e < EPL; ++e) {
              const float kf = Elem<T>::load(dkp + e), vf = Elem<T>::load(dvp + e);
              ka[e] = __builtin_fmaf(a, kf, ka[e]);
              va[e] = __builtin_fmaf(a, vf, va[e]);
              ku[e] += kf;
              vu[e] += vf;
            }
            mass += a;
            ++members;
          }
        }
      }
    }
    if (src[j] < 0) continue;
    T* ko = K_out + ((size_t)u * B + slot[j]) * D + gl * EPL;
    T* vo = V_out + ((size_t)u * B + slot[j]) * D + gl * EPL;
    if (members == 1) {
      *reinterpret_cast<Raw*>(ko) = kraw[j];
      *reinterpret_cast<Raw*>(vo) = vraw[j];
    } else {
      const bool uniform = mass == 0.f;
      const float denom = uniform ? (float)members : mass;
      Raw ok_, ov_;
      T* okp = reinterpret_cast<T*>(&ok_);
      T* ovp = reinterpret_cast<T*>(&ov_);
#pragma unroll
      for (int e = 0; e < EPL; ++e) {
        Elem<T>::store(okp + e, (uniform ? ku[e] : ka[e]) / denom);
        Elem<T>::store(ovp + e, (uniform ? vu[e] : va[e]) / denom);
      }
      *reinterpret_cast<Raw*>(ko) = ok_;
      *reinterpret_cast<Raw*>(vo) = ov_;
    }
    if (out_mass && gl == 0) out_mass[(size_t)u * B + slot[j]] = mass;
  }
}

template <typename T, int D>
hipError_t launch_emit_t(const KParams& kp, const Batch& b, const float* scores,
                         const int32_t* out_src, const int32_t* out_len,
                         const int32_t* ord_of_slot, const int32_t* merged_row,
                         const int32_t* merged_ord, const int32_t* n_merged, void* K_out,
                         void* V_out, float* out_mass, hipStream_t st) {
  const long long waves = (long long)b.n_units * ((kp.B + 15) / 16);
  const long long blocks = (waves + 3) / 4;
  if (blocks == 0) return hipSuccess;
  emit_kernel<T, D><<<dim3((unsigned)blocks), dim3(256), 0, st>>>(
      kp, b.n_units, b.row_off, static_cast<const T*>(b.K), static_cast<const T*>(b.V), scores,
      out_src, out_len, ord_of_slot, merged_row, merged_ord, n_merged, static_cast<T*>(K_out),
      static_cast<T*>(V_out), out_mass);
  return hipGetLastError();
}

template <typename T, int D>
hipError_t launch_similarity_fma(const KParams& kp, const Batch& b, const uint8_t* role,
                                 const int32_t* seed_rows, const int32_t* n_seeds,
                                 int32_t* assign_ord, hipStream_t st) {
  const int tiles = (b.max_decode_len + 255) / 256;
  if (tiles == 0) return hipSuccess;
  similarity_fma_kernel<T, D><<<dim3(b.n_units * tiles), dim3(256), 0, st>>>(
      kp, b.n_units, tiles, b.row_off, b.prefix_len, static_cast<const T*>(b.K), role, seed_rows,
      n_seeds, assign_ord);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_similarity(const KParams& kp, const Batch& b, const uint8_t* role,
                             const int32_t* seed_rows, const int32_t* n_seeds,
                             int32_t* assign_ord, hipStream_t st) {
  if (kp.dtype == CASK_BF16 && kp.d == 128) {
    // a few workgroups per unit, about two per compute unit in all, each walking its share of
    // the unit's donor tiles
    const int tiles = (b.max_decode_len + kDonorTile - 1) / kDonorTile;
    if (tiles == 0) return hipSuccess;
    int chunks = b.n_units > 0 ? 512 / b.n_units : 1;
    if (chunks < 1) chunks = 1;
    if (chunks > tiles) chunks = tiles;
    const int tiles_per_wg = (tiles + chunks - 1) / chunks;
    chunks = (tiles + tiles_per_wg - 1) / tiles_per_wg;
    const int units8 = (b.n_units + 7) / 8 * 8;
    similarity_mfma_kernel<<<dim3(units8 * chunks), dim3(256), 0, st>>>(
        kp, b.n_units, chunks, tiles_per_wg, b.row_off, b.prefix_len,
        static_cast<const uint16_t*>(b.K), role, seed_rows, n_seeds, assign_ord);
    return hipGetLastError();
  }
  if (kp.dtype == CASK_F32)
    return kp.d == 64 ? launch_similarity_fma<float, 64>(kp, b, role, seed_rows, n_seeds, assign_ord, st)
                      : launch_similarity_fma<float, 128>(kp, b, role, seed_rows, n_seeds, assign_ord, st);
  return launch_similarity_fma<uint16_t, 64>(kp, b, role, seed_rows, n_seeds, assign_ord, st);
}

hipError_t launch_gather_merged(const KParams& kp, const Batch& b, const uint8_t* role,
                                const int32_t* assign_ord, const int32_t* slot_of,
                                const int32_t* seed_rows, int32_t* merged_row, int32_t* merged_ord,
                                int32_t* n_merged, int32_t* assign_out, int assign_mode,
                                int32_t* status, hipStream_t st) {
  gather_merged_kernel<<<dim3(b.n_units), dim3(kGatherThreads), 0, st>>>(
      kp, b.row_off, b.prefix_len, role, assign_ord, slot_of, seed_rows, merged_row, merged_ord,
      n_merged, assign_out, assign_mode, status);
  return hipGetLastError();
}

hipError_t launch_emit(const KParams& kp, const Batch& b, const float* scores,
                       const int32_t* out_src, const int32_t* out_len, const int32_t* ord_of_slot,
                       const int32_t* merged_row, const int32_t* merged_ord,
                       const int32_t* n_merged, void* K_out, void* V_out, float* out_mass,
                       hipStream_t st) {
  if (kp.dtype == CASK_F32)
    return kp.d == 64 ? launch_emit_t<float, 64>(kp, b, scores, out_src, out_len, ord_of_slot, merged_row, merged_ord, n_merged, K_out, V_out, out_mass, st)
                      : launch_emit_t<float, 128>(kp, b, scores, out_src, out_len, ord_of_slot, merged_row, merged_ord, n_merged, K_out, V_out, out_mass, st);
  return kp.d == 64 ? launch_emit_t<uint16_t, 64>(kp, b, scores, out_src, out_len, ord_of_slot, merged_row, merged_ord, n_merged, K_out, V_out, out_mass, st)
                    : launch_emit_t<uint16_t, 128>(kp, b, scores, out_src, out_len, ord_of_slot, merged_row, merged_ord, n_merged, K_out, V_out, out_mass, st);
}

}  // namespace cask
