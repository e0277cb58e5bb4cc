// Selective consolidation of the mergeable scratch (Sections 2.1, 2.4, 2.5 of the paper):
//   similarity   every donor against every seed of its unit by key cosine; best seed kept
//                when the cosine reaches tau (bf16 d=128: MFMA contraction seeds x donors^T,
//                each lane owns one donor and scans its seeds in ascending order);
//   gather       ordered list of the donors that merge (ascending row), per unit, then the
//                same list grouped by seed; spare workgroups of the launch copy the kept
//                tokens to the output bit for bit, sixteen lanes per row;
//   emit         a seed with donors becomes the weighted fold m = sum a_i,
//                k~ = sum a_i k_i / m, v~ = sum a_i v_i / m with a_i the token's score,
//                accumulated in fp32 in a fixed order (reruns are bitwise identical).
#include "cask_common.h"
#include <type_traits>

namespace cask {

namespace {

constexpr float kNegInf = -__builtin_inff();

__device__ inline bool better(float sim, int ord, float best, int best_ord) {
  return sim > best || (sim == best && ord < best_ord);
}

// ------------------------------------------------------------------ similarity, MFMA path

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
constexpr int kD = 128;
constexpr int kRowBytes = kD * 2;
constexpr int kGroupPitch = 1024 + 64;  // LDS pitch of a 4-row group (layout: see below)
constexpr int kSeedBlock = 128;         // seeds held in LDS at a time
constexpr int kDonorTile = 128;         // donor rows per tile: 4 waves x 32
constexpr int kPrefetch = 2;            // donor tiles in flight ahead of the one being contracted
constexpr int kMultiTiles = 4;          // tiles per workgroup where a unit's seeds take several blocks
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

__device__ inline float sumsq_bf16x8(const uint4& v) {
  const uint32_t w[4] = {v.x, v.y, v.z, v.w};
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const bf16x2 x = __builtin_bit_cast(bf16x2, w[i]);
    s = __builtin_amdgcn_fdot2_f32_bf16(x, x, s, false);
  }
  return s;
}

// Workgroup = `tiles_per_wg` consecutive donor tiles of one unit; wave w owns rows
// [32 w, 32 w + 32) of every tile.
//
// Memory side: a wave reads its 32 rows with 8 fully coalesced loads (4 whole 256-byte rows
// per instruction: lane l takes 16-byte piece l % 16 of row l / 16), kPrefetch tiles ahead, so
// K streams at memory speed.  The registers then hold rows across lanes, not MFMA operands;
// the wave turns them round through a private LDS region: a 4-row group is kept row by row,
// the 16-byte piece g of row r at slot g ^ r of the row (a 1 KB store per instruction), and lane
// (c32, h) reads back row c32's pieces h, h + 2, ... as the B operand of the eight k-steps; with
// the 1088-byte group pitch both spread any eight consecutive lanes over all banks.  No
// barrier: the region is the wave's own.  The staged seeds use the same layout.
//
// Compute side: the unit's seeds (kSeedBlock at a time, same layout, with inverse norms) are
// the A operand, so a lane owns one donor and sees its seeds in ascending order:
// cos = (dot * |seed|^-1) * |donor|^-1 in fp32, first maximum wins.
// ONE_BLOCK: every unit has at most kSeedBlock seeds, so they are staged once per workgroup and
// the tile loop contains nothing but the donor stream (the host knows the bound).
// RADIUS: a merge radius is set (the epilogue then looks up every seed's cache row).
template <bool ONE_BLOCK, bool RADIUS>
__global__ __launch_bounds__(256, 2) void similarity_mfma_kernel(
    KParams kp, int n_units, int chunks_per_unit, int tiles_per_wg,
    const int64_t* __restrict__ row_off, const int32_t* __restrict__ prefix_len,
    const uint16_t* __restrict__ K, const uint8_t* __restrict__ role,
    const int32_t* __restrict__ seed_rows, const int32_t* __restrict__ n_seeds,
    int32_t* __restrict__ assign_ord) {
  __shared__ __attribute__((aligned(16))) unsigned char seeds[(kSeedBlock / 4) * kGroupPitch];
  __shared__ __attribute__((aligned(16))) unsigned char turn[4][8 * kGroupPitch];
  __shared__ __attribute__((aligned(16))) float seed_inv[kSeedBlock];
  __shared__ __attribute__((aligned(16))) int seed_pos[kSeedBlock];  // cache row of each staged seed
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
  const int tid = threadIdx.x, lane = tid & 63;
  if (M == 0) {  // no seed to fold into: nothing to read
    const int end = min(hi, first + n_tiles * kDonorTile);
    for (int i = first + tid; i < end; i += 256) assign_ord[row0 + i] = -1;
    return;
  }
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: feeds scalar load offsets
  const int c32 = lane & 31, h = lane >> 5;
  const uint16_t* Ku = K + (size_t)row0 * kD;
  const uint8_t* ro = role + row0;
  const int32_t* srow = seed_rows + (size_t)u * kp.B;
  // rows past this workgroup's share of the donor range read as zero through the descriptor's
  // bounds check, without touching memory
  const int last = min(hi, first + n_tiles * kDonorTile);
  const __amdgpu_buffer_rsrc_t krsrc =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(Ku), 0, last * kRowBytes, 0x00020000);

  // ---- donor stream: the wave's 32 rows of tile t, 4 rows per load
  // (the role of the lane's donor row rides along, so that nothing at the end of a tile has
  // to wait on memory behind the loads already issued for the tiles after it)
  uint4 dreg[kPrefetch][8];
  int rreg[kPrefetch];
  auto fetch_donors = [&](int t, uint4 (&d)[8], int& rl) {
    // Always issued, also for tiles past the end (their rows read as zero and are never
    // stored): with an unconditional load count the waits for a tile can leave the loads of
    // the tiles after it in flight.
    const int r0 = first + t * kDonorTile + wv * 32;
    rl = (int)ro[min(r0 + c32, N - 1)];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(
          krsrc, lane * 16, (int)((unsigned)(r0 + 4 * j) * (unsigned)kRowBytes), 2);  // nt: a stream read once
      d[j] = make_uint4(v[0], v[1], v[2], v[3]);
    }
  };
  // ---- seeds [sb, sb + kSeedBlock) -> LDS (16 threads per row, 16 rows per pass) + inverse norms
  auto stage_seeds = [&](int sb) {
    for (int s0 = 0; s0 < kSeedBlock && sb + s0 < M; s0 += 64) {
      int idx[4];
      uint4 v[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int ord = sb + s0 + i * 16 + (tid >> 4);
        idx[i] = ord < M ? srow[ord] : -1;
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        v[i] = make_uint4(0, 0, 0, 0);
        if (idx[i] >= 0) v[i] = reinterpret_cast<const uint4*>(Ku + (size_t)idx[i] * kD)[tid & 15];
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int sr = s0 + i * 16 + (tid >> 4);
        // (row by row with piece g of row r at slot g ^ r, like the waves' turning regions)
        *reinterpret_cast<uint4*>(seeds + (sr >> 2) * kGroupPitch + (sr & 3) * 256 + (((tid & 15) ^ (sr & 3)) * 16)) = v[i];
        float ss = sumsq_bf16x8(v[i]);
#pragma unroll
        for (int o = 8; o > 0; o >>= 1) ss += __shfl_xor(ss, o, 64);
        if ((tid & 15) == 0) {
          seed_inv[sr] = ss > 0.f ? 1.0f / sqrtf(ss) : 0.f;
          seed_pos[sr] = idx[i];
        }
      }
    }
  };
  // merge radius (0 = none): seeds further than this many cache rows from the donor are skipped
  const int radius = kp.radius > 0 ? kp.radius : 0x7fffffff;

  unsigned char* my_turn = turn[wv];
  // The wave's turning region holds a 4-row group row by row, the 16-byte piece g of row r at
  // slot g ^ r of the row: the store of a load's 64 pieces (lane = row l / 16, piece l % 16) and
  // the operand reads (lane = row c32, pieces h, h + 2, ...) then both spread any eight
  // consecutive lanes over all banks.  (Piece-major -- piece g of row r at g * 64 + r * 16 -- the
  // stores ran four lanes to a bank: 44 % of the kernel's LDS cycles were bank conflicts.)
  const int turn_st = (lane >> 4) * 256 + (((lane & 15) ^ (lane >> 4)) * 16);
  const int turn_row = (c32 >> 2) * kGroupPitch + (c32 & 3) * 256;
  const int turn_ld0 = turn_row + ((h ^ (c32 & 3)) * 16);        // k-steps 0, 2, ...: piece 2 ks + h
  const int turn_ld1 = turn_row + (((2 + h) ^ (c32 & 3)) * 16);  // k-steps 1, 3, ...

  // registers -> private LDS region -> B operand of this lane's donor; refills the registers
  // with tile t + kPrefetch; returns the donor's inverse norm
  auto turn_donors = [&](int t, uint4 (&d)[8], int& rl, bf16x8 (&bres)[8]) -> float {
#pragma unroll
    for (int j = 0; j < 8; ++j)
      *reinterpret_cast<uint4*>(my_turn + j * kGroupPitch + turn_st) = d[j];
    fetch_donors(t + kPrefetch, d, rl);  // refill the registers just freed
    float ss = 0.f;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      const uint4 v = *reinterpret_cast<const uint4*>(my_turn + ((ks & 1) ? turn_ld1 : turn_ld0) + (ks >> 1) * 64);
      ss += sumsq_bf16x8(v);
      bres[ks] = __builtin_bit_cast(bf16x8, v);
    }
    ss += __shfl_xor(ss, 32, 64);
    return ss > 0.f ? 1.0f / sqrtf(ss) : 0.f;
  };
  // The lane's donor against the staged seeds [sb, sb + m_blk), ascending ordinal: first maximum
  // wins.  `best` is the cosine without the donor's own inverse norm: a positive factor common
  // to all of a donor's seeds, applied once when the winner is settled.
  auto against_block = [&](int sb, int m_blk, const bf16x8 (&bres)[8], int drow, float& best, int& best_ord) {
    for (int s0 = 0; s0 < m_blk; s0 += 32) {
      bf16x8 a[8];
      const unsigned char* ap = seeds + (s0 >> 2) * kGroupPitch;
#pragma unroll
      for (int ks = 0; ks < 8; ++ks)
        a[ks] = *reinterpret_cast<const bf16x8*>(ap + ((ks & 1) ? turn_ld1 : turn_ld0) + (ks >> 1) * 64);
      f32x16 acc = {0};
#pragma unroll
      for (int ks = 0; ks < 8; ++ks)
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ks], bres[ks], acc, 0, 0, 0);
      auto pick = [&](auto whole_tag) {  // whole: all 32 seeds of this step exist
        constexpr bool kWhole = decltype(whole_tag)::value;
#pragma unroll
        for (int g = 0; g < 4; ++g) {  // ascending seed ordinal within the lane
          const float4 si = *reinterpret_cast<const float4*>(&seed_inv[s0 + g * 8 + h * 4]);
          const float sv[4] = {si.x, si.y, si.z, si.w};
          int pv[4] = {0, 0, 0, 0};
          if (RADIUS) {
            const int4 sp = *reinterpret_cast<const int4*>(&seed_pos[s0 + g * 8 + h * 4]);
            pv[0] = sp.x, pv[1] = sp.y, pv[2] = sp.z, pv[3] = sp.w;
          }
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int sr = s0 + g * 8 + h * 4 + q;
            const float sim = acc[g * 4 + q] * sv[q];
            bool near = true;
            if (RADIUS) near = (pv[q] > drow ? pv[q] - drow : drow - pv[q]) <= radius;
            if ((kWhole || sr < m_blk) && near && sim > best) {
              best = sim;
              best_ord = sb + sr;
            }
          }
        }
      };
      if (s0 + 32 <= m_blk) pick(std::true_type{});
      else pick(std::false_type{});
    }
  };
  // the two half-waves hold the even and the odd groups of four seeds: lowest ordinal wins a tie
  auto settle = [&](float best, int best_ord, float dinv, bool donor, int drow) {
    const float ob = __shfl_xor(best, 32, 64);
    const int oo = __shfl_xor(best_ord, 32, 64);
    if (oo >= 0 && (best_ord < 0 || better(ob, oo, best, best_ord))) {
      best = ob;
      best_ord = oo;
    }
    if (h == 0 && drow < last)  // rows past the workgroup's share belong to another one
      assign_ord[row0 + drow] = (donor && best_ord >= 0 && best * dinv >= kp.tau) ? best_ord : -1;
  };

  if constexpr (ONE_BLOCK) {
#pragma unroll
    for (int t = 0; t < kPrefetch; ++t) fetch_donors(t, dreg[t], rreg[t]);
    stage_seeds(0);
    __syncthreads();
    auto tile_body = [&](int t, uint4 (&d)[8], int& rl) {
      const bool donor = rl == CASK_ROLE_DONOR;
      bf16x8 bres[8];
      const float dinv = turn_donors(t, d, rl, bres);
      const int drow = first + t * kDonorTile + wv * 32 + c32;
      float best = kNegInf;
      int best_ord = -1;
      against_block(0, M, bres, drow, best, best_ord);
      settle(best, best_ord, dinv, donor, drow);
    };
    for (int t = 0; t < n_tiles; t += kPrefetch) {
#pragma unroll
      for (int b = 0; b < kPrefetch; ++b) tile_body(t + b, dreg[b], rreg[b]);
    }
  } else {
    // More seeds than LDS holds at a time: a block of seeds is staged once and meets every tile
    // of the workgroup (at most kMultiTiles; the donors stream again per block, from L2) while
    // each tile's best seed so far waits in registers.  Staging per tile instead made a unit
    // with 282 seeds and four tiles a chain of twelve stagings and twenty-four barriers.
    float best[kMultiTiles], dinv[kMultiTiles];
    int best_ord[kMultiTiles];
    bool donor[kMultiTiles];
#pragma unroll
    for (int t = 0; t < kMultiTiles; ++t) {
      best[t] = kNegInf;
      dinv[t] = 0.f;
      best_ord[t] = -1;
      donor[t] = false;
    }
    for (int sb = 0; sb < M; sb += kSeedBlock) {
      if (sb > 0) __syncthreads();  // previous block fully consumed
#pragma unroll
      for (int t = 0; t < kPrefetch; ++t) fetch_donors(t, dreg[t], rreg[t]);
      stage_seeds(sb);
      __syncthreads();
      const int m_blk = min(kSeedBlock, M - sb);
      static_assert(kMultiTiles % kPrefetch == 0, "whole rounds of the register ring");
#pragma unroll
      for (int t = 0; t < kMultiTiles; ++t) {
        if (t < n_tiles) {  // (the same for the whole workgroup)
          donor[t] = rreg[t % kPrefetch] == CASK_ROLE_DONOR;
          bf16x8 bres[8];
          dinv[t] = turn_donors(t, dreg[t % kPrefetch], rreg[t % kPrefetch], bres);
          against_block(sb, m_blk, bres, first + t * kDonorTile + wv * 32 + c32, best[t], best_ord[t]);
        }
      }
    }
#pragma unroll
    for (int t = 0; t < kMultiTiles; ++t)
      if (t < n_tiles) settle(best[t], best_ord[t], dinv[t], donor[t], first + t * kDonorTile + wv * 32 + c32);
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
      const int gap = srow[s0 + sr] > i ? srow[s0 + sr] - i : i - srow[s0 + sr];
      if (kp.radius > 0 && gap > kp.radius) continue;
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

// ------------------------------------------------------------------ similarity, kappa geometry

// Kappa-weighted merge distance (Section 2.5): d(k_i, k_j) = sum over rotary bands f (channels
// f and f + D/2) of w_f times the Euclidean distance inside the band.  A square root per band
// keeps this off the matrix cores: one thread per donor with its key in registers, seeds staged
// in LDS 32 at a time (every lane reads the same seed element: a broadcast), fp32 throughout.
// Nearest seed wins (first minimum in ascending seed order) if its distance is <= theta.
//
// Every term is non-negative and fp32 addition of non-negative terms is monotone, so a partial
// sum is a lower bound of the finished one.  Bands are summed in chunks of eight, heaviest
// chunk (by summed weight) first, and a wave leaves a seed as soon as no lane's partial sum can
// still win (<= theta and < its best so far).  Lanes that finish hold the full sum in the same
// order as without the early exit, so the result does not depend on it.
template <typename T>
__device__ inline void load8(const T* p, float* out);
template <>
__device__ inline void load8<float>(const float* p, float* out) {
  const float4 a = *reinterpret_cast<const float4*>(p);
  const float4 b = *reinterpret_cast<const float4*>(p + 4);
  out[0] = a.x, out[1] = a.y, out[2] = a.z, out[3] = a.w;
  out[4] = b.x, out[5] = b.y, out[6] = b.z, out[7] = b.w;
}
template <>
__device__ inline void load8<uint16_t>(const uint16_t* p, float* out) {
  const uint4 r = *reinterpret_cast<const uint4*>(p);
  const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    out[2 * j] = __uint_as_float(w[j] << 16);
    out[2 * j + 1] = __uint_as_float(w[j] & 0xffff0000u);
  }
}

template <typename T, int D>
__global__ __launch_bounds__(256) void similarity_kappa_kernel(
    KParams kp, int n_units, int tiles_per_unit, const int64_t* __restrict__ row_off,
    const int32_t* __restrict__ prefix_len, const T* __restrict__ K,
    const uint8_t* __restrict__ role, const int32_t* __restrict__ seed_rows,
    const int32_t* __restrict__ n_seeds, int32_t* __restrict__ assign_ord) {
  constexpr int SEEDS = 32;
  constexpr int H = D / 2;
  constexpr int NCH = H / 8;  // chunks of eight bands
  __shared__ __attribute__((aligned(16))) float sk[SEEDS][D];
  __shared__ __attribute__((aligned(16))) float wband[H];
  __shared__ int spos[SEEDS];
  __shared__ uint32_t chunk_order;  // four bits per position: which chunk is summed there
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
  if (tid < H) wband[tid] = kp.band_w[tid];
  __syncthreads();
  if (tid == 0) {
    float cw[NCH];
    for (int c = 0; c < NCH; ++c) {
      cw[c] = 0.f;
      for (int f = 0; f < 8; ++f) cw[c] += wband[c * 8 + f];
    }
    uint32_t packed = 0;
    for (int c = 0; c < NCH; ++c) {  // rank = chunks that come before c
      int r = 0;
      for (int e = 0; e < NCH; ++e) r += (cw[e] > cw[c]) || (cw[e] == cw[c] && e < c);
      packed |= (uint32_t)c << (4 * r);
    }
    chunk_order = packed;
  }
  __syncthreads();
  const uint32_t order = __builtin_amdgcn_readfirstlane(chunk_order);
  const bool donor = ok && role[row0 + i] == CASK_ROLE_DONOR;
  float k[D];
#pragma unroll
  for (int c = 0; c < D; c += 8) load8<T>(Ku + (size_t)(ok ? i : P) * D + c, k + c);
  float best = __builtin_inff();
  int best_ord = -1;
  for (int s0 = 0; s0 < M; s0 += SEEDS) {
    __syncthreads();
    for (int q = tid; q < SEEDS * D / 8; q += 256) {
      const int sr = q / (D / 8), c = (q % (D / 8)) * 8;
      float v[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
      if (s0 + sr < M) load8<T>(Ku + (size_t)srow[s0 + sr] * D + c, v);
#pragma unroll
      for (int e = 0; e < 8; ++e) sk[sr][c + e] = v[e];
    }
    if (tid < SEEDS) spos[tid] = (s0 + tid < M) ? srow[s0 + tid] : 0;
    __syncthreads();
    const int lim = min(SEEDS, M - s0);
    for (int sr = 0; sr < lim; ++sr) {
      const int gap = spos[sr] > i ? spos[sr] - i : i - spos[sr];
      const bool in_reach = donor && (kp.radius <= 0 || gap <= kp.radius);
      if (__builtin_amdgcn_ballot_w64(in_reach) == 0) continue;
      float dist = 0.f;
      bool finished = true;
      for (int ci = 0; ci < NCH; ++ci) {
        const int c = (int)((order >> (4 * ci)) & 15u);
#pragma unroll
        for (int cc = 0; cc < NCH; ++cc) {
          if (c == cc) {
            const float4 a0 = *reinterpret_cast<const float4*>(&sk[sr][cc * 8]);
            const float4 a1 = *reinterpret_cast<const float4*>(&sk[sr][cc * 8 + 4]);
            const float4 b0 = *reinterpret_cast<const float4*>(&sk[sr][H + cc * 8]);
            const float4 b1 = *reinterpret_cast<const float4*>(&sk[sr][H + cc * 8 + 4]);
            const float4 w0 = *reinterpret_cast<const float4*>(&wband[cc * 8]);
            const float4 w1 = *reinterpret_cast<const float4*>(&wband[cc * 8 + 4]);
            const float sa[8] = {a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w};
            const float sb[8] = {b0.x, b0.y, b0.z, b0.w, b1.x, b1.y, b1.z, b1.w};
            const float ww[8] = {w0.x, w0.y, w0.z, w0.w, w1.x, w1.y, w1.z, w1.w};
#pragma unroll
            for (int f = 0; f < 8; ++f) {
              const float a = k[cc * 8 + f] - sa[f];
              const float b = k[H + cc * 8 + f] - sb[f];
              dist = __builtin_fmaf(ww[f], __builtin_amdgcn_sqrtf(__builtin_fmaf(a, a, b * b)), dist);
            }
          }
        }
        const bool alive = in_reach && dist <= kp.theta && dist < best;
        if (ci + 1 < NCH && __builtin_amdgcn_ballot_w64(alive) == 0) {
          finished = false;
          break;
        }
      }
      if (finished && in_reach && dist < best) {
        best = dist;
        best_ord = s0 + sr;
      }
    }
  }
  if (ok) assign_ord[row0 + i] = (donor && best_ord >= 0 && best <= kp.theta) ? best_ord : -1;
}

template <typename T, int D>
hipError_t launch_similarity_kappa(const KParams& kp, const Batch& b, const uint8_t* role,
                                   const int32_t* seed_rows, const int32_t* n_seeds,
                                   int32_t* assign_ord, hipStream_t st) {
  const int tiles = (b.max_decode_len + 255) / 256;
  if (tiles == 0) return hipSuccess;
  similarity_kappa_kernel<T, D><<<dim3(b.n_units * tiles), dim3(256), 0, st>>>(
      kp, b.n_units, tiles, b.row_off, b.prefix_len, static_cast<const T*>(b.K), role, seed_rows,
      n_seeds, assign_ord);
  return hipGetLastError();
}

// ------------------------------------------------------------------ gather merged donors

constexpr int kGatherThreads = 1024;
constexpr int kGatherPer = 16;  // 64-row groups per wave and chunk, at most (the kernel's instances: 4, 8, 16)
constexpr int kSegLds = 8192;   // seed ordinals whose segment cursors fit in LDS at a time
constexpr int kSmallList = 64;  // donor lists up to this length are split by a single wave

// row groups (of four rows) a copy wave handles one after the other; measured: two beat four
// and one (a long prefix-heavy copy, B = 2048: 64 us against 76 and 74)
constexpr int kCopyRounds = 2;

// Copy of the rows an event keeps as they are (Sections 2.1, 2.4: protected tokens and the kept
// part of the scratch stay untouched; only a seed with donors becomes a folded representative).
// A wave owns 8 consecutive output slots of one unit, sixteen lanes a row (a sixteenth of the
// row each); it puts the loads of its rows of K and V in flight before it touches any of them
// and writes every slot, the seeds' too: the fold that follows in the stream overwrites the
// seeds whose group has donors.  The copy needs nothing but the ordered walk's output, so it
// shares a launch with the grouping of the donors, whose workgroups leave most of the chip
// idle.  The row pieces are native vectors: with HIP's vector classes the staging arrays end up
// in scratch memory.
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

template <typename Vec, int PIECES>
__device__ __forceinline__ void copy_kept_rows(const CopyJob& cj, int B,
                                               const int64_t* __restrict__ row_off,
                                               long long wave, int lane) {
  constexpr int kSlotsPerWave = 4 * kCopyRounds;
  constexpr int BPL = (int)sizeof(Vec) * PIECES;  // a lane's share of a row: a sixteenth of it
  const int grp = lane >> 4, gl = lane & 15;
  const int waves_per_unit = (B + kSlotsPerWave - 1) / kSlotsPerWave;
  const int u = (int)(wave / waves_per_unit);
  const int t_base = (int)(wave % waves_per_unit) * kSlotsPerWave;
  if (u >= cj.n_units) return;
  int slot[kCopyRounds], src[kCopyRounds], c0[kCopyRounds];
  float a0[kCopyRounds];
  Vec kraw[kCopyRounds][PIECES], vraw[kCopyRounds][PIECES];
  // the slots' sources are read along with the unit's length, which says how many of them mean
  // anything (every unit owns B slots of the array: one round trip instead of two)
#pragma unroll
  for (int j = 0; j < kCopyRounds; ++j) {
    slot[j] = t_base + j * 4 + grp;
    src[j] = slot[j] < B ? cj.out_src[(size_t)u * B + slot[j]] : -1;
  }
  const int len = cj.out_len[u];
  if (t_base >= len) return;
  const int64_t row0 = row_off[u];
  const size_t pitch = (size_t)16 * BPL;
#pragma unroll
  for (int j = 0; j < kCopyRounds; ++j) {
    if (slot[j] >= len) src[j] = -1;
    // a slot past the unit's length reads the unit's first row and writes nothing
    const int64_t row = row0 + max(src[j], 0);
    const size_t at = (size_t)row * pitch + (size_t)gl * BPL;
#pragma unroll
    for (int q = 0; q < PIECES; ++q) {
      kraw[j][q] = *reinterpret_cast<const Vec*>(cj.K + at + q * sizeof(Vec));
      vraw[j][q] = *reinterpret_cast<const Vec*>(cj.V + at + q * sizeof(Vec));
    }
    a0[j] = cj.scores[row];
    c0[j] = cj.in_count ? cj.in_count[row] : 1;
  }
#pragma unroll
  for (int j = 0; j < kCopyRounds; ++j) {
    if (src[j] < 0) continue;
    const size_t at = ((size_t)u * cj.out_stride + slot[j]) * pitch + (size_t)gl * BPL;
#pragma unroll
    for (int q = 0; q < PIECES; ++q) {
      *reinterpret_cast<Vec*>(cj.K_out + at + q * sizeof(Vec)) = kraw[j][q];
      *reinterpret_cast<Vec*>(cj.V_out + at + q * sizeof(Vec)) = vraw[j][q];
    }
    if (cj.out_mass && gl == 0) cj.out_mass[(size_t)u * B + slot[j]] = a0[j];
    if (cj.out_count && gl == 0) cj.out_count[(size_t)u * B + slot[j]] = c0[j];
  }
}

// Workgroups below `n_gather` group the donors of one unit each; the ones above copy kept rows
// (`cj.K_out` null: there are none).
// assign_mode: 0 none, 1 output slot (whole event), 2 unit-local source row (consolidate API)
template <int PER>
__global__ __launch_bounds__(kGatherThreads) void gather_merged_kernel(
    KParams kp, int n_gather, CopyJob cj,
    const int64_t* __restrict__ row_off, const int32_t* __restrict__ prefix_len,
    const uint8_t* __restrict__ role, const int32_t* __restrict__ assign_ord,
    const int32_t* __restrict__ slot_of, const int32_t* __restrict__ seed_rows,
    int32_t* __restrict__ merged_row, int32_t* __restrict__ merged_ord,
    int32_t* __restrict__ n_merged, int32_t* __restrict__ assign_out, int assign_mode,
    int32_t* __restrict__ status, const int32_t* __restrict__ n_seeds,
    int32_t* __restrict__ seg_row, int32_t* __restrict__ seg_start) {
  __shared__ int wsum[kGatherThreads / 64];
  __shared__ int cursor[kSegLds];
  const int u = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  if (u >= n_gather) {
    const long long wave = (long long)(u - n_gather) * (kGatherThreads / 64) + wv;
    if (cj.lane_bytes == 16) copy_kept_rows<u32x4, 1>(cj, kp.B, row_off, wave, lane);
    else if (cj.lane_bytes == 32) copy_kept_rows<u32x4, 2>(cj, kp.B, row_off, wave, lane);
    else copy_kept_rows<u32x2, 1>(cj, kp.B, row_off, wave, lane);
    return;
  }
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
  // A wave owns PER * 64 consecutive rows of a chunk, touched 64 consecutive rows at a time
  // (coalesced); positions inside the wave come from ballots with a running carry, and one
  // exchange of the wave totals per chunk orders the waves.
  const unsigned long long below = (1ull << lane) - 1ull;
  int count = 0;
  for (int cb = P; cb < hi; cb += kGatherThreads * PER) {
    const int i0 = cb + wv * (64 * PER) + lane;
    int r[PER], ord[PER], pos[PER];
#pragma unroll
    for (int e = 0; e < PER; ++e) {
      const bool in = i0 + e * 64 < hi;
      r[e] = in ? (int)role[row0 + i0 + e * 64] : (int)CASK_ROLE_PREFIX_DROP;
      ord[e] = in ? assign_ord[row0 + i0 + e * 64] : -1;
    }
    int run = 0;
#pragma unroll
    for (int e = 0; e < PER; ++e) {
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
    for (int e = 0; e < PER; ++e) {
      const int i = i0 + e * 64;
      if (i < hi && ord[e] >= 0) {
        const int at = count + before + pos[e];
        merged_row[row0 + at] = i;
        merged_ord[row0 + at] = ord[e];
        if (at < kSmallList) {  // the head of the list also waits in LDS for the short-list split below
          cursor[at] = ord[e];
          cursor[kSmallList + at] = i;
        }
      }
    }
    if (assign_mode != 0) {
      // What a row maps to: a folding donor to its seed, a kept row to itself, anything else to
      // nothing.  The two dependent lookups (seed's row, then its slot) are taken for all of the
      // thread's rows at a time: one after the other, every row would wait for its own round trip.
      int tgt[PER];
#pragma unroll
      for (int e = 0; e < PER; ++e) {
        const int i = i0 + e * 64;
        const bool kept = r[e] == CASK_ROLE_CORE || r[e] == CASK_ROLE_SEED;
        tgt[e] = (i < hi && ord[e] >= 0) ? srow[ord[e]] : ((i < hi && kept) ? i : -1);  // (ord >= 0 only for donors)
      }
      if (assign_mode == 1) {
#pragma unroll
        for (int e = 0; e < PER; ++e) tgt[e] = tgt[e] >= 0 ? slot_of[row0 + tgt[e]] : -1;
      }
#pragma unroll
      for (int e = 0; e < PER; ++e) {
        const int i = i0 + e * 64;
        if (i < hi) assign_out[row0 + i] = tgt[e];
      }
    }
    count += tot;
  }
  if (tid == 0) {
    if (n_merged) n_merged[u] = count;
    if (status && count == 0 && !(pl.status & (CASK_ST_IDENTITY | CASK_ST_PREFIX_BUDGET_EXHAUSTED)))
      status[u] = pl.status | CASK_ST_MERGE_INACTIVE;
  }
  if (seg_row == nullptr || count == 0) return;  // count is the same in every thread

  // Second pass: the same donors grouped by seed ordinal, rows still ascending inside a group
  // (a stable split), so that a seed's fold reads one contiguous segment.
  __syncthreads();  // the list written above is read by other threads below
  const int M = n_seeds[u];
  const int32_t* mrow = merged_row + row0;
  const int32_t* mord = merged_ord + row0;
  int32_t* sstart = seg_start + (size_t)u * (kp.B + 1);
  if (count <= kSmallList) {
    // A list of at most 64 donors (the usual case: few donors reach the threshold) is split by
    // one wave from its copy in LDS: an entry's place is the number of entries with a smaller
    // ordinal plus the earlier ones with the same ordinal; a segment starts at the number of
    // entries with a smaller ordinal.
    if (wv == 0) {
      const int o_l = lane < count ? cursor[lane] : 0x7fffffff;
      const int r_l = cursor[kSmallList + lane];
      int place = 0;
      for (int j = 0; j < count; ++j) {
        const int oj = __shfl(o_l, j, 64);
        place += (oj < o_l || (oj == o_l && j < lane)) ? 1 : 0;
      }
      if (lane < count) seg_row[row0 + place] = r_l;
    }
    for (int q = tid; q <= M; q += kGatherThreads) {
      int smaller = 0;
      for (int j = 0; j < count; ++j) smaller += cursor[j] < q ? 1 : 0;
      sstart[q] = smaller;
    }
    return;
  }
  // Longer lists: every wave owns a contiguous run of the list.  Per range of kWaveOrds
  // ordinals: a histogram per wave in LDS, from which every (wave, ordinal) pair gets the place
  // of its first entry (the segment's start plus what the earlier waves hold of that ordinal).
  // Then a wave walks its run 64 entries at a time: an entry's place is its pair's cursor plus
  // the number of earlier lanes with the same ordinal (the lanes that agree in every bit of the
  // ordinal: one ballot per bit), so rows stay ascending inside a segment and no two waves
  // touch the same cursor.
  constexpr int NWV = kGatherThreads / 64;
  constexpr int kWaveOrds = kSegLds / NWV;  // ordinals per range: a cursor per wave and ordinal
  static_assert(kWaveOrds <= kGatherThreads, "a thread per ordinal of a range");
  const int run = (count + NWV * 64 - 1) / (NWV * 64) * 64;
  const int c0 = min(count, wv * run), c1 = min(count, c0 + run);
  int* const my_cursor = cursor + wv * kWaveOrds;
  int base = 0;
  for (int o_lo = 0; o_lo < M; o_lo += kWaveOrds) {
    const int range = min(kWaveOrds, M - o_lo);
    int nbits = 1;
    while ((1 << nbits) < range) ++nbits;
    for (int q = tid; q < kSegLds; q += kGatherThreads) cursor[q] = 0;
    __syncthreads();
    for (int idx = c0 + lane; idx < c1; idx += 64) {
      const int o = mord[idx] - o_lo;
      if (o >= 0 && o < range) atomicAdd(&my_cursor[o], 1);
    }
    __syncthreads();
    // thread q: ordinal o_lo + q.  Its entries per wave become the waves' offsets inside the
    // segment; the segment starts come from a scan of the totals.
    int total = 0;
    if (tid < range) {
      for (int w = 0; w < NWV; ++w) {
        const int t = cursor[w * kWaveOrds + tid];
        cursor[w * kWaveOrds + tid] = total;
        total += t;
      }
    }
    int incl = total;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int y = __shfl_up(incl, o, 64);
      if (lane >= o) incl += y;
    }
    if (lane == 63) wsum[wv] = incl;
    __syncthreads();
    int before = 0, tot = 0;
    for (int w = 0; w < NWV; ++w) {
      const int x = wsum[w];
      if (w < wv) before += x;
      tot += x;
    }
    if (tid < range) {
      const int start = base + before + (incl - total);
      sstart[o_lo + tid] = start;
      for (int w = 0; w < NWV; ++w) cursor[w * kWaveOrds + tid] += start;
    }
    base += tot;
    __syncthreads();
    constexpr int kAhead = 4;  // 64-entry steps whose loads are in flight together
    for (int i0 = c0; i0 < c1; i0 += 64 * kAhead) {
      int os[kAhead], rs[kAhead];
#pragma unroll
      for (int e = 0; e < kAhead; ++e) {
        const int idx = min(i0 + e * 64 + lane, c1 - 1);  // clamped: no branch around the loads
        os[e] = mord[idx];
        rs[e] = mrow[idx];
      }
#pragma unroll
      for (int e = 0; e < kAhead; ++e) {
        const int idx = i0 + e * 64 + lane;
        const int o = os[e] - o_lo;
        const bool valid = idx < c1 && o >= 0 && o < range;
        unsigned long long same = __ballot(valid);
        for (int bit = 0; bit < nbits; ++bit) {
          const bool one = ((o >> bit) & 1) != 0;
          const unsigned long long ones = __ballot(valid && one);
          same &= one ? ones : ~ones;
        }
        if (valid) {  // `same`: the valid lanes with this lane's ordinal
          const int rank = __popcll(same & below);
          const int cur = my_cursor[o];
          seg_row[row0 + cur + rank] = rs[e];
          if (rank == __popcll(same) - 1) my_cursor[o] = cur + rank + 1;  // (after every lane's read)
        }
      }
    }
    __syncthreads();  // the cursors are cleared for the next range
  }
  if (tid == 0) sstart[M] = count;
}

// ------------------------------------------------------------------ emit (fold)

// Sixteen lanes hold one row (D / 16 elements each).  A seed with up to kWaveFoldMax donors is
// folded by one wave: its four 16-lane groups take the seed's donors (one contiguous segment of
// the grouped donor list, ascending rows) round-robin, four donors' loads in flight per group,
// accumulate in fp32 in ascending order, and the four partial sums are added in a fixed tree.
// A longer group is folded by the four waves of a workgroup together (sixteen groups, the
// waves' sums added in a fixed tree through LDS).  Either way the result depends on the group
// alone, not on timing.  Runs after the launch that copied every kept row, the seeds' own rows
// included, and overwrites the slots of the seeds that have donors.
constexpr int kWaveFoldMax = 64;  // donors of one seed that a single wave folds (four rounds of its four groups)

template <typename T, int D>
__global__ __launch_bounds__(256) void emit_kernel(
    KParams kp, int n_units, int fold_per_unit,
    const int64_t* __restrict__ row_off, const T* __restrict__ K, const T* __restrict__ V,
    const float* __restrict__ scores, const int32_t* __restrict__ seed_rows,
    const int32_t* __restrict__ n_seeds, const int32_t* __restrict__ slot_of,
    const int32_t* __restrict__ seg_row, const int32_t* __restrict__ seg_start,
    const int32_t* __restrict__ n_merged, T* __restrict__ K_out, T* __restrict__ V_out,
    float* __restrict__ out_mass, const int32_t* __restrict__ in_count,
    int32_t* __restrict__ out_count, int out_stride) {
  constexpr int EPL = D / 16;                    // elements per lane
  constexpr int WORDS = EPL * sizeof(T) / 4;     // 32-bit words per lane
  struct alignas(WORDS * 4 > 16 ? 16 : WORDS * 4) Raw { uint32_t w[WORDS]; };
  __shared__ int long_item[256][4];              // (unit, ordinal, segment bounds) of the long groups of a round
  __shared__ int n_long;
  __shared__ float part[4][4 * EPL][16];         // the waves' sums of a group folded by all four
  __shared__ float part_mass[4];
  __shared__ int part_count[4];
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6, grp = lane >> 4, gl = lane & 15;
  const int B = kp.B;

  // Folds the donors [s0, s1) of one seed.  `ng` 16-lane groups share them round-robin and this
  // one is number `g`; with `all_waves` the groups are the workgroup's sixteen and the waves'
  // sums are added through LDS as (w0 + w1) + (w2 + w3), else they are the wave's four.
  auto fold_group = [&](int u, int ord, int s0, int s1, int g, auto ng_c, auto all_c) {
    constexpr int ng = decltype(ng_c)::value;
    constexpr bool all_waves = decltype(all_c)::value;
    const int64_t row0 = row_off[u];
    const int32_t* seg = seg_row + row0;
    const int srow = seed_rows[(size_t)u * B + ord];
    const int slot = slot_of[row0 + srow];
    float ka[EPL], va[EPL], ku[EPL], vu[EPL];  // score-weighted and count-weighted sums
    float mass = 0.f;
    int count = 0;
#pragma unroll
    for (int e = 0; e < EPL; ++e) ka[e] = va[e] = ku[e] = vu[e] = 0.f;
    if (g == 0) {  // the seed's own row opens the first group's sum
      const float a = scores[row0 + srow];
      const int c = in_count ? in_count[row0 + srow] : 1;
      const Raw sk = *reinterpret_cast<const Raw*>(K + (size_t)(row0 + srow) * D + gl * EPL);
      const Raw sv = *reinterpret_cast<const Raw*>(V + (size_t)(row0 + srow) * D + gl * EPL);
      const T* skp = reinterpret_cast<const T*>(&sk);
      const T* svp = reinterpret_cast<const T*>(&sv);
#pragma unroll
      for (int e = 0; e < EPL; ++e) {
        const float kf = Elem<T>::load(skp + e), vf = Elem<T>::load(svp + e);
        ka[e] = a * kf; va[e] = a * vf; ku[e] = (float)c * kf; vu[e] = (float)c * vf;
      }
      mass = a;
      count = c;
    }
    for (int idx = s0 + g; idx < s1; idx += 4 * ng) {
      int drow[4], dc[4];
      float a[4];
      Raw dk[4], dv[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) drow[q] = seg[min(idx + ng * q, s1 - 1)];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        a[q] = scores[row0 + drow[q]];
        dc[q] = in_count ? in_count[row0 + drow[q]] : 1;
        dk[q] = *reinterpret_cast<const Raw*>(K + (size_t)(row0 + drow[q]) * D + gl * EPL);
        dv[q] = *reinterpret_cast<const Raw*>(V + (size_t)(row0 + drow[q]) * D + gl * EPL);
      }
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        if (idx + ng * q < s1) {
          const float dcf = (float)dc[q];
          const T* dkp = reinterpret_cast<const T*>(&dk[q]);
          const T* dvp = reinterpret_cast<const T*>(&dv[q]);
#pragma unroll
          for (int e = 0; e < EPL; ++e) {
            const float kf = Elem<T>::load(dkp + e), vf = Elem<T>::load(dvp + e);
            ka[e] = __builtin_fmaf(a[q], kf, ka[e]);
            va[e] = __builtin_fmaf(a[q], vf, va[e]);
            ku[e] = __builtin_fmaf(dcf, kf, ku[e]);
            vu[e] = __builtin_fmaf(dcf, vf, vu[e]);
          }
          mass += a[q];
          count += dc[q];
        }
      }
    }
    // (g0 + g1) + (g2 + g3): addition commutes, so every lane ends with the same bits
#pragma unroll
    for (int o = 16; o <= 32; o <<= 1) {
#pragma unroll
      for (int e = 0; e < EPL; ++e) {
        ka[e] += __shfl_xor(ka[e], o, 64);
        va[e] += __shfl_xor(va[e], o, 64);
        ku[e] += __shfl_xor(ku[e], o, 64);
        vu[e] += __shfl_xor(vu[e], o, 64);
      }
      mass += __shfl_xor(mass, o, 64);
      count += __shfl_xor(count, o, 64);
    }
    if constexpr (all_waves) {
      // The waves' sums meet in LDS.  Wave 0 adds them as (w0 + w1) + (w2 + w3), its 16-lane group
      // q taking one of the four sums (score-weighted K, V, count-weighted K, V), and the two
      // groups whose sums the result is made of write it.
      if (grp == 0) {
#pragma unroll
        for (int e = 0; e < EPL; ++e) {
          part[wv][e][gl] = ka[e];
          part[wv][EPL + e][gl] = va[e];
          part[wv][2 * EPL + e][gl] = ku[e];
          part[wv][3 * EPL + e][gl] = vu[e];
        }
        if (gl == 0) {
          part_mass[wv] = mass;
          part_count[wv] = count;
        }
      }
      __syncthreads();
      if (wv == 0) {
        const float m = (part_mass[0] + part_mass[1]) + (part_mass[2] + part_mass[3]);
        const int c = (part_count[0] + part_count[1]) + (part_count[2] + part_count[3]);
        const bool uniform = m == 0.f;  // no score mass: average over the original tokens
        const float denom = uniform ? (float)c : m;
        if ((grp >= 2) == uniform) {
          Raw o_;
          T* op = reinterpret_cast<T*>(&o_);
#pragma unroll
          for (int e = 0; e < EPL; ++e) {
            const int k = grp * EPL + e;
            Elem<T>::store(op + e, ((part[0][k][gl] + part[1][k][gl]) + (part[2][k][gl] + part[3][k][gl])) / denom);
          }
          T* dst = (grp & 1) ? V_out : K_out;
          *reinterpret_cast<Raw*>(dst + ((size_t)u * out_stride + slot) * D + gl * EPL) = o_;
        }
        if (out_mass && lane == 0) out_mass[(size_t)u * B + slot] = m;
        if (out_count && lane == 0) out_count[(size_t)u * B + slot] = c;
      }
      __syncthreads();  // the next group's sums go to the same place
    } else if (grp == 0) {
      const bool uniform = mass == 0.f;  // no score mass: average over the original tokens
      const float denom = uniform ? (float)count : mass;
      Raw ok_, ov_;
      T* okp = reinterpret_cast<T*>(&ok_);
      T* ovp = reinterpret_cast<T*>(&ov_);
#pragma unroll
      for (int e = 0; e < EPL; ++e) {
        Elem<T>::store(okp + e, (uniform ? ku[e] : ka[e]) / denom);
        Elem<T>::store(ovp + e, (uniform ? vu[e] : va[e]) / denom);
      }
      *reinterpret_cast<Raw*>(K_out + ((size_t)u * out_stride + slot) * D + gl * EPL) = ok_;
      *reinterpret_cast<Raw*>(V_out + ((size_t)u * out_stride + slot) * D + gl * EPL) = ov_;
      if (out_mass && gl == 0) out_mass[(size_t)u * B + slot] = mass;
      if (out_count && gl == 0) out_count[(size_t)u * B + slot] = count;
    }
  };

  // Work items are (unit, seed ordinal) pairs; each lane tests one item of a round
  // (neighbouring ordinals go to different waves).  A wave folds its items that have up to
  // kWaveFoldMax donors one after the other; the longer ones are put on a list and folded by
  // the whole workgroup, one after the other: a seed that gathered a thousand donors is
  // otherwise a chain of sixty dependent round trips in one wave while the chip idles.
  const int NW = (int)gridDim.x * 4;
  const int w = (int)blockIdx.x * 4 + wv;
  const long long items = (long long)n_units * fold_per_unit;
  for (long long base = 0; base < items; base += 64LL * NW) {  // (the same trips in every wave)
    if (threadIdx.x == 0) n_long = 0;
    __syncthreads();
    const long long item = base + (long long)lane * NW + w;
    int my_u = 0, my_ord = 0, my_s0 = 0, my_s1 = 0;
    if (item < items) {
      my_u = (int)(item / fold_per_unit);
      my_ord = (int)(item % fold_per_unit);
      // the segment bounds are read along with the counts that say whether they mean anything
      // (the slots exist for every ordinal below B; one round trip instead of two)
      const int s0 = seg_start[(size_t)my_u * (B + 1) + my_ord];
      const int s1 = seg_start[(size_t)my_u * (B + 1) + my_ord + 1];
      if (my_ord < n_seeds[my_u] && n_merged[my_u] > 0) {
        my_s0 = s0;
        my_s1 = s1;
      }
    }
    if (my_s1 - my_s0 > kWaveFoldMax) {
      const int at = atomicAdd(&n_long, 1);  // (the order on the list does not reach the results)
      long_item[at][0] = my_u;
      long_item[at][1] = my_ord;
      long_item[at][2] = my_s0;
      long_item[at][3] = my_s1;
    }
    unsigned long long todo = __ballot(my_s1 > my_s0 && my_s1 - my_s0 <= kWaveFoldMax);
    while (todo != 0ull) {
      const int src_lane = __ffsll((long long)todo) - 1;
      todo &= todo - 1ull;
      fold_group(__shfl(my_u, src_lane, 64), __shfl(my_ord, src_lane, 64), __shfl(my_s0, src_lane, 64),
                 __shfl(my_s1, src_lane, 64), grp, std::integral_constant<int, 4>{}, std::false_type{});
    }
    __syncthreads();
    const int nl = n_long;
    for (int i = 0; i < nl; ++i)
      fold_group(long_item[i][0], long_item[i][1], long_item[i][2], long_item[i][3], wv * 4 + grp,
                 std::integral_constant<int, 16>{}, std::true_type{});
    __syncthreads();  // everyone has read the list's length before it is cleared
  }
}

template <typename T, int D>
hipError_t launch_emit_t(const KParams& kp, const Batch& b, const float* scores,
                         const int32_t* seed_rows, const int32_t* n_seeds,
                         const int32_t* slot_of, const int32_t* seg_row,
                         const int32_t* seg_start, const int32_t* n_merged, void* K_out,
                         void* V_out, float* out_mass, const int32_t* in_count,
                         int32_t* out_count, int out_stride, hipStream_t st) {
  // (unit, seed ordinal) work items; a fold wave tests 64 of them per round
  const int fold_per_unit = plan_seed_bound(kp);
  const long long items = (long long)b.n_units * fold_per_unit;
  long long fold_blocks = (items + 3) / 4;     // an item per wave ...
  if (fold_blocks > 2048) fold_blocks = 2048;  // ... up to 8192 waves
  if (fold_blocks == 0) return hipSuccess;
  emit_kernel<T, D><<<dim3((unsigned)fold_blocks), dim3(256), 0, st>>>(
      kp, b.n_units, fold_per_unit, b.row_off, static_cast<const T*>(b.K),
      static_cast<const T*>(b.V), scores, seed_rows, n_seeds, slot_of, seg_row, seg_start,
      n_merged, static_cast<T*>(K_out), static_cast<T*>(V_out), out_mass, in_count, out_count,
      out_stride);
  return hipGetLastError();
}

// ------------------------------------------------------------------ dispersion and lost mass

// Perturbation diagnostics of a finished event (Section 2.6, Appendix B).  One workgroup per
// unit; sixteen lanes per row (lanes 0-7 hold the first half of the channels, lanes 8-15 the
// second, so a band's two channels sit eight lanes apart).  A group walks rows g, g + 64, ...
// and keeps its sums in double; the 64 group sums are added in order by one thread.
template <typename T, int D>
__global__ __launch_bounds__(1024) void group_diag_kernel(
    KParams kp, const int64_t* __restrict__ row_off, const T* __restrict__ K,
    const float* __restrict__ scores, const int32_t* __restrict__ assign,
    const T* __restrict__ K_out, int out_stride, float* __restrict__ dispersion,
    float* __restrict__ lost_mass) {
  constexpr int EPL = D / 16;
  constexpr int WORDS = EPL * sizeof(T) / 4;
  struct alignas(WORDS * 4 > 16 ? 16 : WORDS * 4) Raw { uint32_t w[WORDS]; };
  __shared__ double part_d[64], part_l[64];
  const int u = blockIdx.x, tid = threadIdx.x, grp = tid >> 4, gl = tid & 15;
  const int64_t row0 = row_off[u];
  const int N = (int)(row_off[u + 1] - row0);
  float w[EPL];
#pragma unroll
  for (int e = 0; e < EPL; ++e) w[e] = kp.band_w ? kp.band_w[(gl & 7) * EPL + e] : 1.f;
  double disp = 0.0, lost = 0.0;
  for (int i = grp; i < N; i += 64) {  // the same row in all sixteen lanes of a group
    const int t = assign[row0 + i];
    const float a = scores[row0 + i];
    if (t < 0) {
      lost += (double)a;
      continue;
    }
    if (t >= kp.B) continue;
    const Raw kr = *reinterpret_cast<const Raw*>(K + (size_t)(row0 + i) * D + gl * EPL);
    const Raw rr = *reinterpret_cast<const Raw*>(K_out + ((size_t)u * out_stride + t) * D + gl * EPL);
    const T* kp_ = reinterpret_cast<const T*>(&kr);
    const T* rp_ = reinterpret_cast<const T*>(&rr);
    float r = 0.f;
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
      const float x = Elem<T>::load(kp_ + e) - Elem<T>::load(rp_ + e);
      const float sq = x * x;
      const float other = __shfl_xor(sq, 8, 64);  // the band's other channel
      r = __builtin_fmaf(w[e], __builtin_amdgcn_sqrtf(sq + other), r);
    }
    if (gl >= 8) r = 0.f;  // both halves computed the same bands
#pragma unroll
    for (int o = 4; o > 0; o >>= 1) r += __shfl_xor(r, o, 64);
    disp += (double)a * (double)r;
  }
  if (gl == 0) {
    part_d[grp] = disp;
    part_l[grp] = lost;
  }
  __syncthreads();
  if (tid == 0) {
    double sd = 0.0, sl = 0.0;
    for (int g = 0; g < 64; ++g) {
      sd += part_d[g];
      sl += part_l[g];
    }
    dispersion[u] = (float)sd;
    lost_mass[u] = (float)sl;
  }
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
                             int32_t* assign_ord, bool roles_follow_plan, hipStream_t st) {
  if (kp.geometry == 1) {
    if (kp.dtype == CASK_F32)
      return kp.d == 64 ? launch_similarity_kappa<float, 64>(kp, b, role, seed_rows, n_seeds, assign_ord, st)
                        : launch_similarity_kappa<float, 128>(kp, b, role, seed_rows, n_seeds, assign_ord, st);
    return kp.d == 64 ? launch_similarity_kappa<uint16_t, 64>(kp, b, role, seed_rows, n_seeds, assign_ord, st)
                      : launch_similarity_kappa<uint16_t, 128>(kp, b, role, seed_rows, n_seeds, assign_ord, st);
  }
  if (kp.dtype == CASK_BF16 && kp.d == 128) {
    // a few workgroups per unit, about two per compute unit in all, each walking its share of
    // the unit's donor tiles
    const int tiles = (b.max_decode_len + kDonorTile - 1) / kDonorTile;
    if (tiles == 0) return hipSuccess;
    // (with more units than workgroup slots, units of different length would leave the longest
    // ones running alone at the end: cut them into pieces of about 32 tiles instead)
    int chunks = b.n_units > 0 ? 512 / b.n_units : 1;
    if (chunks < 1) chunks = (tiles + 31) / 32;
    if (chunks < 1) chunks = 1;
    if (chunks > tiles) chunks = tiles;
    const int seed_bound = plan_seed_bound(kp);
    // (a caller-supplied role array may name any number of seeds: general kernel then)
    const bool one = roles_follow_plan && seed_bound <= kSeedBlock;
    int tiles_per_wg = (tiles + chunks - 1) / chunks;
    if (!one && tiles_per_wg > kMultiTiles) tiles_per_wg = kMultiTiles;  // its tiles' results wait in registers
    chunks = (tiles + tiles_per_wg - 1) / tiles_per_wg;
    const int units8 = (b.n_units + 7) / 8 * 8;
#define CASK_SIM(ONE, RAD)                                                             \
  similarity_mfma_kernel<ONE, RAD><<<dim3(units8 * chunks), dim3(256), 0, st>>>(       \
      kp, b.n_units, chunks, tiles_per_wg, b.row_off, b.prefix_len,                    \
      static_cast<const uint16_t*>(b.K), role, seed_rows, n_seeds, assign_ord)
    if (kp.radius > 0) {
      if (one) CASK_SIM(true, true); else CASK_SIM(false, true);
    } else {
      if (one) CASK_SIM(true, false); else CASK_SIM(false, false);
    }
#undef CASK_SIM
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
                                int32_t* status, const int32_t* n_seeds, int32_t* seg_row,
                                int32_t* seg_start, const CopyJob* copy, hipStream_t st) {
  static_assert((kGatherThreads / 64 & (kGatherThreads / 64 - 1)) == 0, "waves per block: a power of two");
  CopyJob cj{};
  long long copy_blocks = 0;
  if (copy && copy->K_out) {
    cj = *copy;
    cj.n_units = b.n_units;
    cj.lane_bytes = kp.d * (kp.dtype == CASK_F32 ? 4 : 2) / 16;
    const long long waves = (long long)b.n_units * ((kp.B + 4 * kCopyRounds - 1) / (4 * kCopyRounds));
    copy_blocks = (waves + kGatherThreads / 64 - 1) / (kGatherThreads / 64);
    if (b.n_units + copy_blocks > 0x7fffffffLL) return hipErrorInvalidValue;
  }
  // the smallest instance whose chunk covers the longest decode trace: a unit that fits one chunk
  // is then shared by all of the workgroup's waves, not by the first few
  const int per_need = (b.max_decode_len + kGatherThreads - 1) / kGatherThreads;
  auto kern = per_need <= 4 ? &gather_merged_kernel<4>
                            : (per_need <= 8 ? &gather_merged_kernel<8> : &gather_merged_kernel<kGatherPer>);
  kern<<<dim3((unsigned)(b.n_units + copy_blocks)), dim3(kGatherThreads), 0, st>>>(
      kp, b.n_units, cj, b.row_off, b.prefix_len, role, assign_ord, slot_of, seed_rows, merged_row, merged_ord,
      n_merged, assign_out, assign_mode, status, n_seeds, seg_row, seg_start);
  return hipGetLastError();
}

hipError_t launch_group_diag(const KParams& kp, const Batch& b, const float* scores,
                             const int32_t* assign, const void* K_out, int out_stride,
                             float* dispersion, float* lost_mass, hipStream_t st) {
#define CASK_GD(T, D)                                                                     \
  group_diag_kernel<T, D><<<dim3(b.n_units), dim3(1024), 0, st>>>(                        \
      kp, b.row_off, static_cast<const T*>(b.K), scores, assign, static_cast<const T*>(K_out), \
      out_stride, dispersion, lost_mass)
  if (kp.dtype == CASK_F32) {
    if (kp.d == 64) CASK_GD(float, 64); else CASK_GD(float, 128);
  } else {
    if (kp.d == 64) CASK_GD(uint16_t, 64); else CASK_GD(uint16_t, 128);
  }
#undef CASK_GD
  return hipGetLastError();
}

hipError_t launch_emit(const KParams& kp, const Batch& b, const float* scores,
                       const int32_t* seed_rows, const int32_t* n_seeds, const int32_t* slot_of,
                       const int32_t* seg_row, const int32_t* seg_start,
                       const int32_t* n_merged, void* K_out, void* V_out, float* out_mass,
                       const int32_t* in_count, int32_t* out_count, int out_stride,
                       hipStream_t st) {
#define CASK_EMIT(T, D)                                                                     \
  launch_emit_t<T, D>(kp, b, scores, seed_rows, n_seeds, slot_of, seg_row, seg_start, n_merged, \
                      K_out, V_out, out_mass, in_count, out_count, out_stride, st)
  if (kp.dtype == CASK_F32) return kp.d == 64 ? CASK_EMIT(float, 64) : CASK_EMIT(float, 128);
  return kp.d == 64 ? CASK_EMIT(uint16_t, 64) : CASK_EMIT(uint16_t, 128);
#undef CASK_EMIT
}

}  // namespace cask
