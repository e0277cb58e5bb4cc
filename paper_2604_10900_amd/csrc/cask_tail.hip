// Everything after scoring in ONE launch, for units short enough that a workgroup holds a row
// per thread (the steady state of a decode loop: an event fires at budget + a few hundred
// rows).  Same results as the general kernels (select, similarity, gather, emit) up to the
// rounding of the cosines; what it saves is their launches and the trips through memory
// between them.  bf16 caches, cosine geometry (Sections 2.1 - 2.4).
#include <hip/hip_runtime.h>

#include "cask.h"
#include "cask_common.h"

namespace cask {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kTailThreads = 1024;
constexpr int kTailWaves = kTailThreads / 64;
constexpr int kTailRows = kTailThreads;  // longest unit: a row per thread
constexpr int kTailSeedBlock = 128;      // seeds staged in LDS at a time
constexpr float kNegInf = -__builtin_inff();
constexpr int kRepFlag = 0x4000;         // in src_s: the slot holds a representative (rows are < 1024)

__device__ inline float sumsq8(const uint4& v) {
  const uint32_t w[4] = {v.x, v.y, v.z, v.w};
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const bf16x2 x = __builtin_bit_cast(bf16x2, w[i]);
    s = __builtin_amdgcn_fdot2_f32_bf16(x, x, s, false);
  }
  return s;
}

// Thread i owns row i of the unit.
//  1. rank: the order (score descending, index ascending) becomes one 64-bit key per row
//     (score key, then inverted index), and a row's rank inside its range (prefix, or decode
//     trace without the recent tail) is the number of larger keys: a counting loop over LDS,
//     split over the idle threads when the unit is shorter than the workgroup.
//  2. roles from the plan's ranks; output slots and seed ordinals from one block scan.
//  3. cosine of every decode row against every seed on the matrix cores: seeds are the A
//     operand (staged in LDS kTailSeedBlock at a time, with inverse norms), 32 decode rows a
//     tile are the B operand straight from memory, so a lane owns one row and sees its seeds
//     in ascending order: first maximum wins, folded if >= tau.
//  4. kept rows are copied 16 bytes a thread; a wave per seed with donors folds its group in
//     ascending row order in fp32 (score-weighted; count-weighted when the group has no mass).
template <int D>
__global__ __launch_bounds__(kTailThreads) void tail_small_kernel(
    KParams kp, const int64_t* __restrict__ row_off, const int32_t* __restrict__ prefix_len,
    float* scores, const float* __restrict__ parts, int n_parts, int parts_pitch,
    const uint16_t* __restrict__ K,
    const uint16_t* __restrict__ V, const int32_t* __restrict__ in_count,
    uint16_t* __restrict__ K_out, uint16_t* __restrict__ V_out, int out_stride,
    int32_t* __restrict__ out_len, int32_t* __restrict__ out_src, float* __restrict__ out_mass,
    int32_t* __restrict__ out_count, int32_t* __restrict__ assign, int32_t* __restrict__ status) {
  constexpr int ROWB = D * 2;      // bytes per row
  constexpr int PITCH = ROWB + 16; // LDS row pitch of a staged seed: 16-byte reads of 16 rows hit 64 banks
  constexpr int KS = D / 16;       // MFMA k-steps
  constexpr int PPR = ROWB / 16;   // 16-byte pieces per row
  __shared__ __attribute__((aligned(16))) unsigned char seedk[kTailSeedBlock * PITCH];
  __shared__ unsigned long long ckey[kTailRows];  // step 1; afterwards its memory holds bsim
  __shared__ int rank_s[kTailRows];               // step 1; afterwards the donors per seed (seg_cnt)
  __shared__ short slot_s[kTailRows];             // output slot of a row, -1 if it is not kept
  __shared__ short fold_s[kTailRows];             // seed ordinal a row belongs to (seeds: their own), -1 if none
  __shared__ short seed_row_s[kTailRows];         // row of every seed ordinal
  __shared__ short src_s[kTailRows];              // row of every output slot
  __shared__ float seed_inv[kTailSeedBlock];
  __shared__ int wsum[kTailWaves];
  float* bsim_s = reinterpret_cast<float*>(ckey);
  int* seg_cnt = rank_s;

  const int u = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int64_t row0 = row_off[u];
  const int N = (int)(row_off[u + 1] - row0);  // <= kTailRows: the host checked
  const int P = prefix_len[u];
  const UnitPlan pl = make_plan(kp, P, N);
  const int hi = N - pl.r_eff;
  const int B = kp.B;
  const float* s = scores + row0;
  const uint16_t* Ku = K + (size_t)row0 * D;
  const uint16_t* Vu = V + (size_t)row0 * D;
  const int i = tid;

  // ---- 1. ranks
  float my_s = 0.f;
  if (i < N) {
    if (parts) {
      // the one-launch scoring left partial column sums: add them in order, scale, publish
      const float* pp = parts + (size_t)u * n_parts * parts_pitch + i;
      float tot = 0.f;
      for (int q0 = 0; q0 < n_parts; q0 += 8) {  // eight loads in flight, added in order
        float v[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = pp[(size_t)min(q0 + e, n_parts - 1) * parts_pitch];
#pragma unroll
        for (int e = 0; e < 8; ++e)
          if (q0 + e < n_parts) tot += v[e];
      }
      my_s = tot * (1.0f / (float)kp.Mq);
      scores[row0 + i] = my_s;  // read again below by other threads, behind barriers
    } else {
      my_s = s[i];
    }
  }
  ckey[i] = i < N ? (((unsigned long long)score_key(my_s)) << 32) | (unsigned)(~i) : 0ull;
  rank_s[i] = 0;
  __syncthreads();
  {
    int shift = 10;  // rows_per = 1 << shift threads cover the rows once; the rest split the loop
    if (N <= 256) shift = 8;
    else if (N <= 512) shift = 9;
    const int parts = kTailThreads >> shift;
    const int r = tid & ((1 << shift) - 1), part = tid >> shift;
    const bool prefix_row = r < P;
    // a range that is kept or dropped as a whole needs no ranks
    const bool need = prefix_row ? (pl.p_keep > 0 && pl.p_keep < P) : (r < hi && pl.core < hi - P);
    if (need) {
      const int lo_r = prefix_row ? 0 : P, hi_r = prefix_row ? P : hi;
      const int per = (hi_r - lo_r + parts - 1) / parts;
      const int j0 = lo_r + part * per, j1 = min(hi_r, j0 + per);
      const unsigned long long me = ckey[r];
      int cnt = 0, j = j0;
      for (; j + 8 <= j1; j += 8) {  // eight independent LDS reads in flight
        unsigned long long kj[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) kj[e] = ckey[j + e];
#pragma unroll
        for (int e = 0; e < 8; ++e) cnt += kj[e] > me ? 1 : 0;
      }
      for (; j < j1; ++j) cnt += ckey[j] > me ? 1 : 0;
      if (cnt) atomicAdd(&rank_s[r], cnt);
    }
  }
  __syncthreads();

  // ---- 2. roles, slots, seed ordinals
  bool kept = false, seed = false, donor = false;
  if (i < N) {
    const int rk = rank_s[i];
    if (i < P) {
      kept = rk < pl.p_keep;  // ranks are zero when the whole prefix stays or goes
    } else if (i >= hi) {
      kept = true;
    } else {
      const bool core = rk < pl.core;  // zero ranks: core >= range, all core
      seed = !core && rk < pl.core + pl.seeds;
      kept = core || seed;
      donor = !kept;
    }
  }
  const unsigned long long below = (1ull << lane) - 1ull;
  const unsigned long long bk = __ballot(kept), bs = __ballot(seed);
  if (lane == 0) wsum[wv] = __popcll(bk) | (__popcll(bs) << 16);
  __syncthreads();  // also: every rank has been read, seg_cnt may reuse the memory
  int base = 0, tot = 0;
  for (int w = 0; w < kTailWaves; ++w) {
    const int x = wsum[w];
    if (w < wv) base += x;
    tot += x;
  }
  const int n_kept = tot & 0xFFFF, M = tot >> 16;
  const int L = n_kept < B ? n_kept : B;
  int slot = kept ? (base & 0xFFFF) + __popcll(bk & below) : -1;
  if (slot >= B) slot = -1;
  const int ord = seed ? (base >> 16) + __popcll(bs & below) : -1;
  slot_s[i] = (short)slot;
  if (slot >= 0) src_s[slot] = (short)i;
  if (seed) seed_row_s[ord] = (short)i;
  fold_s[i] = -1;
  bsim_s[i] = kNegInf;
  seg_cnt[i] = 0;
  __syncthreads();

  // ---- 3. cosine against the seeds
  const int n = hi - P;
  if (M > 0 && n > pl.core + pl.seeds) {  // there are seeds and there are donors
    const int c32 = lane & 31, h = lane >> 5;
    const int n_tiles = (n + 31) / 32;
    const int radius = kp.radius > 0 ? kp.radius : 0x7fffffff;
    // a decode row's operand: pieces h, h + 2, ... of its key, and its inverse norm
    auto load_tile = [&](int t, bf16x8 (&bres)[KS], float& dinv) {
      const int drow = P + t * 32 + c32;
      const int lrow = drow < hi ? drow : hi - 1;
      float ss = 0.f;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const uint4 v = *reinterpret_cast<const uint4*>(Ku + (size_t)lrow * D + (2 * ks + h) * 8);
        ss += sumsq8(v);
        bres[ks] = __builtin_bit_cast(bf16x8, v);
      }
      ss += __shfl_xor(ss, 32, 64);
      dinv = ss > 0.f ? 1.0f / sqrtf(ss) : 0.f;
    };
    // the wave's first tile is requested before the seeds are staged, so that both trips to
    // memory overlap (with at most 16 tiles and one seed block that is all there is)
    bf16x8 bfirst[KS];
    float dinv_first = 0.f;
    if (wv < n_tiles) load_tile(wv, bfirst, dinv_first);
    for (int sb = 0; sb < M; sb += kTailSeedBlock) {
      if (sb > 0) __syncthreads();  // the previous block has been consumed
      {  // 16 threads a row, 64 rows a pass; the loads of both passes are issued together and
         // without a branch around them (a row past the last seed reads the last seed again)
        static_assert(kTailSeedBlock == 128, "two passes of 64 rows");
        const int piece = (tid & 15) < PPR ? (tid & 15) : PPR - 1;
        uint4 v[2];
#pragma unroll
        for (int e = 0; e < 2; ++e) {
          const int o = sb + e * 64 + (tid >> 4);
          v[e] = *reinterpret_cast<const uint4*>(Ku + (size_t)seed_row_s[o < M ? o : M - 1] * D + piece * 8);
        }
#pragma unroll
        for (int e = 0; e < 2; ++e) {
          const int sr = e * 64 + (tid >> 4);
          const bool live = (tid & 15) < PPR && sb + sr < M;
          if (!live) v[e] = make_uint4(0, 0, 0, 0);
          if ((tid & 15) < PPR) *reinterpret_cast<uint4*>(seedk + sr * PITCH + piece * 16) = v[e];
          float ss = sumsq8(v[e]);
#pragma unroll
          for (int x = 8; x > 0; x >>= 1) ss += __shfl_xor(ss, x, 64);
          if ((tid & 15) == 0) seed_inv[sr] = ss > 0.f ? 1.0f / sqrtf(ss) : 0.f;
        }
      }
      __syncthreads();
      const int m_blk = min(kTailSeedBlock, M - sb);
      for (int t = wv; t < n_tiles; t += kTailWaves) {
        const int drow = P + t * 32 + c32;
        const bool valid = drow < hi;
        bf16x8 bres[KS];
        float dinv;
        if (t == wv) {
#pragma unroll
          for (int ks = 0; ks < KS; ++ks) bres[ks] = bfirst[ks];
          dinv = dinv_first;
        } else {
          load_tile(t, bres, dinv);
        }
        float best = kNegInf;
        int best_ord = -1;
        for (int s0 = 0; s0 < m_blk; s0 += 32) {
          f32x16 acc = {0};
#pragma unroll
          for (int ks = 0; ks < KS; ++ks) {
            const bf16x8 a = *reinterpret_cast<const bf16x8*>(seedk + (s0 + c32) * PITCH + (2 * ks + h) * 16);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bres[ks], acc, 0, 0, 0);
          }
#pragma unroll
          for (int g = 0; g < 4; ++g) {  // ascending seed ordinal within the lane
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              const int sr = s0 + g * 8 + h * 4 + q;
              if (sr < m_blk) {
                const float sim = (acc[g * 4 + q] * seed_inv[sr]) * dinv;
                const int pos = seed_row_s[sb + sr];
                const int gap = pos > drow ? pos - drow : drow - pos;
                if (gap <= radius && sim > best) {
                  best = sim;
                  best_ord = sb + sr;
                }
              }
            }
          }
        }
        const float ob = __shfl_xor(best, 32, 64);
        const int oo = __shfl_xor(best_ord, 32, 64);
        if (oo >= 0 && (best_ord < 0 || ob > best || (ob == best && oo < best_ord))) {
          best = ob;
          best_ord = oo;
        }
        // later blocks hold higher ordinals: only a strictly larger cosine replaces
        if (h == 0 && valid && best_ord >= 0 && (fold_s[drow] < 0 || best > bsim_s[drow])) {
          bsim_s[drow] = best;
          fold_s[drow] = (short)best_ord;
        }
      }
    }
    __syncthreads();
  }
  int target = -1;
  if (donor) {
    const int o = fold_s[i];
    if (o >= 0 && bsim_s[i] >= kp.tau) target = o;
  }
  __syncthreads();  // every candidate has been read before the array changes meaning
  fold_s[i] = (short)(seed ? ord : target);
  if (target >= 0) atomicAdd(&seg_cnt[target], 1);
  const int n_fold = __syncthreads_count(target >= 0 ? 1 : 0);

  // ---- 4. outputs
  if (tid < L) {
    const int src = src_s[tid];
    const int g = fold_s[src];
    out_src[(size_t)u * B + tid] = src;
    if (g >= 0 && seg_cnt[g] > 0) {
      src_s[tid] = (short)(src | kRepFlag);  // a representative: a fold wave writes this slot
    } else {                                 // the row stands for itself
      if (out_mass) out_mass[(size_t)u * B + tid] = s[src];
      if (out_count) out_count[(size_t)u * B + tid] = in_count ? in_count[row0 + src] : 1;
    }
  }
  __syncthreads();
  {
    constexpr int PER_SLOT = 2 * PPR;  // K pieces, then V pieces
    constexpr int NB = 12;             // loads in flight per thread
    const int pieces = L * PER_SLOT;
    uint16_t* Ko = K_out + (size_t)u * out_stride * D;
    uint16_t* Vo = V_out + (size_t)u * out_stride * D;
    for (int p0 = tid; p0 < pieces; p0 += NB * kTailThreads) {
      // every load is issued, without a branch around it (past the end the last piece is
      // read again, a representative's own row is read in vain): only the stores are
      // conditional, so all NB loads are in flight together
      uint4 v[NB];
      int dst[NB];  // element offset in the unit's output, V flagged by bit 30; -1: no store
#pragma unroll
      for (int e = 0; e < NB; ++e) {
        const int p = p0 + e * kTailThreads;
        const int pc = p < pieces ? p : pieces - 1;
        const int t = pc / PER_SLOT, w = pc % PER_SLOT;
        const bool is_v = w >= PPR;
        const int piece = is_v ? w - PPR : w;
        const int src = src_s[t];
        v[e] = *reinterpret_cast<const uint4*>((is_v ? Vu : Ku) + (size_t)(src & (kRepFlag - 1)) * D + piece * 8);
        dst[e] = (p < pieces && !(src & kRepFlag)) ? ((t * D + piece * 8) | (is_v ? (1 << 30) : 0)) : -1;
      }
      // (keeps the compiler from sinking each load into the branch of its store)
#pragma unroll
      for (int e = 0; e < NB; e += 4)
        asm volatile("" : "+v"(v[e].x), "+v"(v[e].y), "+v"(v[e].z), "+v"(v[e].w),
                          "+v"(v[e + 1].x), "+v"(v[e + 1].y), "+v"(v[e + 1].z), "+v"(v[e + 1].w),
                          "+v"(v[e + 2].x), "+v"(v[e + 2].y), "+v"(v[e + 2].z), "+v"(v[e + 2].w),
                          "+v"(v[e + 3].x), "+v"(v[e + 3].y), "+v"(v[e + 3].z), "+v"(v[e + 3].w));
#pragma unroll
      for (int e = 0; e < NB; ++e)
        if (dst[e] >= 0)
          *reinterpret_cast<uint4*>(((dst[e] >> 30) ? Vo : Ko) + (dst[e] & ((1 << 30) - 1))) = v[e];
    }
  }
  if (n_fold > 0) {
    const bool active = lane < D / 2;  // two elements a lane
    for (int g = wv; g < M; g += kTailWaves) {
      if (seg_cnt[g] == 0) continue;
      float ka[2] = {0.f, 0.f}, va[2] = {0.f, 0.f}, ku[2] = {0.f, 0.f}, vu[2] = {0.f, 0.f};
      float mass = 0.f;
      int count = 0;
      for (int c0 = P; c0 < hi; c0 += 64) {  // the seed itself and its donors, ascending rows
        const int j = c0 + lane;
        unsigned long long mask = __ballot(j < hi && fold_s[j] == g);
        while (mask != 0ull) {
          int rows[4], nrows = 0;
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            if (mask != 0ull) {
              rows[q] = c0 + __ffsll((long long)mask) - 1;
              mask &= mask - 1ull;
              ++nrows;
            } else {
              rows[q] = rows[0];
            }
          }
          float a[4];
          int dc[4];
          uint32_t kw[4], vw[4];
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            a[q] = s[rows[q]];
            dc[q] = in_count ? in_count[row0 + rows[q]] : 1;
            kw[q] = active ? *reinterpret_cast<const uint32_t*>(Ku + (size_t)rows[q] * D + lane * 2) : 0u;
            vw[q] = active ? *reinterpret_cast<const uint32_t*>(Vu + (size_t)rows[q] * D + lane * 2) : 0u;
          }
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            if (q < nrows) {
              const float dcf = (float)dc[q];
              const float k0 = __uint_as_float(kw[q] << 16), k1 = __uint_as_float(kw[q] & 0xffff0000u);
              const float v0 = __uint_as_float(vw[q] << 16), v1 = __uint_as_float(vw[q] & 0xffff0000u);
              ka[0] = __builtin_fmaf(a[q], k0, ka[0]); ka[1] = __builtin_fmaf(a[q], k1, ka[1]);
              va[0] = __builtin_fmaf(a[q], v0, va[0]); va[1] = __builtin_fmaf(a[q], v1, va[1]);
              ku[0] = __builtin_fmaf(dcf, k0, ku[0]); ku[1] = __builtin_fmaf(dcf, k1, ku[1]);
              vu[0] = __builtin_fmaf(dcf, v0, vu[0]); vu[1] = __builtin_fmaf(dcf, v1, vu[1]);
              mass += a[q];
              count += dc[q];
            }
          }
        }
      }
      const int t = slot_s[seed_row_s[g]];
      if (t < 0) continue;
      const bool uniform = mass == 0.f;  // no score mass: average over the original tokens
      const float denom = uniform ? (float)count : mass;
      if (active) {
        const uint32_t ko = (uint32_t)float_to_bf16_bits((uniform ? ku[0] : ka[0]) / denom) |
                            ((uint32_t)float_to_bf16_bits((uniform ? ku[1] : ka[1]) / denom) << 16);
        const uint32_t vo = (uint32_t)float_to_bf16_bits((uniform ? vu[0] : va[0]) / denom) |
                            ((uint32_t)float_to_bf16_bits((uniform ? vu[1] : va[1]) / denom) << 16);
        *reinterpret_cast<uint32_t*>(K_out + ((size_t)u * out_stride + t) * D + lane * 2) = ko;
        *reinterpret_cast<uint32_t*>(V_out + ((size_t)u * out_stride + t) * D + lane * 2) = vo;
      }
      if (lane == 0) {
        if (out_mass) out_mass[(size_t)u * B + t] = mass;
        if (out_count) out_count[(size_t)u * B + t] = count;
      }
    }
  }
  if (assign && i < N) {
    int v = slot;
    if (target >= 0) v = slot_s[seed_row_s[target]];
    assign[row0 + i] = v;
  }
  if (tid == 0) {
    out_len[u] = L;
    int st = pl.status;
    if (n_fold == 0 && !(st & (CASK_ST_IDENTITY | CASK_ST_PREFIX_BUDGET_EXHAUSTED))) st |= CASK_ST_MERGE_INACTIVE;
    status[u] = st;
  }
}

}  // namespace

bool tail_small_fits(const KParams& kp, const Batch& b) {
  return kp.dtype == CASK_BF16 && kp.geometry == 0 && b.max_unit_len <= kTailRows && kp.B <= kTailRows;
}

hipError_t launch_tail_small(const KParams& kp, const Batch& b, float* scores, const float* parts,
                             int n_parts, int parts_pitch, const int32_t* in_count, void* K_out, void* V_out, int out_stride,
                             int32_t* out_len, int32_t* out_src, float* out_mass,
                             int32_t* out_count, int32_t* assign, int32_t* status,
                             hipStream_t st) {
  if (!tail_small_fits(kp, b)) return hipErrorInvalidValue;
#define CASK_TAIL(D)                                                                             \
  tail_small_kernel<D><<<dim3(b.n_units), dim3(kTailThreads), 0, st>>>(                          \
      kp, b.row_off, b.prefix_len, scores, parts, n_parts, parts_pitch,                          \
      static_cast<const uint16_t*>(b.K),                                                         \
      static_cast<const uint16_t*>(b.V), in_count, static_cast<uint16_t*>(K_out),                \
      static_cast<uint16_t*>(V_out), out_stride, out_len, out_src, out_mass, out_count, assign,  \
      status)
  if (kp.d == 64) CASK_TAIL(64); else CASK_TAIL(128);
#undef CASK_TAIL
  return hipGetLastError();
}

}  // namespace cask
