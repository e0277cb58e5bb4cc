// Selection: stage-1 prefix eviction (Section 2.2 of the paper) and the stage-2 split of the
// decode trace into protected core, representative seeds and donor scratch (Section 2.1).
//
// "Top k" is exact and order-defined: higher float score first, equal scores by ascending
// cache index.  One workgroup per unit runs an LDS radix select (4 passes of 8 bits over an
// order-preserving key image of the scores) to find the k-th key, then marks the elements;
// when the k-th value is shared by more elements than there are places left, an ordered block
// scan hands the places to the lowest indices -- no atomics decide membership.
//
// index_roles then walks the roles in index order to give every kept row its output slot
// (ascending source order, representatives at their seed's position: |R| <= B with C subset
// of R, Section 2.3) and every seed its ordinal.
#include "cask_common.h"

namespace cask {

namespace {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;

struct Kth {
  uint32_t key;   // key of the k-th element in the order
  int take_eq;    // how many elements equal to `key` belong to the top k
  int total_eq;   // how many elements equal to `key` exist in the range
};

// Block-wide radix select over s[lo, hi): the key of rank k (1 <= k <= hi - lo).
// All threads of the block must call it; `hist` is 256 ints of LDS, `bcast` 4 ints.
__device__ Kth radix_select(const float* __restrict__ s, int lo, int hi, int k, int* hist,
                            int* bcast) {
  const int tid = threadIdx.x;
  uint32_t prefix = 0, mask = 0;
  int remaining = k;
  int eq_total = 0;
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    if (tid < 256) hist[tid] = 0;
    __syncthreads();
    for (int i = lo + tid; i < hi; i += kSelThreads) {
      const uint32_t key = score_key(s[i]);
      if ((key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1);
    }
    __syncthreads();
    // wave 0: lane l owns digits 255-4l .. 252-4l (descending); find the digit where the
    // running count from the top reaches `remaining`
    if (tid < 64) {
      int h4[4];
      int local = 0;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        h4[e] = hist[255 - (tid * 4 + e)];
        local += h4[e];
      }
      int incl = local;
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const int v = __shfl_up(incl, o, 64);
        if (tid >= o) incl += v;
      }
      int before = incl - local;  // elements in digits above this lane's four
      if (before < remaining && remaining <= incl) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          if (before < remaining && remaining <= before + h4[e]) {
            bcast[0] = 255 - (tid * 4 + e);
            bcast[1] = remaining - before;
            bcast[2] = h4[e];
          }
          before += h4[e];
        }
      }
    }
    __syncthreads();
    prefix |= ((uint32_t)bcast[0]) << shift;
    mask |= 0xFFu << shift;
    remaining = bcast[1];
    eq_total = bcast[2];
    __syncthreads();
  }
  Kth r;
  r.key = prefix;
  r.take_eq = remaining;
  r.total_eq = eq_total;
  return r;
}

// Exclusive block scan of a small per-thread count (two 16-bit fields packed in one int).
// Returns the exclusive prefix; *total receives the block total.  `wsum` is kSelWaves ints.
__device__ inline int block_excl_scan(int v, int* wsum, int* total) {
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  int incl = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int t = __shfl_up(incl, o, 64);
    if (lane >= o) incl += t;
  }
  if (lane == 63) wsum[wv] = incl;
  __syncthreads();
  int base = 0, tot = 0;
  for (int w = 0; w < kSelWaves; ++w) {
    const int x = wsum[w];
    if (w < wv) base += x;
    tot += x;
  }
  __syncthreads();
  *total = tot;
  return base + incl - v;
}

__global__ __launch_bounds__(kSelThreads) void select_kernel(
    KParams kp, const int64_t* __restrict__ row_off, const int32_t* __restrict__ prefix_len,
    const float* __restrict__ scores, uint8_t* __restrict__ role, int32_t* __restrict__ status,
    int do_prefix, int do_decode) {
  __shared__ int hist[256];
  __shared__ int bcast[4];
  __shared__ int wsum[kSelWaves];
  const int u = blockIdx.x, tid = threadIdx.x;
  const int64_t row0 = row_off[u];
  const int N = (int)(row_off[u + 1] - row0);
  const int P = prefix_len[u];
  const UnitPlan pl = make_plan(kp, P, N);
  const float* s = scores + row0;
  uint8_t* ro = role + row0;
  if (tid == 0 && status) status[u] = pl.status;

  if (do_prefix && P > 0) {
    if (pl.p_keep >= P) {
      for (int i = tid; i < P; i += kSelThreads) ro[i] = CASK_ROLE_PREFIX_KEEP;
    } else if (pl.p_keep == 0) {
      for (int i = tid; i < P; i += kSelThreads) ro[i] = CASK_ROLE_PREFIX_DROP;
    } else {
      const Kth kt = radix_select(s, 0, P, pl.p_keep, hist, bcast);
      if (kt.take_eq == kt.total_eq) {
        for (int i = tid; i < P; i += kSelThreads)
          ro[i] = score_key(s[i]) >= kt.key ? CASK_ROLE_PREFIX_KEEP : CASK_ROLE_PREFIX_DROP;
      } else {
        int seen = 0;  // elements equal to the k-th key at lower indices
        for (int base = 0; base < P; base += kSelThreads) {
          const int i = base + tid;
          const uint32_t key = i < P ? score_key(s[i]) : 0u;
          const int eq = (i < P && key == kt.key) ? 1 : 0;
          int tot;
          const int ex = block_excl_scan(eq, wsum, &tot);
          if (i < P) {
            const bool keep = key > kt.key || (eq && seen + ex < kt.take_eq);
            ro[i] = keep ? CASK_ROLE_PREFIX_KEEP : CASK_ROLE_PREFIX_DROP;
          }
          seen += tot;
        }
      }
    }
  }

  if (do_decode) {
    const int hi = N - pl.r_eff;
    for (int i = hi + tid; i < N; i += kSelThreads) ro[i] = CASK_ROLE_RECENT;
    const int n = hi - P;
    if (n <= 0) return;
    if (pl.status & CASK_ST_PREFIX_BUDGET_EXHAUSTED) {
      for (int i = P + tid; i < hi; i += kSelThreads) ro[i] = CASK_ROLE_DECODE_EVICT;
      return;
    }
    const int C = pl.core, CM = pl.core + pl.seeds;
    if (C >= n) {
      for (int i = P + tid; i < hi; i += kSelThreads) ro[i] = CASK_ROLE_CORE;
      return;
    }
    // thresholds of rank C (core) and rank C+M (core and seeds); a rank of 0 selects nothing
    Kth kc, km;
    kc.key = 0xFFFFFFFFu; kc.take_eq = 0; kc.total_eq = 0;
    km = kc;
    if (C > 0) kc = radix_select(s, P, hi, C, hist, bcast);
    if (CM >= n) {
      km.key = 0u; km.take_eq = 0; km.total_eq = 0;  // everything not core is a seed
    } else if (CM > C) {
      km = radix_select(s, P, hi, CM, hist, bcast);
    } else {
      km = kc;
    }
    const bool all_seed = CM >= n;
    const bool ties = (C > 0 && kc.take_eq != kc.total_eq) ||
                      (!all_seed && CM > 0 && km.take_eq != km.total_eq);
    if (!ties) {
      for (int i = P + tid; i < hi; i += kSelThreads) {
        const uint32_t key = score_key(s[i]);
        const bool in_c = C > 0 && key >= kc.key;
        const bool in_cm = all_seed || (CM > 0 && key >= km.key);
        ro[i] = in_c ? CASK_ROLE_CORE : (in_cm ? CASK_ROLE_SEED : CASK_ROLE_DONOR);
      }
    } else {
      int seen_c = 0, seen_m = 0;
      for (int base = P; base < hi; base += kSelThreads) {
        const int i = base + tid;
        const bool in = i < hi;
        const uint32_t key = in ? score_key(s[i]) : 0u;
        const int eq_c = (in && C > 0 && key == kc.key) ? 1 : 0;
        const int eq_m = (in && !all_seed && CM > 0 && key == km.key) ? 1 : 0;
        int tot;
        const int ex = block_excl_scan(eq_c | (eq_m << 16), wsum, &tot);
        if (in) {
          const bool in_c = C > 0 && (key > kc.key || (eq_c && seen_c + (ex & 0xFFFF) < kc.take_eq));
          const bool in_cm = all_seed || (CM > 0 && (key > km.key || (eq_m && seen_m + (ex >> 16) < km.take_eq)));
          ro[i] = in_c ? CASK_ROLE_CORE : (in_cm ? CASK_ROLE_SEED : CASK_ROLE_DONOR);
        }
        seen_c += tot & 0xFFFF;
        seen_m += tot >> 16;
      }
    }
  }
}

// Ordered walk over the roles of a unit: output slot of every kept row, ordinal of every seed.
__global__ __launch_bounds__(kSelThreads) void index_roles_kernel(
    KParams kp, const int64_t* __restrict__ row_off, const uint8_t* __restrict__ role,
    int32_t* __restrict__ slot_of, int32_t* __restrict__ out_src, int32_t* __restrict__ out_len,
    int32_t* __restrict__ seed_rows, int32_t* __restrict__ ord_of_slot,
    int32_t* __restrict__ n_seeds) {
  __shared__ int wsum[kSelWaves];
  const int u = blockIdx.x, tid = threadIdx.x;
  const int64_t row0 = row_off[u];
  const int N = (int)(row_off[u + 1] - row0);
  const uint8_t* ro = role + row0;
  const int B = kp.B;
  int kept_before = 0, seeds_before = 0;
  for (int base = 0; base < N; base += kSelThreads) {
    const int i = base + tid;
    const int r = i < N ? ro[i] : CASK_ROLE_PREFIX_DROP;
    const int is_seed = (r == CASK_ROLE_SEED) ? 1 : 0;
    const int kept = (r == CASK_ROLE_PREFIX_KEEP || r == CASK_ROLE_CORE || r == CASK_ROLE_RECENT ||
                      is_seed) ? 1 : 0;
    int tot;
    const int ex = block_excl_scan(kept | (is_seed << 16), wsum, &tot);
    if (i < N) {
      const int slot = kept_before + (ex & 0xFFFF);
      const int ord = seeds_before + (ex >> 16);
      // a caller-supplied role array could keep more rows than the budget: never write
      // past the unit's B output slots
      const bool fits = kept && slot < B;
      if (slot_of) slot_of[row0 + i] = fits ? slot : -1;
      if (fits) {
        if (out_src) out_src[(size_t)u * B + slot] = i;
        if (ord_of_slot) ord_of_slot[(size_t)u * B + slot] = is_seed ? ord : -1;
      }
      if (is_seed && ord < B) seed_rows[(size_t)u * B + ord] = i;
    }
    kept_before += tot & 0xFFFF;
    seeds_before += tot >> 16;
  }
  if (tid == 0) {
    if (out_len) out_len[u] = kept_before < B ? kept_before : B;
    n_seeds[u] = seeds_before < B ? seeds_before : B;
  }
}

}  // namespace

hipError_t launch_select(const KParams& kp, const Batch& b, const float* scores, uint8_t* role,
                         int32_t* status, bool do_prefix, bool do_decode, hipStream_t st) {
  select_kernel<<<dim3(b.n_units), dim3(kSelThreads), 0, st>>>(
      kp, b.row_off, b.prefix_len, scores, role, status, do_prefix ? 1 : 0, do_decode ? 1 : 0);
  return hipGetLastError();
}

hipError_t launch_index_roles(const KParams& kp, const Batch& b, const uint8_t* role,
                              int32_t* slot_of, int32_t* out_src, int32_t* out_len,
                              int32_t* seed_rows, int32_t* ord_of_slot, int32_t* n_seeds,
                              hipStream_t st) {
  index_roles_kernel<<<dim3(b.n_units), dim3(kSelThreads), 0, st>>>(
      kp, b.row_off, role, slot_of, out_src, out_len, seed_rows, ord_of_slot, n_seeds);
  return hipGetLastError();
}

}  // namespace cask
