// Selection: stage-1 prefix eviction (Section 2.2 of the paper) and the stage-2 split of the
// decode trace into protected core, representative seeds and donor scratch (Section 2.1).
//
// "Top k" is exact and order-defined: higher float score first, equal scores by ascending
// cache index.  One workgroup per unit runs an LDS radix select (up to 4 passes of 8 bits over
// an order-preserving key image of the scores, ending early once every rank's boundary bucket
// is taken whole; the three ranks a unit needs -- prefix keep, core, core + seeds -- are found
// in the same passes, or the prefix rank in a walk of its own where that reads fewer keys) to
// find the k-th keys, then marks the elements;
// when the k-th value is shared by more elements than there are places left, an ordered block
// scan hands the places to the lowest indices -- no atomics decide membership.
//
// index_roles then walks the roles in index order to give every kept row its output slot
// (ascending source order, representatives at their seed's position: |R| <= B with C subset
// of R, Section 2.3) and every seed its ordinal.
#include <type_traits>

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

// Up to three rank queries answered together by one block-wide radix select (4 passes of 8
// bits): query q asks for the key of rank k[q] (1 <= k <= hi - lo) among s[lo[q], hi[q]).
// Every pass walks the rows of the active ranges once and feeds one LDS histogram per query;
// wave q then finds the digit of query q.  Inactive queries (k <= 0) are skipped.
// Scores of one unit crowd into a few digits (the top byte holds sign and exponent), and LDS
// atomics on one address serialise; so every histogram exists in kHistCopies copies, a lane
// adds to copy lane % kHistCopies, and the copies are summed in the digit search.
// All threads of the block must call it; `hist` is 2 x 3 x 256 x kHistCopies ints of LDS, `bcast`
// 3 x 4 ints.
constexpr int kHistCopies = 8;
struct Query3 {
  int lo[3], hi[3], k[3];
};

// The number of keys a thread holds at a time is the template parameter PER of the selection (a
// chunk is PER * 1024 rows).  The straight-line code over a thread's keys costs what PER says
// whatever the unit's length, and a unit that fits one chunk keeps its keys in registers across
// the four passes, so the launcher takes the smallest instance that covers the longest unit.
constexpr int kSelPerDefault = 16;

// keys of rows base + e * kSelThreads + tid, e < PER (0 past `end`): all loads of the
// chunk are in flight together
template <int PER>
__device__ inline void load_keys(const float* __restrict__ s, int base, int end, uint32_t (&key)[PER]) {
  float v[PER];
#pragma unroll
  for (int e = 0; e < PER; ++e) {
    const int i = base + e * kSelThreads + (int)threadIdx.x;
    v[e] = i < end ? s[i] : 0.f;
  }
#pragma unroll
  for (int e = 0; e < PER; ++e) key[e] = score_key(v[e]);
}

// `key` holds the chunk starting at lo_all on return when the ranges fit one chunk
// (hi_all - lo_all <= kSelChunk), so the caller can mark the rows without reading them again.
// `early`: the caller only compares keys against the result when a query's k-th value is not
// shared beyond the rank (take_eq == total_eq), so the passes may stop as soon as every query's
// boundary bucket is taken whole; the key then has its remaining low digits zero (a lower
// bound of the bucket: "key >= result" still separates the top k).
template <int PER>
__device__ void radix_select3(const float* __restrict__ s, const Query3& q, int lo_all, int hi_all,
                              Kth (&out)[3], uint32_t (&key)[PER], int* hist, int* bcast, bool early) {
  constexpr int kSelChunk = kSelThreads * PER;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  uint32_t prefix[3] = {0, 0, 0};
  uint32_t mask = 0;
  int remaining[3] = {q.k[0], q.k[1], q.k[2]};
  int eq_total[3] = {0, 0, 0};
  const bool single = hi_all - lo_all <= kSelChunk;
  // single chunk: bit j of live[e] says that row e of this thread still competes in query j
  // (inside its range, all digits so far equal to the chosen ones), so later passes skip most
  // rows with one test
  uint32_t live[PER];
  if (single) {
    load_keys<PER>(s, lo_all, hi_all, key);
#pragma unroll
    for (int e = 0; e < PER; ++e) {
      const int i = lo_all + e * kSelThreads + tid;
      live[e] = 0;
#pragma unroll
      for (int j = 0; j < 3; ++j)
        if (q.k[j] > 0 && i >= q.lo[j] && i < q.hi[j]) live[e] |= 1u << j;
    }
  }
  // queries 1 and 2 over one range have the same first histogram: count it once
  const bool same12 = q.k[1] > 0 && q.k[2] > 0 && q.lo[1] == q.lo[2] && q.hi[1] == q.hi[2];
  // Two barriers per pass: rows are counted into one histogram buffer while the other one is
  // cleared for the next pass; then wave j sums the copies of query j's digits and finds the
  // digit; the threads pick the result up after the second barrier.
  constexpr int kHistInts = 768 * kHistCopies;
  for (int b = tid; b < kHistInts; b += kSelThreads) hist[b] = 0;
  __syncthreads();
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    int* cur = hist + (pass & 1) * kHistInts;
    int* nxt = hist + ((pass & 1) ^ 1) * kHistInts;
    for (int b = tid; b < kHistInts; b += kSelThreads) nxt[b] = 0;
    const bool share = same12 && pass == 0;
    if (single) {
#pragma unroll
      for (int e = 0; e < PER; ++e) {
        uint32_t lv = live[e];
        if (share) lv &= ~4u;
        if (lv != 0u) {
          const uint32_t digit = (key[e] >> shift) & 255u;
#pragma unroll
          for (int j = 0; j < 3; ++j)
            if (lv & (1u << j))
              atomicAdd(&cur[(j * 256 + digit) * kHistCopies + (tid & (kHistCopies - 1))], 1);
        }
      }
    } else {
      for (int base = lo_all; base < hi_all; base += kSelChunk) {
        load_keys<PER>(s, base, hi_all, key);
#pragma unroll
        for (int e = 0; e < PER; ++e) {
          const int i = base + e * kSelThreads + tid;
          const uint32_t digit = (key[e] >> shift) & 255u;
#pragma unroll
          for (int j = 0; j < 3; ++j)
            if (q.k[j] > 0 && !(share && j == 2) && i >= q.lo[j] && i < q.hi[j] &&
                (key[e] & mask) == prefix[j])
              atomicAdd(&cur[(j * 256 + digit) * kHistCopies + (tid & (kHistCopies - 1))], 1);
        }
      }
    }
    __syncthreads();
    // wave j: lane l owns digits 255-4l .. 252-4l (descending) of query j (query 2 reads query
    // 1's counts while they are shared); find the digit where the running count from the top
    // reaches `remaining`
    const int qk_w = wv == 0 ? q.k[0] : (wv == 1 ? q.k[1] : q.k[2]);  // (no indexing by wave: that would put q in memory)
    if (wv < 3 && qk_w > 0) {
      const int rem = wv == 0 ? remaining[0] : (wv == 1 ? remaining[1] : remaining[2]);
      const int* hq = cur + ((share && wv == 2) ? 1 : wv) * 256 * kHistCopies;
      int h4[4];
      int local = 0;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int* bin = hq + (255 - (lane * 4 + e)) * kHistCopies;
        int sum = 0;
#pragma unroll
        for (int cpy = 0; cpy < kHistCopies; ++cpy) sum += bin[(cpy + lane) & (kHistCopies - 1)];
        h4[e] = sum;
        local += sum;
      }
      int incl = local;
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const int v = __shfl_up(incl, o, 64);
        if (lane >= o) incl += v;
      }
      int before = incl - local;  // elements in digits above this lane's four
      if (before < rem && rem <= incl) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          if (before < rem && rem <= before + h4[e]) {
            bcast[wv * 4 + 0] = 255 - (lane * 4 + e);
            bcast[wv * 4 + 1] = rem - before;
            bcast[wv * 4 + 2] = h4[e];
          }
          before += h4[e];
        }
      }
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < 3; ++j)
      if (q.k[j] > 0) {
        prefix[j] |= ((uint32_t)bcast[j * 4 + 0]) << shift;
        remaining[j] = bcast[j * 4 + 1];
        eq_total[j] = bcast[j * 4 + 2];
      }
    mask |= 0xFFu << shift;
    if (early && pass < 3) {
      // (the same values in every thread: they come from the broadcast words)
      bool whole = true;
#pragma unroll
      for (int j = 0; j < 3; ++j)
        if (q.k[j] > 0 && remaining[j] != eq_total[j]) whole = false;
      if (whole) break;
    }
    if (single) {
#pragma unroll
      for (int e = 0; e < PER; ++e) {
        if (live[e] != 0u) {
#pragma unroll
          for (int j = 0; j < 3; ++j)
            if ((live[e] & (1u << j)) && (key[e] & mask) != prefix[j]) live[e] &= ~(1u << j);
        }
      }
    }
  }
  __syncthreads();  // the caller may reuse `bcast` and `hist`
#pragma unroll
  for (int j = 0; j < 3; ++j) {
    out[j].key = prefix[j];
    out[j].take_eq = remaining[j];
    out[j].total_eq = eq_total[j];
  }
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

// Ordered walk over the roles of a unit: output slot of every kept row, ordinal of every seed.
// A wave owns IDX * 64 consecutive rows, read and written 64 consecutive rows at a time
// (coalesced); positions inside the wave come from ballots with a running carry (kept rows in
// the low half of a word, seeds in the high half: a wave sees at most 1024 rows per chunk), and
// one exchange of the wave totals per chunk of kSelThreads * IDX rows orders the waves.
// Inlined on purpose: as a called function its pointers lose their address space and the
// ballots' scalar registers are spilled lane by lane, which made the walk issue-bound.
constexpr int kIdxPer = 16;

__device__ __forceinline__ bool role_is_kept(int r) {
  // prefix survivor, core, seed, recent
  return r <= CASK_ROLE_RECENT && ((0x2E >> r) & 1);
}

template <int IDX>
__device__ __forceinline__ void index_walk(const KParams& kp, int u, int64_t row0, int N,
                                           const uint8_t* __restrict__ ro, int32_t* __restrict__ slot_of,
                                           int32_t* __restrict__ out_src, int32_t* __restrict__ out_len,
                                           int32_t* __restrict__ seed_rows, int32_t* __restrict__ n_seeds,
                                           int* wsum) {
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int B = kp.B;
  int32_t* const slot_u = slot_of ? slot_of + row0 : nullptr;
  int32_t* const src_u = out_src ? out_src + (size_t)u * B : nullptr;
  int32_t* const seed_u = seed_rows + (size_t)u * B;
  int kept_before = 0, seeds_before = 0;  // of the chunks walked so far
  for (int cb = 0; cb < N; cb += kSelThreads * IDX) {
    const int i0 = cb + wv * (64 * IDX) + lane;
    int r[IDX];
#pragma unroll
    for (int e = 0; e < IDX; ++e) r[e] = (i0 + e * 64 < N) ? (int)ro[i0 + e * 64] : (int)CASK_ROLE_PREFIX_DROP;
    int pos[IDX];  // kept rows | seeds << 16 before this row inside the wave
    int run = 0;
#pragma unroll
    for (int e = 0; e < IDX; ++e) {
      const unsigned long long bk = __ballot(role_is_kept(r[e])), bs = __ballot(r[e] == CASK_ROLE_SEED);
      const int nk = __builtin_amdgcn_mbcnt_hi((unsigned)(bk >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)bk, 0));
      const int ns = __builtin_amdgcn_mbcnt_hi((unsigned)(bs >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)bs, 0));
      pos[e] = run + nk + (ns << 16);
      run += __popcll(bk) + (__popcll(bs) << 16);
      // the positions are final here: keep them from being recomputed behind the barrier out
      // of ballots that would have to be kept alive in scalar registers
      asm volatile("" : "+v"(pos[e]));
    }
    int* ws = wsum + ((cb / (kSelThreads * IDX)) & 1) * kSelWaves;  // two buffers: one barrier per chunk
    if (lane == 0) ws[wv] = run;
    __syncthreads();
    int base = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < kSelWaves; ++w) {
      const int x = ws[w];
      base += w < wv ? x : 0;
      tot += x;
    }
#pragma unroll
    for (int e = 0; e < IDX; ++e) {
      const int i = i0 + e * 64;
      const int at = base + pos[e];  // inside the chunk: at most 16 384 in either half
      const int slot = kept_before + (at & 0xFFFF), ord = seeds_before + (at >> 16);
      const bool is_seed = r[e] == CASK_ROLE_SEED;
      // a caller-supplied role array could keep more rows than the budget: never write past
      // the unit's B output slots
      const bool fits = role_is_kept(r[e]) && slot < B;
      if (i < N) {
        if (slot_u) slot_u[i] = fits ? slot : -1;
        if (fits && src_u) src_u[slot] = i;
        if (is_seed && ord < B) seed_u[ord] = i;
      }
    }
    kept_before += tot & 0xFFFF;
    seeds_before += tot >> 16;
  }
  if (tid == 0) {
    if (out_len) out_len[u] = kept_before < B ? kept_before : B;
    n_seeds[u] = seeds_before < B ? seeds_before : B;
  }
}


template <int PER>
__global__ __launch_bounds__(kSelThreads) void select_kernel(
    KParams kp, const int64_t* __restrict__ row_off, const int32_t* __restrict__ prefix_len,
    const float* __restrict__ scores, uint8_t* __restrict__ role, int32_t* __restrict__ status,
    int do_prefix, int do_decode, int do_index, int32_t* __restrict__ slot_of,
    int32_t* __restrict__ out_src, int32_t* __restrict__ out_len, int32_t* __restrict__ seed_rows,
    int32_t* __restrict__ n_seeds) {
  __shared__ int hist[2 * 3 * 256 * kHistCopies];
  __shared__ int bcast[3 * 4];
  __shared__ int wsum[2 * kSelWaves];
  const int u = blockIdx.x, tid = threadIdx.x;
  const int64_t row0 = row_off[u];
  const int N = (int)(row_off[u + 1] - row0);
  const int P = prefix_len[u];
  const UnitPlan pl = make_plan(kp, P, N);
  const float* s = scores + row0;
  uint8_t* ro = role + row0;
  if (tid == 0 && status) status[u] = pl.status;

  // which ranks have to be found: prefix rank p_keep, decode ranks C (core) and C + M (core
  // and seeds).  A rank of 0 selects nothing, a rank >= the range everything.
  const int hi = N - pl.r_eff;
  const int n = hi - P;
  const int C = pl.core, CM = pl.core + seed_range(kp, pl, n);
  const bool pre_sel = do_prefix && P > 0 && pl.p_keep > 0 && pl.p_keep < P;
  const bool dec_sel = do_decode && n > 0 && !(pl.status & CASK_ST_PREFIX_BUDGET_EXHAUSTED) && C < n;
  const bool all_seed = CM >= n;
  Query3 q;
  q.lo[0] = 0; q.hi[0] = P; q.k[0] = pre_sel ? pl.p_keep : 0;
  q.lo[1] = P; q.hi[1] = hi; q.k[1] = (dec_sel && C > 0) ? C : 0;
  q.lo[2] = P; q.hi[2] = hi; q.k[2] = (dec_sel && !all_seed && CM > C) ? CM : 0;
  constexpr int kSelChunk = kSelThreads * PER;
  Kth kth[3];
  uint32_t key[PER];
  // `key` holds rows key_lo + e * kSelThreads + tid of [key_lo, key_hi) when `have_keys`
  bool have_keys = false;
  int key_lo = 0, key_hi = 0;

  auto prefix_roles = [&]() {
    const bool keys_cover_prefix = have_keys && key_lo == 0 && key_hi >= P;
    if (pl.p_keep >= P) {
      for (int i = tid; i < P; i += kSelThreads) ro[i] = CASK_ROLE_PREFIX_KEEP;
    } else if (pl.p_keep == 0) {
      for (int i = tid; i < P; i += kSelThreads) ro[i] = CASK_ROLE_PREFIX_DROP;
    } else {
      const Kth kt = kth[0];
      if (kt.take_eq == kt.total_eq) {
        if (keys_cover_prefix) {
#pragma unroll
          for (int e = 0; e < PER; ++e) {
            const int i = key_lo + e * kSelThreads + tid;
            if (i < P) ro[i] = key[e] >= kt.key ? CASK_ROLE_PREFIX_KEEP : CASK_ROLE_PREFIX_DROP;
          }
        } else {
          for (int i = tid; i < P; i += kSelThreads)
            ro[i] = score_key(s[i]) >= kt.key ? CASK_ROLE_PREFIX_KEEP : CASK_ROLE_PREFIX_DROP;
        }
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
  };

  // The ranks are found together in one walk over [first row of an active range, last), unless
  // the prefix and the decode trace each take fewer chunks of kSelChunk rows on their own than
  // the span of both does (a 16 384-row prefix with a 2048-row trace behind it: one chunk each,
  // keys in registers across the passes, against two chunks read again in every pass): then
  // the prefix rank is found first, its roles are written, and the decode ranks follow.
  const bool pre_q = q.k[0] > 0, dec_q = q.k[1] > 0 || q.k[2] > 0;
  auto chunks = [&](int rows) { return (rows + kSelChunk - 1) / kSelChunk; };
  // (only the largest instance meets units beyond one chunk)
  const bool two_walks = PER == kSelPerDefault && pre_q && dec_q && chunks(P) + chunks(n) <= chunks(hi);
  auto find_ranks = [&](const Query3& qw) {  // the ranks of the active queries of qw -> kth, keys -> key
    int lo_all = N, hi_all = 0;
#pragma unroll
    for (int j = 0; j < 3; ++j)
      if (qw.k[j] > 0) {
        lo_all = min(lo_all, qw.lo[j]);
        hi_all = max(hi_all, qw.hi[j]);
      }
    if (hi_all > lo_all) {
      Kth found[3];
      radix_select3<PER>(s, qw, lo_all, hi_all, found, key, hist, bcast, true);
#pragma unroll
      for (int j = 0; j < 3; ++j)
        if (qw.k[j] > 0) kth[j] = found[j];
      have_keys = hi_all - lo_all <= kSelChunk;
      key_lo = lo_all;
      key_hi = hi_all;
    }
  };
  if (PER == kSelPerDefault && two_walks) {
    Query3 qa = q;
    qa.k[1] = qa.k[2] = 0;
    find_ranks(qa);
    prefix_roles();  // (the prefix rank is only asked for with do_prefix and P > 0)
    Query3 qb = q;
    qb.k[0] = 0;
    find_ranks(qb);
  } else {
    find_ranks(q);
    if (do_prefix && P > 0) prefix_roles();
  }
  const bool keys_cover_decode = have_keys && key_lo <= P && key_hi >= hi;

  auto decode_roles = [&]() {
    for (int i = hi + tid; i < N; i += kSelThreads) ro[i] = CASK_ROLE_RECENT;
    if (n <= 0) return;
    if (pl.status & CASK_ST_PREFIX_BUDGET_EXHAUSTED) {
      for (int i = P + tid; i < hi; i += kSelThreads) ro[i] = CASK_ROLE_DECODE_EVICT;
      return;
    }
    if (C >= n) {
      for (int i = P + tid; i < hi; i += kSelThreads) ro[i] = CASK_ROLE_CORE;
      return;
    }
    // thresholds of rank C (core) and rank C+M (core and seeds)
    Kth kc, km;
    kc.key = 0xFFFFFFFFu; kc.take_eq = 0; kc.total_eq = 0;
    if (C > 0) kc = kth[1];
    if (all_seed) {
      km.key = 0u; km.take_eq = 0; km.total_eq = 0;  // everything not core is a seed
    } else if (CM > C) {
      km = kth[2];
    } else {
      km = kc;
    }
    const bool ties = (C > 0 && kc.take_eq != kc.total_eq) ||
                      (!all_seed && CM > 0 && km.take_eq != km.total_eq);
    if (!ties) {
      auto mark = [&](int i, uint32_t k) {
        const bool in_c = C > 0 && k >= kc.key;
        const bool in_cm = all_seed || (CM > 0 && k >= km.key);
        ro[i] = in_c ? CASK_ROLE_CORE : (in_cm ? CASK_ROLE_SEED : CASK_ROLE_DONOR);
      };
      if (keys_cover_decode) {
#pragma unroll
        for (int e = 0; e < PER; ++e) {
          const int i = key_lo + e * kSelThreads + tid;
          if (i >= P && i < hi) mark(i, key[e]);
        }
      } else {
        for (int i = P + tid; i < hi; i += kSelThreads) mark(i, score_key(s[i]));
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
  };
  if (do_decode) decode_roles();
  if (do_index) {
    // the roles this workgroup just wrote are read back in index order: the barrier makes
    // them visible to all of its threads
    __syncthreads();
    // (as many rows per thread and chunk as the selection holds keys: a unit that fits one chunk
    // of the selection is walked by all sixteen waves, not by the first N / 1024 of them)
    index_walk<PER>(kp, u, row0, N, ro, slot_of, out_src, out_len, seed_rows, n_seeds, wsum);
  }
}

__global__ __launch_bounds__(kSelThreads) void index_roles_kernel(
    KParams kp, const int64_t* __restrict__ row_off, const uint8_t* __restrict__ role,
    int32_t* __restrict__ slot_of, int32_t* __restrict__ out_src, int32_t* __restrict__ out_len,
    int32_t* __restrict__ seed_rows, int32_t* __restrict__ n_seeds) {
  __shared__ int wsum[2 * kSelWaves];
  const int u = blockIdx.x;
  const int64_t row0 = row_off[u];
  const int N = (int)(row_off[u + 1] - row0);
  index_walk<kIdxPer>(kp, u, row0, N, role + row0, slot_of, out_src, out_len, seed_rows, n_seeds, wsum);
}

// Representative-set mass diagnostics (Section 2.6): per unit
//   rho_core = mass(C) / mass(TopK),  rho_rep = mass(R) / mass(TopK)
// with TopK the min(B, N) best rows by (score descending, index ascending), C the rows that
// protection keeps verbatim (prefix survivors, decode core, recent tail) and mass(R) the sum of
// the output rows' masses.  TopK's mass comes from one radix select (the rank-B key) and a sum
// over the keys above it plus the ties that belong; sums are carried in double.
__device__ inline double block_sum(double v, double* red) {
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  __syncthreads();  // `red` may still be read from the previous call
  if (lane == 0) red[wv] = v;
  __syncthreads();
  double t = 0.0;
  for (int w = 0; w < kSelWaves; ++w) t += red[w];
  return t;
}

__global__ __launch_bounds__(kSelThreads) void mass_diag_kernel(
    KParams kp, const int64_t* __restrict__ row_off, const float* __restrict__ scores,
    const uint8_t* __restrict__ role, const float* __restrict__ out_mass,
    const int32_t* __restrict__ out_len, float* __restrict__ rho) {
  __shared__ int hist[2 * 3 * 256 * kHistCopies];
  __shared__ int bcast[3 * 4];
  __shared__ double red[kSelWaves];
  const int u = blockIdx.x, tid = threadIdx.x;
  const int64_t row0 = row_off[u];
  const int N = (int)(row_off[u + 1] - row0);
  const float* s = scores + row0;
  const uint8_t* ro = role + row0;
  const int B = kp.B;
  double top = 0.0, core = 0.0, rep = 0.0;
  Kth kt;
  kt.key = 0u; kt.take_eq = 0; kt.total_eq = 0;
  if (N > B) {  // the key of rank B; with N <= B every row is in TopK
    Query3 q;
    q.lo[0] = 0; q.hi[0] = N; q.k[0] = B;
    q.lo[1] = q.hi[1] = q.k[1] = 0;
    q.lo[2] = q.hi[2] = q.k[2] = 0;
    Kth kth[3];
    uint32_t key[kSelPerDefault];
    radix_select3<kSelPerDefault>(s, q, 0, N, kth, key, hist, bcast, false);  // (the key itself is used below)
    kt = kth[0];
  }
  for (int i = tid; i < N; i += kSelThreads) {
    const float v = s[i];
    if (N <= B || score_key(v) > kt.key) top += (double)v;
    const int r = ro[i];
    if (r == CASK_ROLE_PREFIX_KEEP || r == CASK_ROLE_CORE || r == CASK_ROLE_RECENT) core += (double)v;
  }
  const int L = out_len[u];
  for (int t = tid; t < L; t += kSelThreads) rep += (double)out_mass[(size_t)u * B + t];
  top = block_sum(top, red);
  core = block_sum(core, red);
  rep = block_sum(rep, red);
  if (tid == 0) {
    if (N > B) {  // the ties at the rank-B key that belong to TopK
      const uint32_t bits = (kt.key & 0x80000000u) ? (kt.key & 0x7FFFFFFFu) : ~kt.key;
      top += (double)kt.take_eq * (double)__uint_as_float(bits);
    }
    rho[2 * u + 0] = top > 0.0 ? (float)(core / top) : 1.0f;
    rho[2 * u + 1] = top > 0.0 ? (float)(rep / top) : 1.0f;
  }
}

}  // namespace

namespace {
// calls f with the smallest instance whose single chunk covers the longest unit; units beyond
// the largest instance take the default one and read their keys again in every pass
template <typename F>
void with_select_instance(int max_unit_len, F&& f) {
  const int need = (max_unit_len + kSelThreads - 1) / kSelThreads;
  if (need <= 4) f(std::integral_constant<int, 4>());
  else if (need <= 6) f(std::integral_constant<int, 6>());
  else if (need <= 9) f(std::integral_constant<int, 9>());
  else if (need <= 12) f(std::integral_constant<int, 12>());
  else f(std::integral_constant<int, kSelPerDefault>());  // more keys per thread would spill
}
}  // namespace

hipError_t launch_select(const KParams& kp, const Batch& b, const float* scores, uint8_t* role,
                         int32_t* status, bool do_prefix, bool do_decode, hipStream_t st) {
  with_select_instance(b.max_unit_len, [&](auto per) {
    select_kernel<decltype(per)::value><<<dim3(b.n_units), dim3(kSelThreads), 0, st>>>(
        kp, b.row_off, b.prefix_len, scores, role, status, do_prefix ? 1 : 0, do_decode ? 1 : 0, 0,
        nullptr, nullptr, nullptr, nullptr, nullptr);
  });
  return hipGetLastError();
}

hipError_t launch_select_index(const KParams& kp, const Batch& b, const float* scores,
                               uint8_t* role, int32_t* status, int32_t* slot_of, int32_t* out_src,
                               int32_t* out_len, int32_t* seed_rows, int32_t* n_seeds,
                               hipStream_t st) {
  with_select_instance(b.max_unit_len, [&](auto per) {
    select_kernel<decltype(per)::value><<<dim3(b.n_units), dim3(kSelThreads), 0, st>>>(
        kp, b.row_off, b.prefix_len, scores, role, status, 1, 1, 1, slot_of, out_src, out_len,
        seed_rows, n_seeds);
  });
  return hipGetLastError();
}

hipError_t launch_index_roles(const KParams& kp, const Batch& b, const uint8_t* role,
                              int32_t* slot_of, int32_t* out_src, int32_t* out_len,
                              int32_t* seed_rows, int32_t* n_seeds, hipStream_t st) {
  index_roles_kernel<<<dim3(b.n_units), dim3(kSelThreads), 0, st>>>(
      kp, b.row_off, role, slot_of, out_src, out_len, seed_rows, n_seeds);
  return hipGetLastError();
}

hipError_t launch_mass_diag(const KParams& kp, const Batch& b, const float* scores,
                            const uint8_t* role, const float* out_mass, const int32_t* out_len,
                            float* rho, hipStream_t st) {
  mass_diag_kernel<<<dim3(b.n_units), dim3(kSelThreads), 0, st>>>(kp, b.row_off, scores, role,
                                                                    out_mass, out_len, rho);
  return hipGetLastError();
}

}  // namespace cask
