// Consumer side: one decode step's attention over a compressed cache, with the proportional
// bias ln(count) for rows that stand for several original tokens (the paper's folds preserve
// group mass, Section 2.4; how attention uses it is left open there: this is the rule under
// which a fold of identical tokens is lossless).
#include <hip/hip_runtime.h>

#include <cstdlib>

#include "cask.h"
#include "cask_common.h"

namespace cask {

namespace {

constexpr int kAttThreads = 256;
constexpr int kAttGroups = kAttThreads / 16;  // sixteen lanes per cache row
constexpr int kAttHeads = 4;                  // query heads per pass over the cache
constexpr int kAttAhead = 4;                  // rows a group has in flight
constexpr float kNegInf = -__builtin_inff();

// One workgroup per unit.  Sixteen lanes hold one cache row (D / 16 elements each), so a
// workgroup reads sixteen rows per step, kAttAhead steps in flight; every group keeps an online
// softmax (maximum, denominator, weighted value sum, in base-2 units) for up to kAttHeads query
// heads over the rows it saw.  At the end groups 8-15 hand their state to groups 0-7 through
// LDS, which merge it into their own, and the eight merged states are added in group order:
// the same bits every run.  More query heads than kAttHeads take another pass over the cache
// (served by the L2).
template <typename T, int D>
__global__ __launch_bounds__(kAttThreads) void attend_kernel(
    KParams kp, const T* __restrict__ Q, const T* __restrict__ Kc, const T* __restrict__ Vc,
    int stride, const int32_t* __restrict__ len, const int32_t* __restrict__ count,
    int count_pitch, T* __restrict__ out) {
  constexpr int EPL = D / 16;
  constexpr int WORDS = EPL * sizeof(T) / 4;
  struct alignas(WORDS * 4 > 16 ? 16 : WORDS * 4) Raw { uint32_t w[WORDS]; };
  constexpr int kHalf = kAttGroups / 2;
  __shared__ float red_m[kHalf][kAttHeads], red_l[kHalf][kAttHeads];
  __shared__ float red_acc[kHalf][kAttHeads][D];
  const int u = blockIdx.x, tid = threadIdx.x, grp = tid >> 4, gl = tid & 15;
  int L = len[u];
  L = L < 0 ? 0 : (L > stride ? stride : L);
  const int G = kp.G;
  const T* Ku = Kc + (size_t)u * stride * D;
  const T* Vu = Vc + (size_t)u * stride * D;
  const int32_t* cu = count ? count + (size_t)u * count_pitch : nullptr;
  const float c = kp.scale_log2;  // softmax scale * log2(e)

  for (int g0 = 0; g0 < G; g0 += kAttHeads) {
    float q[kAttHeads][EPL];
#pragma unroll
    for (int h = 0; h < kAttHeads; ++h) {
      Raw qr;
#pragma unroll
      for (int w = 0; w < WORDS; ++w) qr.w[w] = 0u;
      if (g0 + h < G) qr = *reinterpret_cast<const Raw*>(Q + ((size_t)u * G + g0 + h) * D + gl * EPL);
      const T* qp = reinterpret_cast<const T*>(&qr);
#pragma unroll
      for (int e = 0; e < EPL; ++e) q[h][e] = Elem<T>::load(qp + e) * c;  // the scale rides on q
    }
    float m[kAttHeads], l[kAttHeads], acc[kAttHeads][EPL];
#pragma unroll
    for (int h = 0; h < kAttHeads; ++h) {
      m[h] = kNegInf;
      l[h] = 0.f;
#pragma unroll
      for (int e = 0; e < EPL; ++e) acc[h][e] = 0.f;
    }
    for (int t0 = grp; t0 < L; t0 += kAttGroups * kAttAhead) {
      Raw kr[kAttAhead], vr[kAttAhead];
      int cn[kAttAhead];
#pragma unroll
      for (int a = 0; a < kAttAhead; ++a) {  // clamped, not branched: all loads in flight together
        const int t = min(t0 + a * kAttGroups, L - 1);
        kr[a] = *reinterpret_cast<const Raw*>(Ku + (size_t)t * D + gl * EPL);
        vr[a] = *reinterpret_cast<const Raw*>(Vu + (size_t)t * D + gl * EPL);
        cn[a] = cu ? cu[min(t, count_pitch - 1)] : 1;
        if (t >= count_pitch) cn[a] = 1;
      }
#pragma unroll
      for (int a = 0; a < kAttAhead; ++a) {
        if (t0 + a * kAttGroups < L) {  // the same for all sixteen lanes of the group
          const T* kp_ = reinterpret_cast<const T*>(&kr[a]);
          const T* vp_ = reinterpret_cast<const T*>(&vr[a]);
          float kf[EPL], vf[EPL];
#pragma unroll
          for (int e = 0; e < EPL; ++e) {
            kf[e] = Elem<T>::load(kp_ + e);
            vf[e] = Elem<T>::load(vp_ + e);
          }
          const float bias = cn[a] > 1 ? __log2f((float)cn[a]) : 0.f;
#pragma unroll
          for (int h = 0; h < kAttHeads; ++h) {
            float dot = 0.f;
#pragma unroll
            for (int e = 0; e < EPL; ++e) dot = __builtin_fmaf(q[h][e], kf[e], dot);
#pragma unroll
            for (int o = 8; o > 0; o >>= 1) dot += __shfl_xor(dot, o, 64);
            const float x = dot + bias;
            const float mn = fmaxf(m[h], x);
            const float fa = __builtin_amdgcn_exp2f(m[h] - mn);  // exp2(-inf) = 0 on the first row
            const float fp = __builtin_amdgcn_exp2f(x - mn);
            l[h] = l[h] * fa + fp;
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc[h][e] = acc[h][e] * fa + fp * vf[e];
            m[h] = mn;
          }
        }
      }
    }
    auto put = [&](int slot) {
#pragma unroll
      for (int h = 0; h < kAttHeads; ++h) {
        if (gl == 0) {
          red_m[slot][h] = m[h];
          red_l[slot][h] = l[h];
        }
#pragma unroll
        for (int e = 0; e < EPL; ++e) red_acc[slot][h][gl * EPL + e] = acc[h][e];
      }
    };
    if (grp >= kHalf) put(grp - kHalf);
    __syncthreads();
    if (grp < kHalf) {  // merge the partner group's state into this one
#pragma unroll
      for (int h = 0; h < kAttHeads; ++h) {
        const float m2 = red_m[grp][h], l2 = red_l[grp][h];
        const float mn = fmaxf(m[h], m2);
        const float f1 = m[h] == kNegInf ? 0.f : __builtin_amdgcn_exp2f(m[h] - mn);
        const float f2 = m2 == kNegInf ? 0.f : __builtin_amdgcn_exp2f(m2 - mn);
        l[h] = l[h] * f1 + l2 * f2;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[h][e] = acc[h][e] * f1 + red_acc[grp][h][gl * EPL + e] * f2;
        m[h] = mn;
      }
    }
    __syncthreads();
    if (grp < kHalf) put(grp);
    __syncthreads();
    for (int o = tid; o < kAttHeads * D; o += kAttThreads) {
      const int h = o / D, ch = o % D;
      if (g0 + h >= G) continue;
      float top = kNegInf;
      for (int g = 0; g < kHalf; ++g) top = fmaxf(top, red_m[g][h]);
      float num = 0.f, den = 0.f;
      for (int g = 0; g < kHalf; ++g) {  // group order: the same bits every run
        const float f = red_m[g][h] == kNegInf ? 0.f : __builtin_amdgcn_exp2f(red_m[g][h] - top);
        den = __builtin_fmaf(red_l[g][h], f, den);
        num = __builtin_fmaf(red_acc[g][h][ch], f, num);
      }
      Elem<T>::store(out + ((size_t)u * G + g0 + h) * D + ch, den > 0.f ? num / den : 0.f);
    }
    __syncthreads();
  }
}


// ------------------------------------------------------------------ bf16 path: logits on MFMA

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// One workgroup per unit, one tile of 32 cache rows per wave and step, tiles dealt to the waves
// round robin.  Per tile, two MFMA products with the head dimension, then the keys, contracted:
//   logits   S[key][head]  = K_tile (32 x D) . Q^T (D x up to HP heads, zero columns beyond);
//            the two lane halves hold the two halves of the head dimension, in the same order
//            for keys and queries,
//   values   O[dim][head] += V_tile^T (D x 32) . P (32 x heads), 32 dims per product.
// The lane pair of a head column holds that head's 32 logits in registers and takes the block
// step of the online softmax there (running maximum, correction factor, weights); the weights,
// each split into two bf16 terms, are the second product's operand as they stand, because the
// order in which a lane holds its keys is a permutation the value operand simply repeats.  The
// query operand, the same for every wave and tile, waits in LDS.  The value rows
// reach their operand layout (a lane: 8 keys of one dim) through a wave-private LDS area,
// written transposed 2 bytes at a time and read back 16 bytes at a time.  The result columns of
// a head live in the same lanes as its softmax state, so nothing but the value rows crosses
// lanes inside the tile loop, and nothing there is a workgroup barrier.  The key rows of the
// next tile are requested as soon as the first product has consumed this tile's, the value rows
// as soon as they are in LDS, so a wave always has a tile of loads in flight.  At the end the
// waves' states are merged in wave order: the same bits every run.
template <int D>
constexpr int att_vt_bytes() { return D * 64 + (D / 4) * 16; }  // [dim][32 keys] bf16, 16 B pad per 4 dims
template <int D, int HP, int WAVES>
constexpr int att_lds_bytes() {
  return WAVES * att_vt_bytes<D>() + WAVES * 32 * 4 + 2 * WAVES * HP * 4 + (D / 16) * 64 * 16;
}

template <int D, int HP, int WAVES>
__global__ __launch_bounds__(WAVES * 64, 8 / WAVES) void attend_mfma_kernel(
    KParams kp, const uint16_t* __restrict__ Q, const uint16_t* __restrict__ Kc,
    const uint16_t* __restrict__ Vc, int stride, const int32_t* __restrict__ len,
    const int32_t* __restrict__ count, int count_pitch, uint16_t* __restrict__ out) {
  constexpr int KS = D / 16;     // k-steps of the logit product
  constexpr int NB = D / 32;     // 32-dim blocks of the value product
  constexpr int LPR = D / 8;     // lanes per value row
  constexpr int GPW = 64 / LPR;  // value rows one load instruction of a wave covers
  constexpr int RPG = 32 / GPW;  // value rows per lane group and tile
  constexpr int kVt = att_vt_bytes<D>();
  static_assert(HP * D * 4 <= kVt, "a wave's final state reuses its value area");
  extern __shared__ __align__(16) unsigned char att_lds[];
  const int u = blockIdx.x, tid = threadIdx.x, wv = tid >> 6, lane = tid & 63;
  const int c32 = lane & 31, hh = lane >> 5;
  const int g = lane / LPR, gl = lane % LPR;
  unsigned char* vt = att_lds + wv * kVt;
  float* bias_s = reinterpret_cast<float*>(att_lds + WAVES * kVt) + wv * 32;
  float* st_m = reinterpret_cast<float*>(att_lds + WAVES * kVt) + WAVES * 32;  // [WAVES][HP]
  float* st_l = st_m + WAVES * HP;
  u32x4* q_s = reinterpret_cast<u32x4*>(st_l + WAVES * HP);  // [KS][64]: the query operand, lane by lane
  int L = len[u];
  L = L < 0 ? 0 : (L > stride ? stride : L);
  const int n_tiles = (L + 31) >> 5;
  const int G = kp.G;
  const uint16_t* Ku = Kc + (size_t)u * stride * D;
  const uint16_t* Vu = Vc + (size_t)u * stride * D;
  const int32_t* cu = count ? count + (size_t)u * count_pitch : nullptr;
  const float c = kp.scale_log2;  // softmax scale * log2(e)
  const int last = L > 0 ? L - 1 : 0;
  // Value area: dim x at byte x * 64 + (x / 4) * 16, key slots of 2 bytes inside.
  const uint32_t vt_wr = gl * (8 * 64 + 2 * 16);
  const uint32_t vt_rd = c32 * 64 + (c32 >> 2) * 16 + hh * 16;

  for (int g0 = 0; g0 < G; g0 += HP) {
    if (wv == 0) {  // the query operand is the same for every wave and tile: it waits in LDS
      const bool head = c32 < HP && g0 + c32 < G;
      const uint16_t* qp = Q + ((size_t)u * G + (head ? g0 + c32 : 0)) * D + hh * (D / 2);
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        u32x4 qv = *reinterpret_cast<const u32x4*>(qp + ks * 8);
        if (!head) qv = u32x4{0u, 0u, 0u, 0u};
        q_s[ks * 64 + lane] = qv;
      }
    }
    asm volatile("" ::: "memory");
    __syncthreads();
    float m_run = kNegInf, l_run = 0.f;  // of head c32, over the keys this lane has seen
    f32x16 acc[NB];                      // acc[b][r] = O[dim b*32 + (r/4)*8 + hh*4 + r%4][head c32]
#pragma unroll
    for (int b = 0; b < NB; ++b) acc[b] = f32x16{0};

    u32x4 ka[KS], va[RPG];
    int cn;
    // Rows past the end are clamped to the last row (never branched over: every load is in
    // flight at once); past the last tile all lanes read that one row.
    auto load_keys = [&](int t) {
      const int r = min(t * 32 + c32, last);
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
        ka[ks] = *reinterpret_cast<const u32x4*>(Ku + (size_t)r * D + hh * (D / 2) + ks * 8);
      cn = cu ? cu[min(r, count_pitch - 1)] : 1;
      if (r >= count_pitch) cn = 1;  // rows behind the counted ones stand for themselves
    };
    auto load_values = [&](int t) {
#pragma unroll
      for (int j = 0; j < RPG; ++j) {
        const int r = min(t * 32 + j * GPW + g, last);
        va[j] = *reinterpret_cast<const u32x4*>(Vu + (size_t)r * D + gl * 8);
      }
    };
    if (L > 0) {
      load_keys(wv);
      load_values(wv);
    }
    for (int t = wv; t < n_tiles; t += WAVES) {
      {  // bias of key c32 of the tile: log2(count), or -inf past the end of the unit
        const float b = t * 32 + c32 < L ? (cn > 1 ? __log2f((float)cn) : 0.f) : kNegInf;
        if (hh == 0) bias_s[c32] = b;
      }
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      f32x16 s = {0};
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, ka[ks]),
                                                    __builtin_bit_cast(bf16x8, q_s[ks * 64 + lane]), s, 0, 0, 0);
      // s[r] = <key (r / 4) * 8 + hh * 4 + r % 4, head c32>
      float x[16], mx = kNegInf;
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const float4 b4 = *reinterpret_cast<const float4*>(&bias_s[r4 * 8 + hh * 4]);
        x[r4 * 4 + 0] = __builtin_fmaf(s[r4 * 4 + 0], c, b4.x);
        x[r4 * 4 + 1] = __builtin_fmaf(s[r4 * 4 + 1], c, b4.y);
        x[r4 * 4 + 2] = __builtin_fmaf(s[r4 * 4 + 2], c, b4.z);
        x[r4 * 4 + 3] = __builtin_fmaf(s[r4 * 4 + 3], c, b4.w);
      }
      load_keys(t + WAVES);  // the product is done with this tile's key rows
      // Value rows into the wave's LDS area, transposed: key k sits in slot
      // (k / 16) * 16 + (k / 4 % 2) * 8 + (k / 8 % 2) * 4 + k % 4, the order in which a lane's
      // logit registers enumerate the keys of its half.
#pragma unroll
      for (int j = 0; j < RPG; ++j) {
        const int k = j * GPW + g;
        const int slot = ((k >> 4) & 1) * 16 + ((k >> 2) & 1) * 8 + ((k >> 3) & 1) * 4 + (k & 3);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const uint32_t w = va[j][e >> 1];
          *reinterpret_cast<uint16_t*>(vt + vt_wr + e * 64 + (e >> 2) * 16 + slot * 2) =
              (e & 1) ? (uint16_t)(w >> 16) : (uint16_t)w;
        }
      }
      load_values(t + WAVES);  // this tile's value rows are in LDS
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, x[r]);
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      const float mn = fmaxf(m_run, mx);  // finite: key 0 of a tile in range is in range
      const float corr = __builtin_amdgcn_exp2f(m_run - mn);  // exp2(-inf) = 0 on the first tile
      // A weight enters the value product as two bf16 terms, p = hi + lo (lo the rounded
      // remainder: 16 mantissa bits in all), so that the product sees it to 2^-17.
      bf16x8 pb[2], pl[2];
      float ps = 0.f;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float pr = __builtin_amdgcn_exp2f(x[r] - mn);
        const __bf16 hi = (__bf16)pr;
        pb[r >> 3][r & 7] = hi;
        pl[r >> 3][r & 7] = (__bf16)(pr - (float)hi);
        ps += pr;
      }
      l_run = __builtin_fmaf(l_run, corr, ps);
      m_run = mn;
      if (__any(corr != 1.f)) {
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
          for (int r = 0; r < 16; ++r) acc[b][r] *= corr;
      }
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
      for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
          const u32x4 vop = *reinterpret_cast<const u32x4*>(vt + vt_rd + b * (32 * 64 + 8 * 16) + ks * 32);
          acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vop), pb[ks], acc[b], 0, 0, 0);
          acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vop), pl[ks], acc[b], 0, 0, 0);
        }
      asm volatile("" ::: "memory");  // the next tile's LDS writes stay behind these reads
    }
    const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    float* st_acc = reinterpret_cast<float*>(vt);  // [HP][D]: the wave's value area is free now
    if (c32 < HP) {
      if (hh == 0) {
        st_m[wv * HP + c32] = m_run;
        st_l[wv * HP + c32] = l_tot;
      }
#pragma unroll
      for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4)
          *reinterpret_cast<float4*>(&st_acc[c32 * D + b * 32 + r4 * 8 + hh * 4]) =
              float4{acc[b][r4 * 4], acc[b][r4 * 4 + 1], acc[b][r4 * 4 + 2], acc[b][r4 * 4 + 3]};
    }
    asm volatile("" ::: "memory");
    __syncthreads();
    for (int o = tid; o < HP * D; o += WAVES * 64) {
      const int h = o / D, ch = o % D;
      if (g0 + h >= G) continue;
      float top = kNegInf;
      for (int w = 0; w < WAVES; ++w) top = fmaxf(top, st_m[w * HP + h]);
      float num = 0.f, den = 0.f;
      for (int w = 0; w < WAVES; ++w) {  // wave order: the same bits every run
        const float mw = st_m[w * HP + h];
        const float f = mw == kNegInf ? 0.f : __builtin_amdgcn_exp2f(mw - top);
        den = __builtin_fmaf(st_l[w * HP + h], f, den);
        num = __builtin_fmaf(reinterpret_cast<const float*>(att_lds + w * kVt)[h * D + ch], f, num);
      }
      out[((size_t)u * G + g0 + h) * D + ch] = float_to_bf16_bits(den > 0.f ? num / den : 0.f);
    }
    asm volatile("" ::: "memory");
    __syncthreads();
  }
}

template <int D, int HP, int WAVES>
hipError_t launch_attend_mfma_w(const KParams& kp, int n_units, const void* Q, const void* Kc,
                                const void* Vc, int stride, const int32_t* len, const int32_t* count,
                                int count_pitch, void* out, hipStream_t st) {
  constexpr int lds = att_lds_bytes<D, HP, WAVES>();
  static LdsLimitOnce lim;  // one per instantiation
  if (lds > 48 * 1024) {
    const hipError_t e = lim.ensure(reinterpret_cast<const void*>(&attend_mfma_kernel<D, HP, WAVES>), (int)lds);
    if (e != hipSuccess) return e;
  }
  attend_mfma_kernel<D, HP, WAVES><<<dim3(n_units), dim3(WAVES * 64), lds, st>>>(
      kp, static_cast<const uint16_t*>(Q), static_cast<const uint16_t*>(Kc),
      static_cast<const uint16_t*>(Vc), stride, len, count, count_pitch, static_cast<uint16_t*>(out));
  return hipSuccess;
}

// Few units: eight waves per workgroup (more rows of a unit in flight); many: four, so that
// two workgroups share a compute unit and one's merge overlaps the other's loads.
template <int D, int HP>
hipError_t launch_attend_mfma(const KParams& kp, int n_units, const void* Q, const void* Kc, const void* Vc,
                              int stride, const int32_t* len, const int32_t* count, int count_pitch,
                              void* out, hipStream_t st) {
  if (n_units >= 512)
    return launch_attend_mfma_w<D, HP, 4>(kp, n_units, Q, Kc, Vc, stride, len, count, count_pitch, out, st);
  return launch_attend_mfma_w<D, HP, 8>(kp, n_units, Q, Kc, Vc, stride, len, count, count_pitch, out, st);
}

}  // namespace

hipError_t launch_attend(const KParams& kp, int n_units, const void* Q, const void* Kc, const void* Vc,
                         int stride, const int32_t* len, const int32_t* count, int count_pitch,
                         void* out, hipStream_t st) {
  if (n_units == 0) return hipSuccess;
  hipError_t e = hipSuccess;
#define CASK_ATT(T, D)                                                                       \
  attend_kernel<T, D><<<dim3(n_units), dim3(kAttThreads), 0, st>>>(                          \
      kp, static_cast<const T*>(Q), static_cast<const T*>(Kc), static_cast<const T*>(Vc),    \
      stride, len, count, count_pitch, static_cast<T*>(out))
#define CASK_ATT_MFMA(D, HP) \
  e = launch_attend_mfma<D, HP>(kp, n_units, Q, Kc, Vc, stride, len, count, count_pitch, out, st)
  if (kp.dtype == CASK_F32) {
    if (kp.d == 64) CASK_ATT(float, 64); else CASK_ATT(float, 128);
  } else if (kp.path_flags & CASK_PATH_ATTEND_VECTOR) {  // the vector-ALU kernel, for comparisons
    if (kp.d == 64) CASK_ATT(uint16_t, 64); else CASK_ATT(uint16_t, 128);
  } else {
    const int hp = kp.G >= 5 ? 8 : kp.G >= 3 ? 4 : kp.G;  // query heads per pass over the cache
    if (kp.d == 64) {
      if (hp == 8) CASK_ATT_MFMA(64, 8); else if (hp == 4) CASK_ATT_MFMA(64, 4);
      else if (hp == 2) CASK_ATT_MFMA(64, 2); else CASK_ATT_MFMA(64, 1);
    } else {
      if (hp == 8) CASK_ATT_MFMA(128, 8); else if (hp == 4) CASK_ATT_MFMA(128, 4);
      else if (hp == 2) CASK_ATT_MFMA(128, 2); else CASK_ATT_MFMA(128, 1);
    }
  }
#undef CASK_ATT_MFMA
#undef CASK_ATT
  if (e != hipSuccess) return e;
  return hipGetLastError();
}

}  // namespace cask
