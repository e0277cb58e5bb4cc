// Consumer side: one decode step's attention over a compressed cache, with the proportional
// bias ln(count) for rows that stand for several original tokens (the paper's folds preserve
// group mass, Section 2.4; how attention uses it is left open there: this is the rule under
// which a fold of identical tokens is lossless).
#include <hip/hip_runtime.h>

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
        cn[a] = cu ? cu[t] : 1;
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

}  // namespace

hipError_t launch_attend(const KParams& kp, int n_units, const void* Q, const void* Kc, const void* Vc,
                         int stride, const int32_t* len, const int32_t* count, int count_pitch,
                         void* out, hipStream_t st) {
  if (n_units == 0) return hipSuccess;
#define CASK_ATT(T, D)                                                                       \
  attend_kernel<T, D><<<dim3(n_units), dim3(kAttThreads), 0, st>>>(                          \
      kp, static_cast<const T*>(Q), static_cast<const T*>(Kc), static_cast<const T*>(Vc),    \
      stride, len, count, count_pitch, static_cast<T*>(out))
  if (kp.dtype == CASK_F32) {
    if (kp.d == 64) CASK_ATT(float, 64); else CASK_ATT(float, 128);
  } else {
    if (kp.d == 64) CASK_ATT(uint16_t, 64); else CASK_ATT(uint16_t, 128);
  }
#undef CASK_ATT
  return hipGetLastError();
}

}  // namespace cask
