// Measurement aids (not part of the method): plain loops that pin what the device delivers, so
// that a report can print measured ceilings next to the published ones.
//   issue probe  register-only loops of the scoring sweeps' instruction mix: one
//                v_mfma_f32_32x32x16_bf16 per unit, alone or with the vector epilogue of two logits
//                (fma, exp2, add each), or the vector part alone; every workgroup reports its
//                shader-clock cycles and the 100 MHz wall ticks it took;
//   copy probe   a streaming copy of known size (also the reference that scales the profiler's
//                HBM byte counters).
#include "cask_common.h"

namespace cask {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// KIND 0: MFMA alone; 1: MFMA + vector epilogue of two logits; 2: vector epilogue alone;
// 3: as 1, with the MFMA's first operand read from LDS at the sweeps' rate (one 16-byte read per
// lane for every two MFMA, conflict-free), to see what the operand traffic costs.
// One "unit" = one MFMA (32 matrix-pipe cycles) and/or six vector instructions.
template <int KIND>
__global__ __launch_bounds__(1024) void issue_probe_kernel(const uint4* __restrict__ operands, int iters,
                                                           uint64_t* __restrict__ cycles,
                                                           float* __restrict__ sink) {
  const int tid = threadIdx.x;
  // random bf16 operands (constant operands toggle few bits and let the chip clock higher than
  // real data does)
  const uint4 ra = operands[tid & 1023], rb = operands[1024 + (tid & 1023)];
  const bf16x8 a = __builtin_bit_cast(bf16x8, ra), b = __builtin_bit_cast(bf16x8, rb);
  float x[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) x[i] = 0.01f * (float)((ra.x >> i) & 255);
  const float c = 0.127f, nm = -3.0f;
  f32x16 acc = {0};
  float s0 = 0.f, s1 = 0.f;
  __shared__ uint4 tile[KIND == 3 ? 4096 : 1];  // 64 KB: a ring's worth of operand data
  if (KIND == 3) {
    for (int i = tid; i < 4096; i += blockDim.x) tile[i] = operands[i & 2047];
  }
  bf16x8 a_lds[4] = {a, a, a, a};
  __syncthreads();
  const uint64_t t0 = __builtin_amdgcn_s_memtime(), r0 = __builtin_amdgcn_s_memrealtime();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      if (KIND == 3) {
        // operands for four units ahead, read two units apart
        if ((i & 1) == 0) a_lds[(i >> 1) & 3] = __builtin_bit_cast(bf16x8, tile[(((it * 4 + (i >> 1)) * 64) + (tid & 63) + (tid >> 6) * 512) & 4095]);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_lds[((i >> 1) + 2) & 3], b, acc, 0, 0, 0);
      } else if (KIND != 2) {
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc, 0, 0, 0);
      }
      if (KIND != 0) {
        // the sweeps' epilogue for two logits, written as the six instructions themselves so
        // that the optimiser cannot hoist or merge any of them: fma, fma, exp2, exp2, add, add
        float t, u;
        if (KIND == 4) {
          // the same six instructions in dependent order with one running sum
          asm volatile("v_fma_f32 %0, %1, %2, %3" : "=v"(t) : "v"(x[2 * i]), "v"(c), "v"(nm));
          asm volatile("v_exp_f32 %0, %0" : "+v"(t));
          asm volatile("v_fma_f32 %0, %1, %2, %3" : "=v"(u) : "v"(x[2 * i + 1]), "v"(c), "v"(nm));
          asm volatile("v_exp_f32 %0, %0" : "+v"(u));
          asm volatile("v_add_f32 %0, %0, %1" : "+v"(s0) : "v"(t));
          asm volatile("v_add_f32 %0, %0, %1" : "+v"(s0) : "v"(u));
          __builtin_amdgcn_sched_barrier(0);
          continue;
        }
        asm volatile("v_fma_f32 %0, %1, %2, %3" : "=v"(t) : "v"(x[2 * i]), "v"(c), "v"(nm));
        asm volatile("v_fma_f32 %0, %1, %2, %3" : "=v"(u) : "v"(x[2 * i + 1]), "v"(c), "v"(nm));
        asm volatile("v_exp_f32 %0, %0" : "+v"(t));
        asm volatile("v_exp_f32 %0, %0" : "+v"(u));
        asm volatile("v_add_f32 %0, %0, %1" : "+v"(s0) : "v"(t));
        asm volatile("v_add_f32 %0, %0, %1" : "+v"(s1) : "v"(u));
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  const uint64_t t1 = __builtin_amdgcn_s_memtime(), r1 = __builtin_amdgcn_s_memrealtime();
  float s = s0 + s1;
#pragma unroll
  for (int i = 0; i < 16; ++i) s += acc[i];
  sink[(size_t)blockIdx.x * blockDim.x + tid] = s;
  if (tid == 0) {
    cycles[2 * blockIdx.x] = t1 - t0;
    cycles[2 * blockIdx.x + 1] = r1 - r0;
  }
}

// 16 bytes per thread per step, grid-stride, four loads in flight per thread.
__global__ __launch_bounds__(256) void copy_probe_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst,
                                                         size_t n16) {
  const size_t stride = (size_t)gridDim.x * 256;
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  for (; i + 3 * stride < n16; i += 4 * stride) {
    const uint4 v0 = src[i], v1 = src[i + stride], v2 = src[i + 2 * stride], v3 = src[i + 3 * stride];
    dst[i] = v0;
    dst[i + stride] = v1;
    dst[i + 2 * stride] = v2;
    dst[i + 3 * stride] = v3;
  }
  for (; i < n16; i += stride) dst[i] = src[i];
}

// Read-only stream: every thread keeps eight 16-byte loads in flight and folds what it reads
// into one word (written once at the end so that the loads cannot be dropped).
__global__ __launch_bounds__(256) void read_probe_kernel(const u32x4* __restrict__ src, size_t n16,
                                                         uint32_t* __restrict__ sink) {
  const size_t stride = (size_t)gridDim.x * 256;
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  uint32_t acc = 0;
  for (; i + 7 * stride < n16; i += 8 * stride) {
    u32x4 v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = __builtin_nontemporal_load(src + i + j * stride);
#pragma unroll
    for (int j = 0; j < 8; ++j) acc ^= v[j].x ^ v[j].y ^ v[j].z ^ v[j].w;
  }
  for (; i < n16; i += stride) {
    const u32x4 v = src[i];
    acc ^= v.x ^ v.y ^ v.z ^ v.w;
  }
  sink[(size_t)blockIdx.x * 256 + threadIdx.x] = acc;
}

}  // namespace
}  // namespace cask

using namespace cask;

extern "C" {

int cask_probe_issue(int kind, int waves_per_simd, int blocks, int iters, const void* operands,
                     uint64_t* cycles, float* sink, void* hip_stream) {
  if (kind < 0 || kind > 4 || waves_per_simd < 1 || waves_per_simd > 4 || blocks < 1 || blocks > 65536 ||
      iters < 1 || iters > (1 << 24) || !operands || !cycles || !sink)
    return CASK_EINVAL;
  if ((reinterpret_cast<uintptr_t>(operands) & 15u) != 0) return CASK_EINVAL;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const dim3 grid(blocks), block(256 * waves_per_simd);
  const uint4* ops = static_cast<const uint4*>(operands);
  if (kind == 0) issue_probe_kernel<0><<<grid, block, 0, st>>>(ops, iters, cycles, sink);
  else if (kind == 1) issue_probe_kernel<1><<<grid, block, 0, st>>>(ops, iters, cycles, sink);
  else if (kind == 2) issue_probe_kernel<2><<<grid, block, 0, st>>>(ops, iters, cycles, sink);
  else if (kind == 3) issue_probe_kernel<3><<<grid, block, 0, st>>>(ops, iters, cycles, sink);
  else issue_probe_kernel<4><<<grid, block, 0, st>>>(ops, iters, cycles, sink);
  return hipGetLastError() == hipSuccess ? CASK_OK : CASK_EDEVICE;
}

int cask_probe_copy(const void* src, void* dst, size_t bytes, void* hip_stream) {
  if (!src || !dst || bytes == 0 || (bytes & 15u) != 0) return CASK_EINVAL;
  if (((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 15u) != 0) return CASK_EINVAL;
  copy_probe_kernel<<<dim3(256 * 16), dim3(256), 0, static_cast<hipStream_t>(hip_stream)>>>(
      static_cast<const uint4*>(src), static_cast<uint4*>(dst), bytes / 16);
  return hipGetLastError() == hipSuccess ? CASK_OK : CASK_EDEVICE;
}

int cask_probe_read(const void* src, size_t bytes, uint32_t* sink, int blocks, void* hip_stream) {
  if (!src || !sink || bytes == 0 || (bytes & 15u) != 0 || blocks < 1 || blocks > 65536) return CASK_EINVAL;
  if ((reinterpret_cast<uintptr_t>(src) & 15u) != 0) return CASK_EINVAL;
  read_probe_kernel<<<dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(hip_stream)>>>(
      static_cast<const u32x4*>(src), bytes / 16, sink);
  return hipGetLastError() == hipSuccess ? CASK_OK : CASK_EDEVICE;
}

}  // extern "C"
