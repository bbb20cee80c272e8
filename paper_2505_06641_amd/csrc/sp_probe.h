// Diagnostics, not on the hot path and no part of the paper's method: what the device sustains on the two
// resources the kernels are priced against.
//   k_mfma_rate: the rate at which the matrix cores run v_mfma_f32_32x32x16_f16 when nothing else competes,
//     on operands that are constant or have random bits, optionally with idle gaps between bursts.  The
//     chip runs this instruction under a power limit: the clock it sustains falls with the number of
//     operand bits that toggle and rises again when the matrix cores are given idle time, so that the
//     throughput on real data saturates well below the data-sheet peak whatever the duty cycle.
//   k_copy_rate: a plain streaming copy, for the memory bandwidth a kernel can reach.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sp {

typedef float probe_f32x16 __attribute__((ext_vector_type(16)));
typedef _Float16 probe_f16x8 __attribute__((ext_vector_type(8)));

constexpr int kProbeBlocks = 256, kProbeThreads = 512, kProbeMfmaPerIter = 8;
constexpr int kProbeIdleThreads = 256;        // with idle gaps: one wavefront per SIMD, so that the duty cycle is defined

__device__ __forceinline__ uint32_t probe_hash(uint32_t x) {
  x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16;
  return x;
}

// Two independent accumulator chains over four operand sets per lane; after every eight instructions the
// wavefront sleeps IDLE * 64 cycles.  out: one float per thread (keeps the work alive); clk: {shader
// cycles, 100 MHz ticks} of workgroup 0.
template <int IDLE>
__global__ __launch_bounds__(kProbeThreads) void k_mfma_rate(int random_bits, int iters, float* __restrict__ out,
                                                             long long* __restrict__ clk) {
  probe_f16x8 a[4], b[4];
  for (int q = 0; q < 4; ++q)
    for (int i = 0; i < 8; ++i) {
      const uint32_t h = probe_hash(threadIdx.x * 64u + q * 8u + i + blockIdx.x * 7919u);
      a[q][i] = random_bits ? (_Float16)(((int)(h & 0xffff) - 32768) * (1.0f / 8192.f)) : (_Float16)1.0f;
      b[q][i] = random_bits ? (_Float16)(((int)(h >> 16) - 32768) * (1.0f / 8192.f)) : (_Float16)0.5f;
    }
  probe_f32x16 acc0, acc1;
  for (int v = 0; v < 16; ++v) { acc0[v] = 0.f; acc1[v] = 0.f; }
  const long long c0 = __builtin_readcyclecounter();
  const long long w0 = wall_clock64();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      acc0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[q], b[q], acc0, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[(q + 1) & 3], b[q], acc1, 0, 0, 0);
    }
    if (IDLE > 0) __builtin_amdgcn_s_sleep(IDLE);
  }
  const long long c1 = __builtin_readcyclecounter();
  const long long w1 = wall_clock64();
  out[blockIdx.x * blockDim.x + threadIdx.x] = acc0[0] + acc0[5] + acc1[0] + acc1[5];
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    clk[0] = c1 - c0;
    clk[1] = w1 - w0;
  }
}

// dst[i] = src[i] over n 16-byte pieces, grid-stride.
__global__ __launch_bounds__(256) void k_copy_rate(const float4* __restrict__ src, float4* __restrict__ dst, int64_t n) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}

}  // namespace sp
