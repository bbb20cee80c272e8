// Diagnostic: the rate at which the matrix cores run v_mfma_f32_32x32x16_f16 when nothing else competes,
// on operands that are constant or have random bits.  The clock the device sustains depends on how many
// operand bits toggle, so the second figure, not the data-sheet peak, is the ceiling a kernel fed with real
// data can reach; the scoring kernel (Sec. 4.1 eq. (9) fused with the posterior of Def. 4.1.2) is compared
// against it.  Not on the hot path.
#pragma once
#include "sp_common.h"
#include "sp_score_split.h"   // the vector types of the matrix-core operands

namespace sp {

constexpr int kProbeBlocks = 256, kProbeThreads = 512, kProbeMfmaPerIter = 8;

__device__ __forceinline__ uint32_t probe_hash(uint32_t x) {
  x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16;
  return x;
}

// Two independent accumulator chains over four operand sets per lane.  out: one float per thread (keeps
// the work alive); clk: {shader cycles, 100 MHz ticks} of workgroup 0.
__global__ __launch_bounds__(kProbeThreads) void k_mfma_rate(int random_bits, int iters, float* __restrict__ out,
                                                             long long* __restrict__ clk) {
  f16x8 a[4], b[4];
  for (int q = 0; q < 4; ++q)
    for (int i = 0; i < 8; ++i) {
      const uint32_t h = probe_hash(threadIdx.x * 64u + q * 8u + i + blockIdx.x * 7919u);
      a[q][i] = random_bits ? (_Float16)(((int)(h & 0xffff) - 32768) * (1.0f / 8192.f)) : (_Float16)1.0f;
      b[q][i] = random_bits ? (_Float16)(((int)(h >> 16) - 32768) * (1.0f / 8192.f)) : (_Float16)0.5f;
    }
  f32x16 acc0, acc1;
  for (int v = 0; v < 16; ++v) { acc0[v] = 0.f; acc1[v] = 0.f; }
  const long long c0 = __builtin_readcyclecounter();
  const long long w0 = wall_clock64();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      acc0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[q], b[q], acc0, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[(q + 1) & 3], b[q], acc1, 0, 0, 0);
    }
  }
  const long long c1 = __builtin_readcyclecounter();
  const long long w1 = wall_clock64();
  out[blockIdx.x * kProbeThreads + threadIdx.x] = acc0[0] + acc0[5] + acc1[0] + acc1[5];
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    clk[0] = c1 - c0;
    clk[1] = w1 - w0;
  }
}

}  // namespace sp
