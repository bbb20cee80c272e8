// Cross-lane primitives of a 64-lane wavefront built on data-parallel primitives (DPP), used by the segmented
// scans of the radix passes (Alg. 1 "requests in g sorted by priority") and by the window walks of the
// greedy rounds.
#pragma once
#include <hip/hip_runtime.h>
#include <cstdint>

namespace sp {

// Orders this wavefront's LDS accesses around it (compiler fence; the hardware already runs one wavefront's
// LDS operations in issue order).
__device__ __forceinline__ void wave_sync() {
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
}

// Inclusive prefix sum across a wavefront, or (ROWS_ONLY) inside each row of 16 lanes, with data-parallel
// primitives: four shifts inside the rows, then the last lane of row 0/2 broadcast into row 1/3 and the
// last lane of row 1 into rows 2 and 3.  No LDS traffic, one vector instruction per step.  Every lane of
// the wavefront must be active.
template <bool ROWS_ONLY = false>
__device__ __forceinline__ uint32_t wave_scan_incl(uint32_t v) {
  int x = (int)v;
  x += __builtin_amdgcn_update_dpp(0, x, 0x111, 0xf, 0xf, false);   // row_shr:1
  x += __builtin_amdgcn_update_dpp(0, x, 0x112, 0xf, 0xf, false);   // row_shr:2
  x += __builtin_amdgcn_update_dpp(0, x, 0x114, 0xf, 0xf, false);   // row_shr:4
  x += __builtin_amdgcn_update_dpp(0, x, 0x118, 0xf, 0xf, false);   // row_shr:8
  if (!ROWS_ONLY) {
    x += __builtin_amdgcn_update_dpp(0, x, 0x142, 0xa, 0xf, false); // row_bcast:15 into rows 1 and 3
    x += __builtin_amdgcn_update_dpp(0, x, 0x143, 0xc, 0xf, false); // row_bcast:31 into rows 2 and 3
  }
  return (uint32_t)x;
}

// Maximum of a 64-bit value over the wavefront, returned on every lane: the same six steps as the prefix
// sum (the last lane ends up with the maximum of everything before and including it), then one read of
// lane 63.  Zero is the identity: lanes a step does not write see zero.  Every lane must be active.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ unsigned long long wave_max_step(unsigned long long v) {
  const uint32_t lo = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)v, CTRL, ROW_MASK, 0xf, false);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)(v >> 32), CTRL, ROW_MASK, 0xf, false);
  const unsigned long long o = ((unsigned long long)hi << 32) | (unsigned long long)lo;
  return o > v ? o : v;
}
__device__ __forceinline__ unsigned long long wave_max_u64(unsigned long long v) {
  v = wave_max_step<0x111, 0xf>(v);
  v = wave_max_step<0x112, 0xf>(v);
  v = wave_max_step<0x114, 0xf>(v);
  v = wave_max_step<0x118, 0xf>(v);
  v = wave_max_step<0x142, 0xa>(v);
  v = wave_max_step<0x143, 0xc>(v);
  const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)v, 63);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(v >> 32), 63);
  return ((unsigned long long)hi << 32) | (unsigned long long)lo;
}

// Sum of a float over each aligned group of 8 lanes, on every lane of the group: lane ^ 1 and lane ^ 2 inside
// the quad, then the mirrored half (whose quad already holds one value).  Every lane adds the same two
// numbers as in the butterfly over lane ^ 1, ^ 2, ^ 4, so the result has the same bits.
__device__ __forceinline__ float sum8(float v) {
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xf, 0xf, false));    // quad_perm:[1,0,3,2]
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xf, 0xf, false));    // quad_perm:[2,3,0,1]
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x141, 0xf, 0xf, false));   // row_half_mirror
  return v;
}

// The same over each row of 16 lanes: after sum8 both halves of the row are uniform, so the mirrored lane
// holds the other half's sum.
__device__ __forceinline__ float sum16(float v) {
  v = sum8(v);
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x140, 0xf, 0xf, false));   // row_mirror
  return v;
}

}  // namespace sp
