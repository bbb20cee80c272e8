// Cross-lane primitives of a 64-lane wavefront built on data-parallel primitives (DPP), used by the segmented
// scans of the radix passes (Alg. 1 "requests in g sorted by priority") and by the window walks of the
// greedy rounds.
#pragma once
#include <hip/hip_runtime.h>
#include <cstdint>

namespace sp {

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

}  // namespace sp
