// Shared device-side declarations of the SneakPeek HIP library (gfx950).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sp {

constexpr int kMaxModels = 16;   // variants per application
constexpr int kMaxBatch = 256;   // largest batch size
constexpr int kWave = 64;

// error bits raised by kernels on bad request data
constexpr uint32_t kErrApp = 1u;
constexpr uint32_t kErrDeadline = 2u;
constexpr uint32_t kErrWeight = 4u;
constexpr uint32_t kErrSync = 8u;       // a bounded wait between resident workgroups ran out
constexpr uint32_t kErrSortSync = 16u;  // a bounded look-back between tiles of a radix pass ran out

// Immutable per-context tables (device pointers).
struct Tables {
  int32_t A, d, H, B, Mmax, Cmax, dtype;
  // policy knobs (Sec. 6.1 baselines, Alg. 1); all zero = the default policy, Bcap = B
  int32_t pol_edf;            // 1: requests of an application are served earliest deadline first
  int32_t pol_group_first;    // 1: first the application with the highest mean priority (eq. 14), then (m, b)
  int32_t pol_whole;          // 1: only the whole candidate window is a candidate batch
  int32_t pol_max_accuracy;   // 1: candidates are compared under the step penalty
  int32_t pol_unit_weight;    // 1: utilities of a batch are summed without the keys as weights
  int32_t pol_split;          // 1: an application's requests are split into subgroups by predicted class (Sec. 5.3.2)
  int32_t Bcap;               // largest batch (<= B)
  float inv_timescale;
  const int32_t* n_classes;   // [A]
  const int32_t* n_models;    // [A]
  const int32_t* penalty;     // [A]
  const void* W1;             // concatenated per-app matrices, feat_dtype
  const int64_t* W1_off;      // [A] element offsets
  const float* b1;
  const int32_t* b1_off;      // [A]
  const void* W2;
  const int64_t* W2_off;
  const float* b2;
  const int32_t* b2_off;
  const float* acc;           // per app [M_a, C_a]
  const int32_t* acc_off;     // [A]
  const float* lat;           // [A, Mmax, B]
  const float* lmin;          // [A] min_m L[a][m][1]
  // Dirichlet prior of Sec. 4.2 folded into an affine map of the expected accuracies:
  // EA' = ea_gain[a] * EA + ea_bias[a][m]   (1 and 0 without a prior)
  const float* swap;          // [A, Mmax] cost of bringing a variant in, paid unless the previous batch ran it
  const float* ea_gain;       // [A]
  const float* ea_bias;       // [A, Mmax]
};

struct Decision {             // mirrors sp_decision
  int32_t app, model, batch, round;
  double t_start, t_end;
  float score, batch_utility;
};

// Scalars of the running window, one instance in device memory.
struct State {
  double t;                   // worker clock, ms since window start
  double total_wu;            // sum w*u over served requests
  double total_u;             // sum u
  double total_viol;          // sum max(0, e - D)
  int32_t round;              // rounds committed so far
  int32_t next_order;         // next global execution order (starts at 1)
  int32_t n_sched;
  int32_t done;               // 1 once a round found nothing live
  uint32_t err;               // kErr* bits
  int32_t pad;
  unsigned long long n_evals; // utility evaluations (terms of the candidates' sums) by the rounds so far
  Decision last;              // the most recent committed batch
};

// Mutable window buffers (device pointers).
struct Window {
  int32_t n;
  int32_t* seg;               // [A+2] start of each app's range in service order; seg[A] = #valid, seg[A+1] = n
  int32_t* tile_start;        // [A+1] prefix of scoring tiles
  int4* tile_desc;            // per scoring tile: (application, first position, end of the application's range, 0)
  int32_t* unit_start;        // [A+1] prefix of sort units
  float* ea;                  // [n, Mmax]
  float* key;                 // [n]
  float4* rec_g;              // [n] (request id bits, deadline, weight, 0) at each position of the application-grouped (pre-order) array
  int32_t* id_s;              // [n] request id at each service position
  float* D_s;                 // [n]
  float* w_s;                 // [n]
  float* key_s;               // [n]
  uint8_t* alive_s;           // [n] 1 = pending
  // Groups: what the rounds iterate over.  Without splitting, group g is application g; with it, the
  // non-empty (application, subgroup) pairs in ascending order.  gcap = capacity of the per-group arrays.
  int32_t gcap;
  int32_t* sub_g;             // [n] subgroup code of the request at each grouped position: 0, or 1 + predicted class
  int32_t* grp_app;           // [gcap] application of each group
  int32_t* grp_end;           // [gcap] end of each group's range in service order
  int32_t* grp_n;             // [2] number of groups; the most groups any application has
  int32_t* head;              // [2, gcap] first position that may still be live (double-buffered by round parity)
  int32_t* model;             // [n] outputs, indexed by request id
  int32_t* round_of;          // [n]
  int32_t* order_of;          // [n]
  float* util;                // [n]
  unsigned long long* cand;   // [gcap, Mmax] best packed candidate per (group, m) of the running round
  float* cand_prio;           // [gcap, Mmax] group priority (eq. 14) of the group's window, per (group, m)
  int32_t* win_pos;           // [gcap, B] service positions of each group's candidate window
  int32_t* win_n;             // [gcap]
  Decision* log;              // [log_cap]
  int32_t log_cap;
  int32_t* last_ids;          // [B] members of the last committed batch
  State* st;
  State* st_host;             // pinned host copy of *st that the two-kernel round path keeps current (device-visible address)
};

__device__ __forceinline__ float bf16_bits_to_float(uint16_t b) {
  return __uint_as_float(((uint32_t)b) << 16);
}

template <typename T> __device__ __forceinline__ float load_as_float(const T* p, int64_t i);
template <> __device__ __forceinline__ float load_as_float<float>(const float* p, int64_t i) { return p[i]; }
template <> __device__ __forceinline__ float load_as_float<uint16_t>(const uint16_t* p, int64_t i) {
  return bf16_bits_to_float(p[i]);
}

// 1 - gamma_a(D, E) of Sec. 6.1 with the clock kept in double so that the
// comparisons E > D and E >= 2D are exact and the small remainders 2D - E and
// E - D lose nothing to cancellation.  kind: 0 step, 1 linear, 2 sigmoid.
// With x = (E-D)/D and y = 1 - x = (2D-E)/D: linear 1 - x = y; sigmoid
// 1 - x^3/(x^3+y^3) = y^3/(x^3+y^3); x + y = 1 keeps the denominator >= 1/4.
__device__ __forceinline__ float one_minus_penalty(int kind, float D, float invD, double E) {
  double Dd = (double)D;
  if (E <= Dd) return 1.0f;
  if (kind == 0) return 0.0f;
  double rem = 2.0 * Dd - E;
  if (rem <= 0.0) return 0.0f;
  float y = (float)rem * invD;
  if (kind == 1) return y;
  float x = (float)(E - Dd) * invD;
  float y3 = y * y * y, x3 = x * x * x;
  return y3 / (x3 + y3);
}

// Same quantity with the completion time given as an unevaluated float pair E = e_hi + e_lo
// (e_hi = float(E), e_lo = float(E - e_hi)), for inner loops that should stay in float32; the penalty
// kind is a template parameter so that those loops carry no branches.
// Step: l = (e_hi - D) + e_lo; a rounded sum has the sign of the exact sum, so l <= 0 (on time) is decided
// exactly as in double precision.  Linear and sigmoid: r = (2D - e_hi) - e_lo; where E and 2D are within a
// factor two of each other the first difference is exact (Sterbenz), so r carries E's full precision
// exactly where cancellation would hurt, elsewhere its relative error is one rounding.  y = r / D clamped
// to [0, 1] is 1 when the request is on time and 0 once the penalty has reached 1, and both penalties are
// continuous there, so no comparison is needed: linear 1 - gamma = y; sigmoid y^3 / (x^3 + y^3) with
// x = 1 - y (exact for y >= 1/2; below that x is near 1 and one rounding is harmless).  The denominator is
// at least 1/4, so the hardware reciprocal (1 ulp) is safe.
template <int KIND>
__device__ __forceinline__ float one_minus_penalty_f32(float D, float twoD, float invD, float e_hi, float e_lo) {
  if (KIND == 0) {
    const float l = (e_hi - D) + e_lo;
    return l <= 0.f ? 1.0f : 0.f;
  }
  const float r = (twoD - e_hi) - e_lo;
  const float y = __builtin_amdgcn_fmed3f(r * invD, 0.f, 1.f);
  if (KIND == 1) return y;
  const float x = 1.0f - y;
  const float y3 = y * y * y, x3 = x * x * x;
  return y3 * __builtin_amdgcn_rcpf(x3 + y3);
}

// dead: penalty already 1 on the earliest possible completion E0.
__device__ __forceinline__ bool is_dead(int kind, float D, double E0) {
  double Dd = (double)D;
  return kind == 0 ? (E0 > Dd) : (E0 >= 2.0 * Dd);
}

}  // namespace sp
