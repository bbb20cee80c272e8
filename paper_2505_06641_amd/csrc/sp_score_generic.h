// Scoring kernel for arbitrary head shapes (any d, H, C; M <= 16; fp32 or bf16
// inputs, fp32 arithmetic).  One wavefront owns RW requests of one application
// from the features to EA and the priority key; lanes span hidden units, then
// classes.  The posterior is never written: each lane keeps an online-softmax
// state (running max, running sum of exponentials, M running sums of
// exp * Acc[m][c]) over the classes it visits, and the 64 lane states are
// merged once per request (Def. 4.1.2 posterior; Sec. 4.1 eq. (9); Sec. 5.1.1
// eq. (12)).
#pragma once
#include "sp_common.h"

namespace sp {

constexpr int kScoreWaves = 4;
constexpr int kScoreRW = 8;                          // requests per wavefront
constexpr int kScoreTile = kScoreWaves * kScoreRW;   // requests per workgroup

// Find s with start[s] <= v < start[s+1] (start has nseg+1 entries, non-decreasing).
__device__ __forceinline__ int find_segment(const int32_t* start, int nseg, int v) {
  int lo = 0, hi = nseg;
  while (hi - lo > 1) {
    int mid = (lo + hi) >> 1;
    if (start[mid] <= v) lo = mid; else hi = mid;
  }
  return lo;
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

// EA row -> population variance -> key; also the order-preserving sort key.
// Called by one lane per request.
template <int MT>
__device__ __forceinline__ void finish_request(const Tables& tb, const Window& w, int a, int pos, int id, int M,
                                               const float (&ea_raw)[MT], const float2* dw_g, uint32_t* sortkey,
                                               int sub) {
  if (tb.pol_split) w.sub_g[pos] = sub;
  // with a prior (Sec. 4.2 eq. (10)-(11)) the posterior is (alpha + k theta) / (sum alpha + k), and
  // eq. (9) on it is an affine map of eq. (9) on theta; gain 1 and bias 0 leave the value untouched
  float ea[MT];
  const float gain = tb.ea_gain[a];
#pragma unroll
  for (int m = 0; m < MT; ++m) ea[m] = (m < M) ? fmaf(gain, ea_raw[m], tb.ea_bias[a * tb.Mmax + m]) : 0.f;
  float mean = 0.f;
#pragma unroll
  for (int m = 0; m < MT; ++m) mean += (m < M) ? ea[m] : 0.f;
  mean /= (float)M;
  float var = 0.f;
#pragma unroll
  for (int m = 0; m < MT; ++m) {
    float dv = ea[m] - mean;
    var += (m < M) ? dv * dv : 0.f;
  }
  var /= (float)M;
  const float2 dw = dw_g[pos];            // (deadline, weight), brought to the grouped position by the grouping pass
  float Di = dw.x, wi = dw.y;
  uint32_t err = 0;
  if (!(Di > 0.f)) err |= kErrDeadline;
  if (!(wi >= 0.f)) err |= kErrWeight;
  if (err) atomicOr(&w.st->err, err);
  float key = fabsf(wi * (1.0f + var) * expf(-Di * tb.inv_timescale));   // a weight of -0 must not give the key -0: its bits would sort first
  w.key[id] = key;
  sortkey[pos] = tb.pol_edf ? __float_as_uint(Di) : ~__float_as_uint(key);   // ascending deadline, or descending key
  w.rec_g[pos] = make_float4(__int_as_float(id), Di, wi, 0.f);   // what the ordering needs of this request, in one piece
  float* row = w.ea + (int64_t)id * tb.Mmax;
  for (int m = 0; m < tb.Mmax; ++m) {
    float v = 0.f;
#pragma unroll
    for (int q = 0; q < MT; ++q) v = (q == m && q < M) ? ea[q] : v;
    row[m] = v;
  }
}

template <typename T, int MT>
__global__ __launch_bounds__(kScoreWaves* kWave) void k_score_generic(
    Tables tb, Window w, const T* __restrict__ x, const int32_t* __restrict__ ids, const float2* __restrict__ dw_g,
    uint32_t* __restrict__ sortkey, float* __restrict__ logits_out) {
  constexpr int RW = kScoreRW;
  extern __shared__ float lds[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int tile = blockIdx.x;
  if (tile >= w.tile_start[tb.A]) return;
  const int4 desc = w.tile_desc[tile];
  const int a = desc.x, seg_e = desc.z;
  const int p0 = desc.y + wave * RW;                                           // first service position of this wave
  const int nr = min(RW, seg_e - p0);                                          // may be <= 0
  const int d = tb.d, H = tb.H, C = tb.n_classes[a], M = tb.n_models[a];
  float* xs = lds + (size_t)wave * RW * (d + H);
  float* hs = xs + (size_t)RW * d;

  // stage this wave's feature rows as float
  for (int r = 0; r < RW; ++r) {
    if (r < nr) {
      const T* row = x + (int64_t)ids[p0 + r] * d;
      for (int k = lane; k < d; k += 64) xs[r * d + k] = load_as_float<T>(row, k);
    } else {
      for (int k = lane; k < d; k += 64) xs[r * d + k] = 0.f;
    }
  }
  __syncthreads();

  const float* in = xs;
  int K = d;
  const T* Wout = (const T*)tb.W1 + tb.W1_off[a];
  const float* bout = tb.b1 + tb.b1_off[a];
  if (H > 0) {
    const T* W1 = Wout;
    const float* b1 = bout;
    for (int j0 = 0; j0 < H; j0 += 64) {
      const int j = j0 + lane;
      const bool ok = j < H;
      float acc[RW];
      const float bj = ok ? b1[j] : 0.f;
#pragma unroll
      for (int r = 0; r < RW; ++r) acc[r] = bj;
      for (int k = 0; k < d; ++k) {
        const float wv = ok ? load_as_float<T>(W1, (int64_t)k * H + j) : 0.f;
#pragma unroll
        for (int r = 0; r < RW; ++r) acc[r] = fmaf(xs[r * d + k], wv, acc[r]);
      }
      if (ok) {
#pragma unroll
        for (int r = 0; r < RW; ++r) hs[r * H + j] = fmaxf(acc[r], 0.f);
      }
    }
    __syncthreads();
    in = hs;
    K = H;
    Wout = (const T*)tb.W2 + tb.W2_off[a];
    bout = tb.b2 + tb.b2_off[a];
  }

  // classes: lanes stride over c; online softmax state per (lane, request)
  constexpr float kNegBig = -1e30f;
  float mx[RW], sm[RW], ea[RW][MT];
  int bestc[RW];                             // class of this lane's largest logit (subgroup label, Sec. 5.3.2)
#pragma unroll
  for (int r = 0; r < RW; ++r) {
    bestc[r] = 0x7fffffff;
    mx[r] = kNegBig;
    sm[r] = 0.f;
#pragma unroll
    for (int m = 0; m < MT; ++m) ea[r][m] = 0.f;
  }
  const float* acc_a = tb.acc + tb.acc_off[a];
  for (int c0 = 0; c0 < C; c0 += 64) {
    const int c = c0 + lane;
    const bool ok = c < C;
    float z[RW];
    const float bc = ok ? bout[c] : 0.f;
#pragma unroll
    for (int r = 0; r < RW; ++r) z[r] = bc;
    for (int k = 0; k < K; ++k) {
      const float wv = ok ? load_as_float<T>(Wout, (int64_t)k * C + c) : 0.f;
#pragma unroll
      for (int r = 0; r < RW; ++r) z[r] = fmaf(in[r * K + k], wv, z[r]);
    }
    if (ok) {
      float ac[MT];
#pragma unroll
      for (int m = 0; m < MT; ++m) ac[m] = (m < M) ? acc_a[m * C + c] : 0.f;
#pragma unroll
      for (int r = 0; r < RW; ++r) {
        if (logits_out != nullptr && r < nr) logits_out[(int64_t)ids[p0 + r] * tb.Cmax + c] = z[r];
        bestc[r] = z[r] > mx[r] ? c : bestc[r];
        const float mn = fmaxf(mx[r], z[r]);
        const float sc = expf(mx[r] - mn);
        const float p = expf(z[r] - mn);
        sm[r] = sm[r] * sc + p;
#pragma unroll
        for (int m = 0; m < MT; ++m) ea[r][m] = fmaf(p, ac[m], ea[r][m] * sc);
        mx[r] = mn;
      }
    }
  }

  // merge the 64 lane states of each request
#pragma unroll
  for (int r = 0; r < RW; ++r) {
    const float mt = wave_max(mx[r]);
    const float f = expf(mx[r] - mt);
    const float st = wave_sum(sm[r] * f);
    float row[MT];
#pragma unroll
    for (int m = 0; m < MT; ++m) row[m] = wave_sum(ea[r][m] * f) / st;
    // the largest posterior is exp(0) / st; its class is the smallest class among the lanes that hold the maximum
    int cls = mx[r] == mt ? bestc[r] : 0x7fffffff;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) cls = min(cls, __shfl_xor(cls, o));
    const int sub = (1.0f / st > 0.5f) ? 1 + cls : 0;
    if (lane == 0 && r < nr && logits_out == nullptr)
      finish_request<MT>(tb, w, a, p0 + r, ids[p0 + r], M, row, dw_g, sortkey, sub);
  }
}

}  // namespace sp
