// Scoring kernel for logistic heads with float32 features on the matrix cores
// (v_mfma_f32_32x32x2_f32), d <= 256, M <= 16.
//
// One workgroup = 8 wavefronts = 256 requests of one application; a wavefront
// keeps the features of its 32 requests in registers for the whole kernel and
// walks the application's classes 32 at a time.  Per class tile it computes
// the transposed logit tile  Z^T[class, request] = W^T x  (classes on the MFMA
// row axis, so that every lane owns one request column and 16 of the 32
// classes and the softmax statistics stay inside a lane), keeps a running
// maximum per request (online softmax), and feeds the exponentials straight
// back into the matrix cores against a [17 x 32] table tile -- the 16 variants'
// per-class accuracies plus a row of ones -- so that rows 0..15 accumulate
// sum_c exp(z_c) Acc[m][c] and row 16 accumulates sum_c exp(z_c).  The
// posterior is never formed or stored (Def. 4.1.2; Sec. 4.1 eq. (9));
// EA = rows 0..15 / row 16, then variance and key (Sec. 5.1.1 eq. (12)).
//
// Weights, table and bias of each (application, class tile) are packed once at
// context creation into one contiguous block in exactly the order the lanes
// read it from LDS, so staging is a straight copy (double-buffered).
#pragma once
#include "sp_common.h"
#include "sp_score_generic.h"

namespace sp {

typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kMfWaves = 8;
constexpr int kMfThreads = kMfWaves * kWave;
constexpr int kMfTile = kMfWaves * 32;      // requests per workgroup
constexpr int kClassTile = 32;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kNegBig = -1e30f;

// Packed block of one (application, class tile), in floats:
//   W    [2][D/8][32][4]  W[k = g*D/2 + 4*kk4 + j][class = 32*ct + c]      at ((g*D/8 + kk4)*32 + c)*4 + j
//   tab  [4][64][4]       row m = lane%32 of the table (Acc[m][.], ones at m = 16, else 0) for
//                         class 32*ct + 8*q + 4*(lane/32) + j                at (q*64 + lane)*4 + j
//   bias [4][2][4]        b[class 32*ct + 8*q + 4*g + j], -1e30 beyond C    at (q*2 + g)*4 + j
template <int D>
struct LogisticBlock {
  static constexpr int kW = D * 32;
  static constexpr int kTab = 16 * 64;
  static constexpr int kBias = 32;
  static constexpr int kFloats = kW + kTab + kBias;
  static constexpr int kVec4 = kFloats / 4;
  static constexpr int kStage = (kVec4 + kMfThreads - 1) / kMfThreads;
};

// Host-side packing of one application's head (called at context creation).
template <int D>
inline void pack_logistic_blocks(const float* W /*[d,C]*/, const float* b /*[C]*/, const float* acc /*[M,C]*/,
                                 int d, int C, int M, float* out /*[CT * kFloats]*/) {
  using LB = LogisticBlock<D>;
  const int CT = (C + kClassTile - 1) / kClassTile;
  for (int ct = 0; ct < CT; ++ct) {
    float* blk = out + (size_t)ct * LB::kFloats;
    for (int g = 0; g < 2; ++g)
      for (int kk4 = 0; kk4 < D / 8; ++kk4)
        for (int c = 0; c < 32; ++c)
          for (int j = 0; j < 4; ++j) {
            const int k = g * (D / 2) + 4 * kk4 + j, cls = 32 * ct + c;
            blk[((g * (D / 8) + kk4) * 32 + c) * 4 + j] = (k < d && cls < C) ? W[(size_t)k * C + cls] : 0.f;
          }
    float* tab = blk + LB::kW;
    for (int q = 0; q < 4; ++q)
      for (int lane = 0; lane < 64; ++lane)
        for (int j = 0; j < 4; ++j) {
          const int m = lane % 32, cls = 32 * ct + 8 * q + 4 * (lane / 32) + j;
          float v = 0.f;
          if (cls < C) v = (m < M) ? acc[(size_t)m * C + cls] : (m == 16 ? 1.f : 0.f);
          tab[(q * 64 + lane) * 4 + j] = v;
        }
    float* bias = tab + LB::kTab;
    for (int q = 0; q < 4; ++q)
      for (int g = 0; g < 2; ++g)
        for (int j = 0; j < 4; ++j) {
          const int cls = 32 * ct + 8 * q + 4 * g + j;
          bias[(q * 2 + g) * 4 + j] = cls < C ? b[cls] : kNegBig;
        }
  }
}

template <int D>
__global__ __launch_bounds__(kMfThreads) void k_score_logistic_mfma(
    Tables tb, Window w, const float* __restrict__ x, const int32_t* __restrict__ ids, const float* __restrict__ Dl,
    const float* __restrict__ wt, uint32_t* __restrict__ sortkey, const float* __restrict__ blocks,
    const int64_t* __restrict__ block_off, float* __restrict__ logits_out) {
  using LB = LogisticBlock<D>;
  extern __shared__ float4 lds4[];                       // two blocks
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r = lane & 31, g = lane >> 5;
  const int tile = blockIdx.x;
  if (tile >= w.tile_start[tb.A]) return;
  const int a = find_segment(w.tile_start, tb.A, tile);
  const int seg_b = w.seg[a], seg_e = w.seg[a + 1];
  const int pos = seg_b + (tile - w.tile_start[a]) * kMfTile + wave * 32 + r;
  const bool valid = pos < seg_e;
  const int id = ids[valid ? pos : seg_e - 1];           // padding lanes recompute the last request, never store
  const int d = tb.d, C = tb.n_classes[a], M = tb.n_models[a];
  const int CT = (C + kClassTile - 1) / kClassTile;

  // this lane's half of its request's features: k = g*D/2 + [0, D/2)
  float xr[D / 2];
  {
    const float* row = x + (int64_t)id * d;
    const bool vec_ok = (d & 3) == 0;
#pragma unroll
    for (int q = 0; q < D / 8; ++q) {
      const int k0 = g * (D / 2) + 4 * q;
      if (vec_ok && k0 + 3 < d) {
        const float4 v = *reinterpret_cast<const float4*>(row + k0);
        xr[4 * q + 0] = v.x; xr[4 * q + 1] = v.y; xr[4 * q + 2] = v.z; xr[4 * q + 3] = v.w;
      } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) xr[4 * q + j] = (k0 + j < d) ? row[k0 + j] : 0.f;
      }
    }
  }

  const float4* src = reinterpret_cast<const float4*>(blocks + block_off[a]);
  for (int i = tid; i < LB::kVec4; i += kMfThreads) lds4[i] = src[i];
  __syncthreads();

  float m2 = kNegBig;                                    // running maximum, in units of log2
  f32x16 eacc;
#pragma unroll
  for (int v = 0; v < 16; ++v) eacc[v] = 0.f;

  for (int ct = 0; ct < CT; ++ct) {
    const float4* cur = lds4 + (ct & 1) * LB::kVec4;
    float4* nxt = lds4 + ((ct + 1) & 1) * LB::kVec4;
    const bool more = ct + 1 < CT;
    // prefetch the next block into registers (the last iteration re-reads its own block and drops it)
    float4 stage[LB::kStage];
    {
      const float4* s2 = src + (size_t)(more ? ct + 1 : ct) * LB::kVec4;
#pragma unroll
      for (int i = 0; i < LB::kStage; ++i) stage[i] = s2[min(tid + i * kMfThreads, LB::kVec4 - 1)];
    }
    // logits of this class tile, starting from the bias
    f32x16 acc;
    {
      const float4* bp = cur + (LB::kW + LB::kTab) / 4;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const float4 bq = bp[q * 2 + g];
        acc[4 * q + 0] = bq.x; acc[4 * q + 1] = bq.y; acc[4 * q + 2] = bq.z; acc[4 * q + 3] = bq.w;
      }
    }
    const float4* wp = cur + (g * (D / 8)) * 32 + r;
#pragma unroll
    for (int kk4 = 0; kk4 < D / 8; ++kk4) {
      const float4 a4 = wp[kk4 * 32];
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a4.x, xr[4 * kk4 + 0], acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a4.y, xr[4 * kk4 + 1], acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a4.z, xr[4 * kk4 + 2], acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a4.w, xr[4 * kk4 + 3], acc, 0, 0, 0);
    }
    if (logits_out != nullptr && valid) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int cls = 32 * ct + 8 * (v >> 2) + 4 * g + (v & 3);
        if (cls < C) logits_out[(int64_t)id * tb.Cmax + cls] = acc[v];
      }
    }
    // online softmax: the request's maximum spans both lane halves
    float mt = acc[0];
#pragma unroll
    for (int v = 1; v < 16; ++v) mt = fmaxf(mt, acc[v]);
    mt = fmaxf(mt, __shfl_xor(mt, 32));
    const float m2n = fmaxf(m2, mt * kLog2e);
    const float scale = __builtin_amdgcn_exp2f(m2 - m2n);
    m2 = m2n;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      acc[v] = __builtin_amdgcn_exp2f(fmaf(acc[v], kLog2e, -m2n));
      eacc[v] *= scale;
    }
    // exponentials x table tile (accuracies and the row of ones)
    const float4* tp = cur + LB::kW / 4;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const float4 t4 = tp[q * 64 + lane];
      eacc = __builtin_amdgcn_mfma_f32_32x32x2f32(t4.x, acc[4 * q + 0], eacc, 0, 0, 0);
      eacc = __builtin_amdgcn_mfma_f32_32x32x2f32(t4.y, acc[4 * q + 1], eacc, 0, 0, 0);
      eacc = __builtin_amdgcn_mfma_f32_32x32x2f32(t4.z, acc[4 * q + 2], eacc, 0, 0, 0);
      eacc = __builtin_amdgcn_mfma_f32_32x32x2f32(t4.w, acc[4 * q + 3], eacc, 0, 0, 0);
    }
    if (more) {
#pragma unroll
      for (int i = 0; i < LB::kStage; ++i) {
        const int idx = tid + i * kMfThreads;
        if (idx < LB::kVec4) nxt[idx] = stage[i];
      }
    }
    __syncthreads();
  }
  if (logits_out != nullptr) return;

  // eacc[v] of lane (r, g) is table row 8*(v/4) + 4*g + v%4 for request r:
  // v 0..3 -> variants 4g..4g+3, v 4..7 -> variants 8+4g..8+4g+3, v = 8 at g = 0 -> the sum of exponentials
  const float ssum = __shfl(eacc[8], r);
  const float inv = 1.0f / ssum;
  float ea[8];
  float part = 0.f;
#pragma unroll
  for (int v = 0; v < 8; ++v) {
    const int m = 8 * (v >> 2) + 4 * g + (v & 3);
    ea[v] = (m < M) ? eacc[v] * inv : 0.f;
    part += ea[v];
  }
  const float mean = (part + __shfl_xor(part, 32)) / (float)M;
  float vpart = 0.f;
#pragma unroll
  for (int v = 0; v < 8; ++v) {
    const int m = 8 * (v >> 2) + 4 * g + (v & 3);
    const float dv = ea[v] - mean;
    vpart += (m < M) ? dv * dv : 0.f;
  }
  const float var = (vpart + __shfl_xor(vpart, 32)) / (float)M;
  if (!valid) return;
  float* rowo = w.ea + (int64_t)id * tb.Mmax;
#pragma unroll
  for (int v = 0; v < 8; ++v) {
    const int m = 8 * (v >> 2) + 4 * g + (v & 3);
    if (m < tb.Mmax) rowo[m] = ea[v];
  }
  if (g == 0) {
    const float Di = Dl[id], wi = wt[id];
    uint32_t err = 0;
    if (!(Di > 0.f)) err |= kErrDeadline;
    if (!(wi >= 0.f)) err |= kErrWeight;
    if (err) atomicOr(&w.st->err, err);
    const float key = wi * (1.0f + var) * expf(-Di * tb.inv_timescale);
    w.key[id] = key;
    sortkey[pos] = ~__float_as_uint(key);
  }
}

}  // namespace sp
