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
// read it from LDS, so staging is a straight global -> LDS DMA copy of the next
// block while the current one is being used.
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
  static constexpr int kChunks = ((kW + kTab + kBias) / 4 + 63) / 64;   // 1 KB pieces, one LDS-DMA instruction each
  static constexpr int kVec4 = kChunks * 64;
  static constexpr int kFloats = kVec4 * 4;                             // padded to whole pieces
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

// Global -> LDS copy of one packed block with the LDS-DMA load (no registers in between): every lane
// of a wavefront supplies the address of its own 16 bytes, the data lands at the (wave-uniform) LDS
// base plus 16 * lane.  Wavefront w moves pieces w, w + 8, ...
template <int D>
__device__ __forceinline__ void stage_block(const float4* __restrict__ src, float4* dst_lds, int wave, int lane) {
  using LB = LogisticBlock<D>;
  for (int ch = wave; ch < LB::kChunks; ch += kMfWaves)
    __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)(src + ch * 64 + lane),
                                     (void __attribute__((address_space(3)))*)(dst_lds + ch * 64), 16, 0, 0);
}

// One class tile: logits from `cur`, online softmax update, exponentials x table; meanwhile the next
// block streams into `nxt`.
template <int D, bool DUMP>
__device__ __forceinline__ void class_tile(const float4* cur, float4* nxt, const float4* __restrict__ next_src,
                                           const float (&xr)[D / 2], f32x16& eacc, float& m2, int ct, int C, int g,
                                           int r, int lane, int wave, bool valid, int64_t dump_row,
                                           float* __restrict__ logits_out) {
  using LB = LogisticBlock<D>;
  if (next_src != nullptr) stage_block<D>(next_src, nxt, wave, lane);
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
  if (DUMP && valid) {
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int cls = 32 * ct + 8 * (v >> 2) + 4 * g + (v & 3);
      if (cls < C) logits_out[dump_row + cls] = acc[v];
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
  __syncthreads();   // everyone is done with `cur`, and `nxt` has landed (the barrier waits for the DMA)
}

template <int D, bool DUMP>
__global__ __launch_bounds__(kMfThreads) void k_score_logistic_mfma(
    Tables tb, Window w, const float* __restrict__ x, const int32_t* __restrict__ ids, const float* __restrict__ Dl,
    const float* __restrict__ wt, uint32_t* __restrict__ sortkey, const float* __restrict__ blocks,
    const int64_t* __restrict__ block_off, float* __restrict__ logits_out) {
  using LB = LogisticBlock<D>;
  // two separate arrays (not one array split in two) so that the compiler can tell that the block
  // being read and the block being filled never overlap
  __shared__ float4 buf_a[LB::kVec4];
  __shared__ float4 buf_b[LB::kVec4];
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

  const float4* src = reinterpret_cast<const float4*>(blocks + block_off[a]);
  stage_block<D>(src, buf_a, wave, lane);

  // this lane's half of its request's features: k = g*D/2 + [0, D/2)
  float xr[D / 2];
  {
    const float* row = x + (int64_t)id * d;
    if ((d & 3) == 0) {                                  // rows are 16-byte aligned: whole float4 in or out of range
#pragma unroll
      for (int q = 0; q < D / 8; ++q) {
        const int k0 = g * (D / 2) + 4 * q;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (k0 < d) v = *reinterpret_cast<const float4*>(row + k0);
        xr[4 * q + 0] = v.x; xr[4 * q + 1] = v.y; xr[4 * q + 2] = v.z; xr[4 * q + 3] = v.w;
      }
    } else {
#pragma unroll
      for (int q = 0; q < D / 2; ++q) {
        const int k = g * (D / 2) + q;
        xr[q] = (k < d) ? row[k] : 0.f;
      }
    }
  }
  __syncthreads();

  float m2 = kNegBig;                                    // running maximum, in units of log2
  f32x16 eacc;
#pragma unroll
  for (int v = 0; v < 16; ++v) eacc[v] = 0.f;
  const int64_t dump_row = (int64_t)id * tb.Cmax;

  for (int ct = 0; ct < CT; ct += 2) {
    class_tile<D, DUMP>(buf_a, buf_b, ct + 1 < CT ? src + (size_t)(ct + 1) * LB::kVec4 : nullptr, xr, eacc, m2, ct, C,
                        g, r, lane, wave, valid, dump_row, logits_out);
    if (ct + 1 < CT)
      class_tile<D, DUMP>(buf_b, buf_a, ct + 2 < CT ? src + (size_t)(ct + 2) * LB::kVec4 : nullptr, xr, eacc, m2,
                          ct + 1, C, g, r, lane, wave, valid, dump_row, logits_out);
  }
  if (DUMP) return;

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
