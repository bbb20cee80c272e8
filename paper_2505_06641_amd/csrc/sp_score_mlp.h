// Scoring kernel for one-hidden-layer ReLU heads with bfloat16 features and weights (H <= 256, M <= 16).
//
// Layer 1, h = relu(x W1 + b1), runs on v_mfma_f32_32x32x16_bf16 (bf16 x bf16 products are exact,
// float32 accumulation): a wavefront owns 32 requests and keeps the whole transposed hidden tile
// H^T[hidden, request] in eight float32 accumulators (128 VGPRs) while it streams its requests' features
// 64 input channels at a time; the matching W1 slices (32 KB each, packed at context creation in the
// order the lanes read them) go through two LDS buffers shared by the workgroup's eight wavefronts.
// The hidden tile never leaves the registers: after bias and ReLU each request's row is scaled by a
// power of two, split into half-precision hi + lo (22 bits) and used directly as the input operand of
// the class tiles (layer 2 + online softmax + accuracy-table contraction) shared with the logistic
// kernel, whose weight blocks are packed with the row order an MFMA output tile has (Def. 4.1.2;
// Sec. 4.1 eq. (9); Sec. 5.1.1 eq. (12)).
#pragma once
#include "sp_common.h"
#include "sp_score_split.h"

namespace sp {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int kMlpH = 256;                       // padded hidden width (zero weights beyond H)
constexpr int kL1Chunk = 64;                     // input channels per W1 slice
constexpr int kL1Units = (kMlpH / 32) * (kL1Chunk / 16) * 64;   // 16-byte units per slice (2048 = 32 KB)
constexpr int kL1PerThread = kL1Units / kMfThreads;             // 4
constexpr int kL1Pre = 2;                                       // weight fragments in flight from LDS per wavefront

// Bytes of one application's packed layer 1: its slices, then the bias padded with zeros to kMlpH floats.
inline size_t mlp_layer1_bytes(int d) { return (size_t)((d + kL1Chunk - 1) / kL1Chunk) * kL1Units * 16 + kMlpH * sizeof(float); }

// W1 slice kc of an application, 16-byte units:
//   unit ((hb*4 + s)*64 + lane), element e: W1[k = 64 kc + 16 s + 8 (lane/32) + e][hidden = 32 hb + lane%32]
inline void pack_mlp_layer1(const uint16_t* W1 /*[d,H] bf16 bits*/, int d, int H, uint16_t* out /*[nkc * kL1Units * 8]*/) {
  const int nkc = (d + kL1Chunk - 1) / kL1Chunk;
  for (int kc = 0; kc < nkc; ++kc)
    for (int hb = 0; hb < kMlpH / 32; ++hb)
      for (int s = 0; s < kL1Chunk / 16; ++s)
        for (int lane = 0; lane < 64; ++lane)
          for (int e = 0; e < 8; ++e) {
            const int k = kL1Chunk * kc + 16 * s + 8 * (lane / 32) + e, hid = 32 * hb + lane % 32;
            out[(((size_t)kc * kL1Units) + ((hb * 4 + s) * 64 + lane)) * 8 + e] =
                (k < d && hid < H) ? W1[(size_t)k * H + hid] : (uint16_t)0;
          }
}

__device__ __forceinline__ bf16x8 as_bf16x8(const f32x4& v) { return __builtin_bit_cast(bf16x8, v); }

// DUMP: the launch only writes the logits (logits_out) and ends before the epilogue; dw_g and sortkey are
// then null and must not be touched.
template <bool DUMP, bool SPLIT>
__global__ __launch_bounds__(kMfThreads) void k_score_mlp_bf16(
    Tables tb, Window w, const uint16_t* __restrict__ x, const int32_t* __restrict__ ids, const float2* __restrict__ dw_g,
    uint32_t* __restrict__ sortkey, const unsigned char* __restrict__ w1p,
    const int64_t* __restrict__ w1_off /*[A] bytes*/, const unsigned char* __restrict__ blocks,
    const int64_t* __restrict__ block_off /*[A] bytes*/, const float* __restrict__ w_unscale /*[A]*/,
    float* __restrict__ logits_out) {
  constexpr int D = kMlpH;
  using SB = SplitBlock<D>;
  __shared__ float4 buf_a[SB::kUnits];
  __shared__ float4 buf_b[SB::kUnits];
  __shared__ float4 buf_c[SB::kUnits];
  static_assert(kL1Units <= SB::kUnits, "a W1 slice must fit in one block buffer");
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r = lane & 31, g = lane >> 5;
  const int tile = xcd_tile(blockIdx.x, w.tile_start[tb.A]);
  if (tile < 0) return;
  const int4 desc = w.tile_desc[tile];
  const int a = desc.x, seg_e = desc.z;
  const int pos = desc.y + wave * 32 + r;
  const bool valid = pos < seg_e;
  const int id = ids[valid ? pos : seg_e - 1];           // padding lanes recompute the last request, never store
  const int d = tb.d, C = tb.n_classes[a], M = tb.n_models[a];
  const int CT = (C + kClassTile - 1) / kClassTile;
  const int nkc = (d + kL1Chunk - 1) / kL1Chunk;

  // the first class-tile block can travel while layer 1 runs
  const float4* src = reinterpret_cast<const float4*>(blocks + block_off[a]);
  stage_block_dma<D>(src, buf_a, wave, lane);

  // ---- layer 1 ----
  const f32x4* w1 = reinterpret_cast<const f32x4*>(w1p + w1_off[a]);
  const uint16_t* row = x + (int64_t)id * d + 8 * g;     // this lane half's 8 channels of every 16
  f32x16 hacc[kMlpH / 32];
#pragma unroll
  for (int hb = 0; hb < kMlpH / 32; ++hb)
#pragma unroll
    for (int v = 0; v < 16; ++v) hacc[hb][v] = 0.f;

  // Features travel two slices ahead of the matrix cores in a ring of three register sets (a slice's rows
  // come from HBM: one slice of lead leaves the loop waiting for them), the W1 slice one ahead (L2).  All of
  // these are ordinary loads, so the compiler counts what is in flight; a set is written in one step and read
  // two steps later under its own name (the loop is unrolled by three), so nothing in flight is ever copied.
  f32x4 x0[kL1Chunk / 16], x1[kL1Chunk / 16], x2[kL1Chunk / 16];
  // d is a multiple of 8, so a lane's 16-byte piece lies wholly inside or outside a row; pieces outside are
  // read from the start of the packed weights instead (one line that every workgroup has in cache anyway)
  // and zeroed by the slice that uses them (only a last, partial slice has any)
  auto load_x = [&](f32x4 (&xs)[kL1Chunk / 16], int kc) {
#pragma unroll
    for (int s = 0; s < kL1Chunk / 16; ++s) {
      const int k0 = kL1Chunk * kc + 16 * s;
      xs[s] = *((kc < nkc && k0 + 8 * g < d) ? reinterpret_cast<const f32x4*>(row + k0) : w1);
    }
  };
  {
    f32x4* dst = reinterpret_cast<f32x4*>(buf_b);
#pragma unroll
    for (int i = 0; i < kL1PerThread; ++i) dst[tid + i * kMfThreads] = w1[tid + i * kMfThreads];
    load_x(x0, 0);
    load_x(x1, 1);
  }
  __syncthreads();
  // one slice: W1 slice kc + 1 and the features of slice kc + 2 start, the 32 MFMAs of slice kc run on xs
  auto slice = [&](int kc, f32x4 (&xs)[kL1Chunk / 16], f32x4 (&xfar)[kL1Chunk / 16]) {
    const f32x4* cur = reinterpret_cast<const f32x4*>((kc & 1) ? buf_c : buf_b);
    f32x4* nxt = reinterpret_cast<f32x4*>((kc & 1) ? buf_b : buf_c);
    // every step issues the same loads whatever is left to do (the last one reads its own slice again, into
    // the idle buffer, and one cached line in place of features that do not exist), so that the number of loads in
    // flight behind any register is the same on every path and the waits the compiler inserts are exact
    f32x4 wst[kL1PerThread];
    {
      const f32x4* nsrc = w1 + (size_t)(kc + 1 < nkc ? kc + 1 : nkc - 1) * kL1Units;
#pragma unroll
      for (int i = 0; i < kL1PerThread; ++i) wst[i] = nsrc[tid + i * kMfThreads];
    }
    load_x(xfar, kc + 2);
    __builtin_amdgcn_sched_barrier(0);
    // the slice's 32 weight fragments in the order they are used, each read kL1Pre fragments ahead of the
    // MFMA that takes it, so that LDS latency and matrix cores overlap inside a wavefront too
    if (kc < nkc) {
      if (kL1Chunk * (kc + 1) > d) {
#pragma unroll
        for (int s = 0; s < kL1Chunk / 16; ++s)
          if (kL1Chunk * kc + 16 * s + 8 * g >= d) xs[s] = f32x4{0.f, 0.f, 0.f, 0.f};
      }
      constexpr int kSteps = (kMlpH / 32) * (kL1Chunk / 16);
      f32x4 af[kL1Pre];
#pragma unroll
      for (int i = 0; i < kL1Pre; ++i) af[i] = cur[i * 64 + lane];
#pragma unroll
      for (int i = 0; i < kSteps; ++i) {
        const f32x4 a = af[i % kL1Pre];
        if (i + kL1Pre < kSteps) af[i % kL1Pre] = cur[(i + kL1Pre) * 64 + lane];
        __builtin_amdgcn_sched_barrier(0);
        hacc[i / 4] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(a), as_bf16x8(xs[i % 4]), hacc[i / 4], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
#pragma unroll
    for (int i = 0; i < kL1PerThread; ++i) nxt[tid + i * kMfThreads] = wst[i];
    __syncthreads();
  };
  // whole trips of three steps (a step past the last slice only moves data nobody reads): the loop has one
  // way in and one way round, so the counts of loads in flight are the same wherever a step is entered from
  for (int kc = 0; kc < nkc; kc += 3) {
    slice(kc, x0, x2);
    slice(kc + 1, x1, x0);
    slice(kc + 2, x2, x1);
  }

  // ---- bias, ReLU, per-request scale, split into half-precision hi + lo ----
  // hacc[hb][v] of lane (r, g) is hidden unit 32 hb + 8 (v/4) + 4 g + v%4 of request r
  const float4* b1p = reinterpret_cast<const float4*>(w1p + w1_off[a] + (size_t)nkc * kL1Units * 16);   // padded to kMlpH
  float amax = 0.f;
#pragma unroll
  for (int hb = 0; hb < kMlpH / 32; ++hb) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const float4 bq = b1p[8 * hb + 2 * q + g];
      hacc[hb][4 * q + 0] = fmaxf(hacc[hb][4 * q + 0] + bq.x, 0.f);
      hacc[hb][4 * q + 1] = fmaxf(hacc[hb][4 * q + 1] + bq.y, 0.f);
      hacc[hb][4 * q + 2] = fmaxf(hacc[hb][4 * q + 2] + bq.z, 0.f);
      hacc[hb][4 * q + 3] = fmaxf(hacc[hb][4 * q + 3] + bq.w, 0.f);
      amax = fmaxf(amax, fmaxf(fmaxf(hacc[hb][4 * q + 0], hacc[hb][4 * q + 1]),
                               fmaxf(hacc[hb][4 * q + 2], hacc[hb][4 * q + 3])));
    }
  }
  amax = fmaxf(amax, other_half(amax, g));
  int ex = 0;
  if (amax >= 1e-30f && amax <= 3e38f) ex = kSplitExp - (int)(((__float_as_uint(amax) >> 23) & 0xffu) - 126u);
  const float hs = __uint_as_float((uint32_t)(127 + ex) << 23);
  const float unscale = __uint_as_float((uint32_t)(127 - ex) << 23) * w_unscale[a];
  f16x8 xh[D / 16], xl[D / 16];
#pragma unroll
  for (int hb = 0; hb < kMlpH / 32; ++hb) {
#pragma unroll
    for (int v = 0; v < 16; v += 2) {
      f16x2 hi, lo;
      split_f16x2(hacc[hb][v] * hs, hacc[hb][v + 1] * hs, hi, lo);
      xh[2 * hb + (v >> 3)][v & 7] = hi[0]; xh[2 * hb + (v >> 3)][(v & 7) + 1] = hi[1];
      xl[2 * hb + (v >> 3)][v & 7] = lo[0]; xl[2 * hb + (v >> 3)][(v & 7) + 1] = lo[1];
    }
  }

  class_tiles_and_finish<D, DUMP, SPLIT>(tb, w, buf_a, buf_b, buf_c, src, xh, xl, unscale, a, CT, C, M, pos, id, valid, dw_g,
                                  sortkey, logits_out);
}

}  // namespace sp
