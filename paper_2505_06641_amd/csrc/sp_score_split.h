// Scoring kernel for logistic heads with float32 features on the matrix cores,
// d <= 256, M <= 16: float32 products emulated by three half-precision MFMAs.
//
// Every float32 operand v is scaled by a power of two (per request row for the
// features, per application for the weights; exact) into (-2^15, 2^15) and
// split as v = hi + lo with hi = fp16(v), lo = fp16(v - hi): 22 significant
// bits.  x.w is then  hi.hi + lo.hi + hi.lo  on v_mfma_f32_32x32x16_f16 with
// float32 accumulation (fp16 x fp16 products are exact in float32; the dropped
// lo.lo term is below 2^-22 of the product), at 16x the float32 MFMA rate per
// instruction, i.e. 5.3x per float32 product.
//
// Work split as in the float32 kernel it replaces: one workgroup = 8 wavefronts
// = 256 requests of one application; a wavefront keeps the split features of
// its 32 requests in registers (D/2 VGPRs) and walks the classes 32 at a time.
// Per class tile it computes the transposed logit tile Z^T[class, request]
// (classes on the MFMA row axis: every lane owns one request column and 16 of
// the 32 classes, so softmax statistics stay inside a lane), keeps a running
// maximum per request (online softmax), splits the exponentials the same way
// and feeds them back into the matrix cores against the [16 x 32] tile of the
// variants' per-class accuracies on v_mfma_f32_16x16x32_f16 (16 variants x 16
// requests x 32 classes per instruction, half the matrix-core time of a 32-row
// tile whose upper half would be empty; one exchange of lane rows puts the
// exponentials where that instruction reads them), accumulating
// sum_c exp(z_c) Acc[m][c]; the denominator sum_c exp(z_c) is a plain sum in
// the lanes.  The posterior is never formed or stored (Def. 4.1.2; Sec. 4.1
// eq. (9)); EA = numerators / denominator, then variance and key (Sec. 5.1.1
// eq. (12)).
//
// Weights, table and bias of each (application, class tile) are packed once at
// context creation into one contiguous block in exactly the order the lanes
// read it from LDS; the next block is fetched through registers while the current one is in use
// (three LDS buffers).
#pragma once
#include "sp_common.h"
#include "sp_score_generic.h"

namespace sp {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

constexpr int kMfWaves = 8;
constexpr int kMfThreads = kMfWaves * kWave;
constexpr int kMfTile = kMfWaves * 32;      // requests per workgroup
constexpr int kClassTile = 32;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kNegBig = -1e30f;
constexpr int kSplitExp = 15;               // operands are scaled into (-2^15, 2^15)
constexpr float kExpShift = 14.0f;          // exponentials are scaled into (0, 2^14]

// Packed block of one (application, class tile), in 16-byte units (8 halves or 4 floats each):
//   W     [D/16][2][64]  unit ((s*2 + part)*64 + lane): halves e = 0..7 hold part (0 = hi, 1 = lo) of
//                        W'[k = (lane/32)*D/2 + 8 s + e][class = 32 ct + lane%32], W' = W * 2^ew
//   table [2][64]        unit (part*64 + lane): halves e hold part of Acc[m = lane%16][class] (0 for m >= M),
//                        class = 32 ct + 16 s + 8 (e/4) + 4 g + e%4 with g = lane/32, s = (lane/16)%2: the
//                        A operand of a 16x16x32 MFMA whose K index 8 (lane/16) + e runs over the classes
//                        in the order the exponentials sit in the lanes after the row swap (softmax_phase)
//   bias  [4][2]         unit (q*2 + g): floats j = 0..3 hold b[32 ct + 8 q + 4 g + j], -1e30 beyond C
template <int D>
struct SplitBlock {
  static constexpr int kWUnits = (D / 16) * 2 * 64;
  static constexpr int kTabUnits = 2 * 64;
  static constexpr int kBiasUnits = 8;
  static constexpr int kChunks = (kWUnits + kTabUnits + kBiasUnits + 63) / 64;   // 1 KB pieces, one LDS-DMA each
  static constexpr int kUnits = kChunks * 64;
  static constexpr int kBytes = kUnits * 16;
};

inline uint16_t host_f32_to_f16_bits(float f) { return __builtin_bit_cast(uint16_t, (_Float16)f); }

inline void host_split(float v, uint16_t& hi, uint16_t& lo) {
  const _Float16 h = (_Float16)v;
  hi = __builtin_bit_cast(uint16_t, h);
  lo = __builtin_bit_cast(uint16_t, (_Float16)(v - (float)h));
}

// Power-of-two scale that brings |v| <= vmax into (-2^15, 2^15): returns the exponent ew (scale = 2^ew).
inline int host_scale_exponent(float vmax) {
  if (!(vmax > 0.f) || !std::isfinite(vmax)) return 0;
  int e = 0;
  (void)std::frexp(vmax, &e);            // vmax = f * 2^e, f in [0.5, 1)
  int ew = kSplitExp - e;
  if (ew > 100) ew = 100;
  if (ew < -100) ew = -100;
  return ew;
}

// Which input index k a weight unit holds at (k-step s, lane half g, element e).  kMapRows: the lane
// half owns one half of the input row (features loaded from memory).  kMapTile: the input comes out of
// a previous 32x32 MFMA tile, where lane half g owns rows 8q + 4g + j of every block of 32.
constexpr int kMapRows = 0, kMapTile = 1;
template <int D, int KMAP>
inline int split_k_index(int s, int g, int e) {
  return KMAP == kMapRows ? g * (D / 2) + 8 * s + e : 32 * (s / 2) + 8 * (2 * (s % 2) + e / 4) + 4 * g + e % 4;
}

// Host-side packing of one application's head (called at context creation).  Returns 2^-ew.
template <int D, int KMAP>
inline float pack_split_blocks(const float* W /*[d,C]*/, const float* b /*[C]*/, const float* acc /*[M,C]*/, int d,
                               int C, int M, unsigned char* out /*[CT * kBytes]*/) {
  using SB = SplitBlock<D>;
  float wmax = 0.f;
  for (size_t i = 0; i < (size_t)d * C; ++i) wmax = std::max(wmax, std::fabs(W[i]));
  const int ew = host_scale_exponent(wmax);
  const float ws = std::ldexp(1.0f, ew);
  const int CT = (C + kClassTile - 1) / kClassTile;
  for (int ct = 0; ct < CT; ++ct) {
    unsigned char* blk = out + (size_t)ct * SB::kBytes;
    std::memset(blk, 0, SB::kBytes);
    uint16_t* wh = reinterpret_cast<uint16_t*>(blk);
    for (int s = 0; s < D / 16; ++s)
      for (int lane = 0; lane < 64; ++lane)
        for (int e = 0; e < 8; ++e) {
          const int k = split_k_index<D, KMAP>(s, lane / 32, e), cls = 32 * ct + lane % 32;
          const float v = (k < d && cls < C) ? W[(size_t)k * C + cls] * ws : 0.f;
          uint16_t hi, lo;
          host_split(v, hi, lo);
          wh[((size_t)(s * 2 + 0) * 64 + lane) * 8 + e] = hi;
          wh[((size_t)(s * 2 + 1) * 64 + lane) * 8 + e] = lo;
        }
    uint16_t* tab = wh + (size_t)SB::kWUnits * 8;
    for (int lane = 0; lane < 64; ++lane)
      for (int e = 0; e < 8; ++e) {
        const int m = lane % 16, g = lane / 32, sl = (lane / 16) % 2;
        const int cls = 32 * ct + 16 * sl + 8 * (e / 4) + 4 * g + e % 4;
        const float v = (cls < C && m < M) ? acc[(size_t)m * C + cls] : 0.f;
        uint16_t hi, lo;
        host_split(v, hi, lo);
        tab[((size_t)0 * 64 + lane) * 8 + e] = hi;
        tab[((size_t)1 * 64 + lane) * 8 + e] = lo;
      }
    float* bias = reinterpret_cast<float*>(blk + (size_t)(SB::kWUnits + SB::kTabUnits) * 16);
    for (int q = 0; q < 4; ++q)
      for (int g = 0; g < 2; ++g)
        for (int j = 0; j < 4; ++j) {
          const int cls = 32 * ct + 8 * q + 4 * g + j;
          bias[(q * 2 + g) * 4 + j] = cls < C ? b[cls] : kNegBig;
        }
  }
  return std::ldexp(1.0f, -ew);
}

// Global -> LDS copy of one packed block with the LDS-DMA load (no registers in between): every lane
// of a wavefront supplies the address of its own 16 bytes, the data lands at the (wave-uniform) LDS
// base plus 16 * lane.  Used for the first block only: the instruction keeps the issuing wavefront
// busy for about 300 cycles per KB on this part, too slow for the steady state.
template <int D, int WAVES = kMfWaves>
__device__ __forceinline__ void stage_block_dma(const float4* __restrict__ src, float4* dst_lds, int wave, int lane) {
  using SB = SplitBlock<D>;
  for (int ch = wave; ch < SB::kChunks; ch += WAVES)
    __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)(src + ch * 64 + lane),
                                     (void __attribute__((address_space(3)))*)(dst_lds + ch * 64), 16, 0, 0);
}

// Steady-state staging through registers, half a block per phase: the loads are issued when a phase
// starts (fetch), the data is parked in LDS when it ends (park), so the L2 latency hides behind the
// phase's own work.  Part 0 covers the first (up to) three units per thread, part 1 the rest.
template <int D>
struct StageRegs {
  static constexpr int kPerThread = (SplitBlock<D>::kUnits + kMfThreads - 1) / kMfThreads;   // 16-byte units
  static constexpr int kCount0 = kPerThread < 3 ? kPerThread : 3;
  static constexpr int kCount1 = kPerThread - kCount0;
  static_assert(kCount1 <= 3, "block too large for the two-part staging");
  f32x4 v[3];
};
// The loads are written as inline assembly so that the compiler cannot sink them down to their use
// (it would, across the whole phase); since it then does not know that they are asynchronous, the
// matching s_waitcnt is explicit in stage_park, tied to the same registers.
template <int D, int PART>
__device__ __forceinline__ void stage_fetch(const float4* __restrict__ src, StageRegs<D>& st, int tid) {
  using SB = SplitBlock<D>;
  constexpr int kFirst = PART == 0 ? 0 : StageRegs<D>::kCount0 * kMfThreads;
  constexpr int kCount = PART == 0 ? StageRegs<D>::kCount0 : StageRegs<D>::kCount1;
#pragma unroll
  for (int i = 0; i < kCount; ++i) {
    const float4* p = src + min(kFirst + tid + i * kMfThreads, SB::kUnits - 1);
    asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(st.v[i]) : "v"(p) : "memory");
  }
}
template <int D, int PART>
__device__ __forceinline__ void stage_park(float4* dst_lds, StageRegs<D>& st, int tid) {
  using SB = SplitBlock<D>;
  constexpr int kFirst = PART == 0 ? 0 : StageRegs<D>::kCount0 * kMfThreads;
  constexpr int kCount = PART == 0 ? StageRegs<D>::kCount0 : StageRegs<D>::kCount1;
  if (kCount == 0) return;
  asm volatile("s_waitcnt vmcnt(0)" : "+v"(st.v[0]), "+v"(st.v[1]), "+v"(st.v[2]) : : "memory");
#pragma unroll
  for (int i = 0; i < kCount; ++i) {
    const int idx = kFirst + tid + i * kMfThreads;
    if (idx < SB::kUnits) reinterpret_cast<f32x4*>(dst_lds)[idx] = st.v[i];
  }
}

__device__ __forceinline__ f16x8 as_f16x8(const float4& v) { return __builtin_bit_cast(f16x8, v); }

// v = hi + lo in half precision (v already inside the fp16 range)
__device__ __forceinline__ void split_f16(float v, _Float16& hi, _Float16& lo) {
  hi = (_Float16)v;
  lo = (_Float16)(v - (float)hi);
}
// The same for two values at once, written so that the conversions pair up (one packed conversion for
// the two hi parts, one for the two lo parts) and the remainder is a single fused operation on the
// half-precision value: 2 instructions per value instead of 4.
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void split_f16x2(float a, float b, f16x2& hi, f16x2& lo) {
  const f32x2 v = {a, b};
  hi = __builtin_convertvector(v, f16x2);
  // remainder v - hi with the half-precision operand read straight out of the packed register
  // (mixed-precision fma: op_sel_hi marks source 0 as fp16, op_sel picks its upper half)
  const uint32_t hb = __builtin_bit_cast(uint32_t, hi);
  f32x2 r;
  asm("v_fma_mix_f32 %0, %1, -1.0, %2 op_sel_hi:[1,0,0]" : "=v"(r[0]) : "v"(hb), "v"(a));
  asm("v_fma_mix_f32 %0, %1, -1.0, %2 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(r[1]) : "v"(hb), "v"(b));
  lo = __builtin_convertvector(r, f16x2);
}

// Matrix phase of one class tile: acc = (W' x') for the tile's 32 classes and the wavefront's 32 requests.
template <int D>
__device__ __forceinline__ void logits_phase(const float4* blk, const f16x8 (&xh)[D / 16], const f16x8 (&xl)[D / 16],
                                             f32x16& acc, int lane) {
  // two accumulator chains: a dependent 32x32x16 MFMA can only issue every ~52 cycles, an independent
  // one every 32
  f32x16 acc2;
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    acc[v] = 0.f;
    acc2[v] = 0.f;
  }
  // weight fragments are fetched kPre k-steps ahead of the MFMAs that use them
  constexpr int S = D / 16;
  constexpr int kPre = S < 2 ? S : 2;
  const float4* wp = blk + lane;
  float4 wbuf[kPre][2];
#pragma unroll
  for (int s = 0; s < kPre; ++s) {
    wbuf[s][0] = wp[(s * 2 + 0) * 64];
    wbuf[s][1] = wp[(s * 2 + 1) * 64];
  }
#pragma unroll
  for (int s = 0; s < S; ++s) {
    const f16x8 wh = as_f16x8(wbuf[s % kPre][0]);
    const f16x8 wl = as_f16x8(wbuf[s % kPre][1]);
    if (s + kPre < S) {
      wbuf[s % kPre][0] = wp[((s + kPre) * 2 + 0) * 64];
      wbuf[s % kPre][1] = wp[((s + kPre) * 2 + 1) * 64];
    }
    __builtin_amdgcn_sched_barrier(0);   // keep the reads of step s + kPre ahead of the MFMAs of step s
    // strict alternation between the two chains, also across k-steps (three MFMAs per step)
    if (s & 1) {
      acc2 = __builtin_amdgcn_mfma_f32_32x32x16_f16(wh, xh[s], acc2, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(wl, xh[s], acc, 0, 0, 0);
      acc2 = __builtin_amdgcn_mfma_f32_32x32x16_f16(wh, xl[s], acc2, 0, 0, 0);
    } else {
      acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(wh, xh[s], acc, 0, 0, 0);
      acc2 = __builtin_amdgcn_mfma_f32_32x32x16_f16(wl, xh[s], acc2, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(wh, xl[s], acc, 0, 0, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
  }
#pragma unroll
  for (int v = 0; v < 16; ++v) acc[v] += acc2[v];
}

__device__ __forceinline__ float other_half(float v, int g) {
  // value held by lane ^ 32 (v_permlane32_swap: pure vector ALU, does not go through the LDS queue)
  typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
  const u32x2 sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return __uint_as_float(g == 0 ? sw[1] : sw[0]);
}

// Softmax phase of one class tile (mostly vector ALU work): logits = acc * 2^-(ex+ew) + bias, online
// softmax update, exponentials x table tile.
template <int D, bool DUMP, bool SPLIT>
__device__ __forceinline__ void softmax_phase(const float4* blk, f32x16& acc, float unscale, f32x4& ea_lo, f32x4& ea_hi,
                                              float& ssum, float& m2, int ct, int C, int g, int lane, bool valid,
                                              int64_t dump_row, float* __restrict__ logits_out, float& best_z,
                                              int& best_c) {
  using SB = SplitBlock<D>;
  // The other wavefront of this SIMD is, most of the time, streaming the MFMAs of its matrix phase and
  // always has the next one ready; without a higher priority the few MFMAs of this phase would wait
  // for that whole stream to end.
  __builtin_amdgcn_s_setprio(2);
  float4 bq[4];
  {
    const float4* bp = blk + SB::kWUnits + SB::kTabUnits;
#pragma unroll
    for (int q = 0; q < 4; ++q) bq[q] = bp[q * 2 + g];
  }
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    acc[4 * q + 0] = fmaf(acc[4 * q + 0], unscale, bq[q].x);
    acc[4 * q + 1] = fmaf(acc[4 * q + 1], unscale, bq[q].y);
    acc[4 * q + 2] = fmaf(acc[4 * q + 2], unscale, bq[q].z);
    acc[4 * q + 3] = fmaf(acc[4 * q + 3], unscale, bq[q].w);
  }
  if (DUMP && valid) {
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int cls = 32 * ct + 8 * (v >> 2) + 4 * g + (v & 3);
      if (cls < C) logits_out[dump_row + cls] = acc[v];
    }
  }
  // the request's maximum spans both lane halves
  float mt = acc[0];
#pragma unroll
  for (int v = 1; v < 16; ++v) mt = fmaxf(mt, acc[v]);
  if (SPLIT && __builtin_amdgcn_ballot_w64(mt > best_z) != 0ull) {
    // subgroup label (Sec. 5.3.2): class of the largest logit seen by this lane so far; equal logits keep
    // the smallest class (v ascending is class ascending inside a lane)
    int vi = 15;
#pragma unroll
    for (int v = 14; v >= 0; --v) vi = acc[v] == mt ? v : vi;
    const bool up = mt > best_z;
    best_c = up ? 32 * ct + 8 * (vi >> 2) + 4 * g + (vi & 3) : best_c;
    best_z = up ? mt : best_z;
  }
  mt = fmaxf(mt, other_half(mt, g));
  const float m2n = fmaxf(m2, mt * kLog2e);
  const float scale = __builtin_amdgcn_exp2f(m2 - m2n);
  m2 = m2n;
  const float shift = kExpShift - m2n;
  // Exponentials x accuracy-table tile on 16x16x32 MFMAs (16 variants x 16 requests x 32 classes each):
  // ea_lo of lane (row q = lane/16, j = lane%16) holds variants 4q..4q+3 of request j, ea_hi those of
  // request 16 + j.  A lane's own request is lane%32, so in the odd rows ea_lo belongs to the neighbouring
  // row's request and in the even rows ea_hi does: they take that row's rescaling factor.
  typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
  {
    const u32x2 sw = __builtin_amdgcn_permlane16_swap(__float_as_uint(scale), __float_as_uint(scale), false, false);
    const bool odd = (lane & 16) != 0;
    const float nb = __uint_as_float(odd ? sw[0] : sw[1]);
    const float sc_lo = odd ? nb : scale, sc_hi = odd ? scale : nb;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      ea_lo[v] *= sc_lo;
      ea_hi[v] *= sc_hi;
    }
  }
  // the softmax denominator of this lane's 16 classes is a plain sum (two chains)
  float s0 = 0.f, s1 = 0.f;
  f16x8 ph[2], pl[2];
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
    for (int e = 0; e < 8; e += 2) {
      const float p0 = __builtin_amdgcn_exp2f(fmaf(acc[8 * ks + e], kLog2e, shift));       // in (0, 2^14]
      const float p1 = __builtin_amdgcn_exp2f(fmaf(acc[8 * ks + e + 1], kLog2e, shift));
      s0 += p0;
      s1 += p1;
      f16x2 hi, lo;
      split_f16x2(p0, p1, hi, lo);
      ph[ks][e] = hi[0]; ph[ks][e + 1] = hi[1];
      pl[ks][e] = lo[0]; pl[ks][e + 1] = lo[1];
    }
  }
  ssum = fmaf(ssum, scale, s0 + s1);
  // Row swap: a lane holds classes slice 0 (ph[0]) and slice 1 (ph[1]) of its own request.  Exchanging
  // slice 0 of the odd rows with slice 1 of the even rows leaves, in the first register set, requests
  // 0..15 with K slices (g, slice) = (0,0), (0,1), (1,0), (1,1) in rows 0..3, and in the second set the
  // same for requests 16..31: the B operands of the two MFMAs.
  f16x8 bh_lo, bh_hi, bl_lo, bl_hi;
  {
    typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
    const u32x4 h0 = __builtin_bit_cast(u32x4, ph[0]), h1 = __builtin_bit_cast(u32x4, ph[1]);
    const u32x4 l0 = __builtin_bit_cast(u32x4, pl[0]), l1 = __builtin_bit_cast(u32x4, pl[1]);
    u32x4 a_h, b_h, a_l, b_l;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const u32x2 sh = __builtin_amdgcn_permlane16_swap(h0[i], h1[i], false, false);
      const u32x2 sl = __builtin_amdgcn_permlane16_swap(l0[i], l1[i], false, false);
      a_h[i] = sh[0]; b_h[i] = sh[1];
      a_l[i] = sl[0]; b_l[i] = sl[1];
    }
    bh_lo = __builtin_bit_cast(f16x8, a_h); bh_hi = __builtin_bit_cast(f16x8, b_h);
    bl_lo = __builtin_bit_cast(f16x8, a_l); bl_hi = __builtin_bit_cast(f16x8, b_l);
  }
  const float4* tp = blk + SB::kWUnits + lane;
  const f16x8 th = as_f16x8(tp[0]);
  const f16x8 tl = as_f16x8(tp[64]);
  ea_lo = __builtin_amdgcn_mfma_f32_16x16x32_f16(th, bh_lo, ea_lo, 0, 0, 0);
  ea_hi = __builtin_amdgcn_mfma_f32_16x16x32_f16(th, bh_hi, ea_hi, 0, 0, 0);
  ea_lo = __builtin_amdgcn_mfma_f32_16x16x32_f16(tl, bh_lo, ea_lo, 0, 0, 0);
  ea_hi = __builtin_amdgcn_mfma_f32_16x16x32_f16(tl, bh_hi, ea_hi, 0, 0, 0);
  ea_lo = __builtin_amdgcn_mfma_f32_16x16x32_f16(th, bl_lo, ea_lo, 0, 0, 0);
  ea_hi = __builtin_amdgcn_mfma_f32_16x16x32_f16(th, bl_hi, ea_hi, 0, 0, 0);
  __builtin_amdgcn_s_setprio(0);
}

// After the last class tile: expected accuracies (eq. (9), with the prior's affine map), variance and key
// (eq. (12)), the subgroup label, and the request's entries of the grouped arrays.
template <bool SPLIT>
__device__ __forceinline__ void score_epilogue(const Tables& tb, const Window& w, const f32x16& eacc, float m2,
                                               float best_z, int best_c, int a, int M, int pos, int id, bool valid,
                                               int r, int g, const float2* __restrict__ dw_g,
                                               uint32_t* __restrict__ sortkey) {
  // eacc[v] of lane (r, g) is table row 8*(v/4) + 4*g + v%4 for request r:
  // v 0..3 -> variants 4g..4g+3, v 4..7 -> variants 8+4g..8+4g+3, v = 8 at g = 0 -> the sum of exponentials
  const float ssum = __shfl(eacc[8], r);
  const float inv = 1.0f / ssum;
  // prior of Sec. 4.2 eq. (10)-(11) as an affine map of the expected accuracies (gain 1, bias 0 without one)
  const float gain = tb.ea_gain[a];
  const float* biasp = tb.ea_bias + a * tb.Mmax;
  float ea[8];
  float part = 0.f;
#pragma unroll
  for (int v = 0; v < 8; ++v) {
    const int m = 8 * (v >> 2) + 4 * g + (v & 3);
    ea[v] = (m < M) ? fmaf(gain, eacc[v] * inv, biasp[m]) : 0.f;
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
  if (SPLIT) {
    // the lane halves' candidates meet; the largest posterior is exp(z_max - reference) / sum
    const float oz = other_half(best_z, g);
    const int oc = __float_as_int(other_half(__int_as_float(best_c), g));
    const bool take = oz > best_z || (oz == best_z && oc < best_c);
    const float zmax = take ? oz : best_z;
    const int cmax = take ? oc : best_c;
    const float pmax = __builtin_amdgcn_exp2f(fmaf(zmax, kLog2e, kExpShift - m2));
    if (g == 0) w.sub_g[pos] = (pmax * inv > 0.5f) ? 1 + cmax : 0;
  }
  if (g == 0) {
    const float2 dw = dw_g[pos];           // (deadline, weight), brought to the grouped position by the grouping pass
    const float Di = dw.x, wi = dw.y;
    uint32_t err = 0;
    if (!(Di > 0.f)) err |= kErrDeadline;
    if (!(wi >= 0.f)) err |= kErrWeight;
    if (err) atomicOr(&w.st->err, err);
    const float key = fabsf(wi * (1.0f + var) * expf(-Di * tb.inv_timescale));   // a weight of -0 must not give the key -0: its bits would sort first
    w.key[id] = key;
    sortkey[pos] = tb.pol_edf ? __float_as_uint(Di) : ~__float_as_uint(key);   // ascending deadline, or descending key
    w.rec_g[pos] = make_float4(__int_as_float(id), Di, wi, 0.f);   // what the ordering needs of this request, in one piece
  }
}

// Class tiles and epilogue shared by the scoring kernels: given the wavefront's 32 requests as split
// half-precision inputs (xh, xl; logits = unscale * W' x' + b), walk the application's packed blocks,
// then EA, variance, key.  buf_a already holds (or is receiving by DMA) block 0; the caller has not yet
// synchronised the workgroup on it.
template <int D, bool DUMP, bool SPLIT>
__device__ __forceinline__ void class_tiles_and_finish(
    const Tables& tb, const Window& w, float4* buf_a, float4* buf_b, float4* buf_c, const float4* __restrict__ src,
    const f16x8 (&xh)[D / 16], const f16x8 (&xl)[D / 16], float unscale, int a, int CT, int C, int M, int pos, int id,
    bool valid, const float2* __restrict__ dw_g, uint32_t* __restrict__ sortkey,
    float* __restrict__ logits_out) {
  using SB = SplitBlock<D>;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r = lane & 31, g = lane >> 5;
  __syncthreads();

  float m2 = kNegBig;                                    // running maximum, in units of log2
  float best_z = kNegBig;                                // largest logit of this lane's classes and its class
  int best_c = 0x7fffffff;
  f32x4 ea_lo = {0.f, 0.f, 0.f, 0.f}, ea_hi = {0.f, 0.f, 0.f, 0.f};   // EA numerators (layout: softmax_phase)
  float ssum = 0.f;                                      // softmax denominator of this lane's classes
  const int64_t dump_row = (int64_t)id * tb.Cmax;

  // The two wavefronts that share a SIMD take the phases of a class tile in opposite order, so that the
  // matrix cores always have a wavefront feeding them while the other one keeps the vector ALU busy:
  // in the iteration that has block T+1 complete in LDS, wavefronts 0..3 ("early") run the matrix phase
  // and then the softmax phase of tile T+1, wavefronts 4..7 ("late") the softmax phase of tile T (whose
  // logits they carried over the barrier) and then the matrix phase of tile T+1.  Either way a wavefront
  // holds one logit tile at a time.  One barrier per tile: block T+2 is fetched through registers in two
  // halves during the iteration and is complete in LDS at its end.
  const bool late = wave >= kMfWaves / 2;
  f32x16 acc;
  StageRegs<D> stg;
  stg.v[0] = stg.v[1] = stg.v[2] = f32x4{0.f, 0.f, 0.f, 0.f};
  // block 1 has to be in LDS before the first iteration reads it
  {
    const float4* nsrc = src + (size_t)(CT > 1 ? 1 : 0) * SB::kUnits;
    stage_fetch<D, 0>(nsrc, stg, tid);
    logits_phase<D>(buf_a, xh, xl, acc, lane);
    stage_park<D, 0>(buf_b, stg, tid);
    stage_fetch<D, 1>(nsrc, stg, tid);
    if (!late)
      softmax_phase<D, DUMP, SPLIT>(buf_a, acc, unscale, ea_lo, ea_hi, ssum, m2, 0, C, g, lane, valid, dump_row,
                                    logits_out, best_z, best_c);
    stage_park<D, 1>(buf_b, stg, tid);
    __syncthreads();
  }
#define SP_TILE(T, CUR, NXT, FILL)                                                                             \
  if ((T) < CT) {                                                                                              \
    const bool more = (T) + 1 < CT;                                                                            \
    const float4* nsrc = src + (size_t)((T) + 2 < CT ? (T) + 2 : CT - 1) * SB::kUnits;                        \
    stage_fetch<D, 0>(nsrc, stg, tid);                                                                         \
    if (!late) {                                                                                               \
      if (more) logits_phase<D>(NXT, xh, xl, acc, lane);                                                       \
      stage_park<D, 0>(FILL, stg, tid);   /* (past the last block: a copy nobody reads) */                     \
      stage_fetch<D, 1>(nsrc, stg, tid);                                                                       \
      if (more)                                                                                                \
        softmax_phase<D, DUMP, SPLIT>(NXT, acc, unscale, ea_lo, ea_hi, ssum, m2, (T) + 1, C, g, lane, valid,  \
                                      dump_row, logits_out, best_z, best_c);                                   \
    } else {                                                                                                   \
      softmax_phase<D, DUMP, SPLIT>(CUR, acc, unscale, ea_lo, ea_hi, ssum, m2, (T), C, g, lane, valid,        \
                                    dump_row, logits_out, best_z, best_c);                                     \
      stage_park<D, 0>(FILL, stg, tid);                                                                        \
      stage_fetch<D, 1>(nsrc, stg, tid);                                                                       \
      if (more) logits_phase<D>(NXT, xh, xl, acc, lane);                                                       \
    }                                                                                                          \
    stage_park<D, 1>(FILL, stg, tid);                                                                          \
    __syncthreads();                       /* block T+2 is complete in LDS, blocks T and T+1 are free */       \
  }
  for (int t0 = 0; t0 < CT; t0 += 3) {
    SP_TILE(t0, buf_a, buf_b, buf_c)
    SP_TILE(t0 + 1, buf_b, buf_c, buf_a)
    SP_TILE(t0 + 2, buf_c, buf_a, buf_b)
  }
#undef SP_TILE
  if (DUMP) return;
  // Back to one request per lane pair for the epilogue: lane (r, g) takes variants 4g..4g+3 from row g and
  // 8+4g..8+4g+3 from row 2+g, column r%16, out of ea_lo (r < 16) or ea_hi; entry 8 is the denominator.
  f32x16 eacc;
  {
    const int src_a = 16 * g + (r & 15), src_b = 16 * (2 + g) + (r & 15);
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const float a_lo = __shfl(ea_lo[v], src_a), a_hi = __shfl(ea_hi[v], src_a);
      const float b_lo = __shfl(ea_lo[v], src_b), b_hi = __shfl(ea_hi[v], src_b);
      eacc[v] = r < 16 ? a_lo : a_hi;
      eacc[4 + v] = r < 16 ? b_lo : b_hi;
    }
    eacc[8] = ssum + other_half(ssum, g);
#pragma unroll
    for (int v = 9; v < 16; ++v) eacc[v] = 0.f;
  }
  score_epilogue<SPLIT>(tb, w, eacc, m2, best_z, best_c, a, M, pos, id, valid, r, g, dw_g, sortkey);
}

// This lane's half of its request's features, k = g*D/2 + [0, D/2): the row scaled by a power of two into
// (-2^15, 2^15) and split into half-precision hi and lo parts.  Returns the factor that undoes the scaling
// of row and weights.  `scratch` is 8 x 66 units of LDS private to the wavefront.
template <int D>
__device__ __forceinline__ float load_split_features(const float* __restrict__ x, int id, int d, float4* scratch,
                                                     int lane, float w_unscale_a, f16x8 (&xh)[D / 16],
                                                     f16x8 (&xl)[D / 16]) {
  const int r = lane & 31, g = lane >> 5;
    float xr[D / 2];
    const float* row = x + (int64_t)id * d;
    if (D == 256 && (d & 3) == 0) {
      // Coalesced: the wavefront reads whole rows (one 16-byte piece per lane, 1 KB per instruction),
      // parks eight rows at a time in the block buffers that are still idle, and every lane then
      // picks its own half row out of LDS.  Row stride 66 and half offset 33 (in 16-byte units) keep
      // both the writes and the reads free of bank conflicts.
      // (scratch: this wavefront's own 8 x 66 units of an idle block buffer)
      // rows of pass ps+1 are already in flight while pass ps goes through LDS
      float4 rows[2][8];
      auto fetch_rows = [&](int ps, float4 (&dst)[8]) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const int rid = __shfl(id, 8 * ps + i);
          dst[i] = make_float4(0.f, 0.f, 0.f, 0.f);
          // feature rows are read once: a streaming load, so that they do not push the packed blocks,
          // which every workgroup of the die reads again, out of its L2
          if (4 * lane < d) {
            const f32x4 v = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(x + (int64_t)rid * d + 4 * lane));
            dst[i] = make_float4(v[0], v[1], v[2], v[3]);
          }
        }
      };
      fetch_rows(0, rows[0]);
#pragma unroll
      for (int ps = 0; ps < 4; ++ps) {
        if (ps + 1 < 4) fetch_rows(ps + 1, rows[(ps + 1) & 1]);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < 8; ++i) scratch[i * 66 + g * 33 + r] = rows[ps & 1][i];
        if ((r >> 3) == ps) {
          const float4* mine = scratch + (r & 7) * 66 + g * 33;
#pragma unroll
          for (int q = 0; q < D / 8; ++q) {
            const float4 v = mine[q];
            xr[4 * q + 0] = v.x; xr[4 * q + 1] = v.y; xr[4 * q + 2] = v.z; xr[4 * q + 3] = v.w;
          }
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    } else if ((d & 3) == 0) {                           // rows are 16-byte aligned: whole float4 in or out of range
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
    float amax = 0.f;
#pragma unroll
    for (int q = 0; q < D / 2; ++q) amax = fmaxf(amax, fabsf(xr[q]));
    amax = fmaxf(amax, __shfl_xor(amax, 32));
    // amax = f * 2^e with f in [0.5, 1): scale by 2^(15 - e); rows of zeros (or denormals) keep scale 1
    int ex = 0;
    if (amax >= 1e-30f && amax <= 3e38f) ex = kSplitExp - (int)(((__float_as_uint(amax) >> 23) & 0xffu) - 126u);
    const float xs = __uint_as_float((uint32_t)(127 + ex) << 23);
    const float unscale = __uint_as_float((uint32_t)(127 - ex) << 23) * w_unscale_a;
#pragma unroll
    for (int q = 0; q < D / 2; q += 2) {
      f16x2 hi, lo;
      split_f16x2(xr[q] * xs, xr[q + 1] * xs, hi, lo);
      xh[q >> 3][q & 7] = hi[0]; xh[q >> 3][(q & 7) + 1] = hi[1];
      xl[q >> 3][q & 7] = lo[0]; xl[q >> 3][(q & 7) + 1] = lo[1];
    }
  return unscale;
}

// Which scoring tile a workgroup takes.  Consecutive workgroup ids go to the chip's eight accelerator dies
// (XCDs) in turn, each with an L2 of its own; tiles are ordered by application, so giving every die one
// contiguous eighth of the tiles lets each application's packed blocks live in one L2 instead of eight.
// The launch must hold at least 8 * ceil(n_tiles / 8) workgroups; returns -1 for a workgroup without a tile.
constexpr int kXcds = 8;
__device__ __forceinline__ int xcd_tile(int wg, int n_tiles) {
  const int per = (n_tiles + kXcds - 1) / kXcds;
  const int j = wg / kXcds, tile = (wg % kXcds) * per + j;
  return (j < per && tile < n_tiles) ? tile : -1;
}

// DUMP: the launch only writes the logits (logits_out) and ends before the epilogue; dw_g and sortkey are
// then null and must not be touched.
template <int D, bool DUMP, bool SPLIT>
__global__ __launch_bounds__(kMfThreads) void k_score_logistic_split(
    Tables tb, Window w, const float* __restrict__ x, const int32_t* __restrict__ ids, const float2* __restrict__ dw_g,
    uint32_t* __restrict__ sortkey, const unsigned char* __restrict__ blocks,
    const int64_t* __restrict__ block_off /*[A] bytes*/, const float* __restrict__ w_unscale /*[A]*/,
    float* __restrict__ logits_out) {
  using SB = SplitBlock<D>;
  // three separate arrays (not one array split in three) so that the compiler can tell that the
  // blocks being read and the block being filled never overlap
  __shared__ float4 buf_a[SB::kUnits];
  __shared__ float4 buf_b[SB::kUnits];
  __shared__ float4 buf_c[SB::kUnits];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r = lane & 31;
  const int tile = xcd_tile(blockIdx.x, w.tile_start[tb.A]);
  if (tile < 0) return;
  const int4 desc = w.tile_desc[tile];
  const int a = desc.x, seg_e = desc.z;
  const int pos = desc.y + wave * 32 + r;
  const bool valid = pos < seg_e;
  const int id = ids[valid ? pos : seg_e - 1];           // padding lanes recompute the last request, never store
  const int d = tb.d, C = tb.n_classes[a], M = tb.n_models[a];
  const int CT = (C + kClassTile - 1) / kClassTile;

  const float4* src = reinterpret_cast<const float4*>(blocks + block_off[a]);
  stage_block_dma<D>(src, buf_a, wave, lane);

  f16x8 xh[D / 16], xl[D / 16];
  float4* scratch = (wave < kMfWaves / 2 ? buf_b : buf_c) + (wave % (kMfWaves / 2)) * (8 * 66);
  const float unscale = load_split_features<D>(x, id, d, scratch, lane, w_unscale[a], xh, xl);
  class_tiles_and_finish<D, DUMP, SPLIT>(tb, w, buf_a, buf_b, buf_c, src, xh, xl, unscale, a, CT, C, M, pos, id, valid, dw_g,
                                  sortkey, logits_out);
}


}  // namespace sp
