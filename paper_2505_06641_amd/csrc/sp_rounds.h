// One greedy batch-selection round (Alg. 1 generalised to batch-capped rounds;
// eq. (2) utility; eq. (13) arg max; eq. (1) clock with the batch as the unit).
//
// k_round_score: one workgroup per (application, variant).  It walks the
// application's service order from the head pointer, keeps the first B live
// requests (pending, and penalty on the earliest possible completion below 1)
// as the candidate window, and evaluates
//   Score[a,m,b] = sum_{j<=b} key_j * EA[j,m] * (1 - gamma_a(D_j, t + L[a][m][b]))
// for every b, pairing batch sizes b and B+1-b on the same lanes so that all
// lanes do the same amount of work.  Its best (score, candidate id) goes to
// cand[a,m] as one 64-bit word whose unsigned order is (score ascending,
// candidate id descending): the maximum is the best score and, among equal
// scores, the smallest (a, m, b).
// k_round_commit: one workgroup.  Takes the maximum over cand, assigns the
// chosen requests, clears their pending flags, appends the decision to the
// log and advances the clock.
#pragma once
#include "sp_common.h"

namespace sp {

constexpr int kRoundThreads = 256;
constexpr int kScanSpan = 16 * kRoundThreads;   // positions looked at per scan step

__device__ __forceinline__ unsigned long long pack_candidate(float score, uint32_t cand_id) {
  return ((unsigned long long)__float_as_uint(score) << 32) | (unsigned long long)(0xFFFFFFFFu - cand_id);
}

__device__ __forceinline__ unsigned long long block_max_u64(unsigned long long v, unsigned long long* scratch) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const unsigned long long other = __shfl_xor(v, o);
    v = other > v ? other : v;
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  __syncthreads();
  if (lane == 0) scratch[wave] = v;
  __syncthreads();
  unsigned long long r = scratch[0];
  for (int i = 1; i < (int)(blockDim.x >> 6); ++i) r = scratch[i] > r ? scratch[i] : r;
  return r;
}

__global__ __launch_bounds__(kRoundThreads) void k_round_score(Tables tb, Window w, float* __restrict__ cube_out) {
  __shared__ int32_t win[kMaxBatch];
  __shared__ float aj[kMaxBatch], Dj[kMaxBatch], invDj[kMaxBatch];
  __shared__ int32_t wave_cnt[kRoundThreads / 64];
  __shared__ unsigned long long red[kRoundThreads / 64];
  const State* st = w.st;
  if (st->done || st->err) return;
  const int a = blockIdx.x / tb.Mmax, m = blockIdx.x % tb.Mmax;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int M = tb.n_models[a], B = tb.B;
  if (m >= M) {
    if (tid == 0) w.cand[blockIdx.x] = 0ull;
    return;
  }
  const int r = st->round;
  const double t = st->t;
  const int kind = tb.penalty[a];
  const double E0 = t + (double)tb.lmin[a];
  const int seg_e = w.seg[a + 1];
  const int head = w.head[(r & 1) * tb.A + a];

  // ---- candidate window: first B live requests in service order ----
  // Each step looks at kScanSpan consecutive positions, 16 per thread (one 16-byte load of pending flags,
  // four of deadlines), so that even an application whose queue is almost entirely dead is walked in
  // a handful of dependent memory round trips.
  int found = 0;
  for (int base = head & ~15; base < seg_e && found < B; base += kScanSpan) {
    const int p0 = base + 16 * tid;
    uint32_t mask = 0;
    if (p0 < seg_e) {                                  // D_s and alive_s are padded by 16 entries: always whole vectors
      const uint4 al = *reinterpret_cast<const uint4*>(w.alive_s + p0);
      const uint32_t alw[4] = {al.x, al.y, al.z, al.w};
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const float4 dv = *reinterpret_cast<const float4*>(w.D_s + p0 + 4 * q);
        const float dd[4] = {dv.x, dv.y, dv.z, dv.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int pos = p0 + 4 * q + j;
          const bool live = ((alw[q] >> (8 * j)) & 0xffu) != 0 && !is_dead(kind, dd[j], E0) && pos >= head && pos < seg_e;
          mask |= live ? (1u << (4 * q + j)) : 0u;
        }
      }
    }
    // exclusive prefix of the per-thread counts over the workgroup
    const int cnt = __popc(mask);
    int incl = cnt;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int up = __shfl_up(incl, o);
      if (lane >= o) incl += up;
    }
    if (lane == 63) wave_cnt[wave] = incl;
    __syncthreads();
    int before = found, total = found;
    for (int i = 0; i < kRoundThreads / 64; ++i) {
      if (i < wave) before += wave_cnt[i];
      total += wave_cnt[i];
    }
    int rank = before + incl - cnt;
    uint32_t mk = mask;
    while (mk != 0 && rank < B) {
      const int j = __ffs((int)mk) - 1;
      mk &= mk - 1;
      win[rank++] = p0 + j;
    }
    found = total;
    __syncthreads();
  }
  const int nb = min(found, B);
  if (m == 0) {
    for (int j = tid; j < nb; j += kRoundThreads) w.win_pos[a * B + j] = win[j];
    if (tid == 0) {
      w.win_n[a] = nb;
      w.head[((r + 1) & 1) * tb.A + a] = nb > 0 ? win[0] : seg_e;
    }
  }
  if (nb == 0) {
    if (tid == 0) w.cand[blockIdx.x] = 0ull;
    return;
  }
  for (int j = tid; j < nb; j += kRoundThreads) {
    const int pos = win[j];
    const float D = w.D_s[pos];
    aj[j] = w.key_s[pos] * w.ea[(int64_t)w.id_s[pos] * tb.Mmax + m];
    Dj[j] = D;
    invDj[j] = 1.0f / D;
  }
  __syncthreads();

  // ---- triangle: groups of 4 lanes own the batch sizes (p+1, B-p) ----
  const float* lat = tb.lat + ((int64_t)a * tb.Mmax + m) * B;
  const int sub = tid & 3, grp = tid >> 2;
  const int n_pairs = (B + 1) / 2;
  unsigned long long best = 0ull;
  for (int p = grp; p < n_pairs; p += kRoundThreads / 4) {
    for (int side = 0; side < 2; ++side) {
      const int b = side == 0 ? p + 1 : B - p;
      if (side == 1 && b == p + 1) break;          // middle batch size of an odd B
      float s = 0.f;
      if (b <= nb) {
        const double E = t + (double)lat[b - 1];
        for (int j = sub; j < b; j += 4) s += aj[j] * one_minus_penalty(kind, Dj[j], invDj[j], E);
      }
      s += __shfl_xor(s, 1);
      s += __shfl_xor(s, 2);
      if (b <= nb && sub == 0) {
        const uint32_t cid = (uint32_t)((a * tb.Mmax + m) * B + (b - 1));
        const unsigned long long pk = pack_candidate(s, cid);
        best = pk > best ? pk : best;
        if (cube_out) cube_out[cid] = s;
      }
    }
  }
  best = block_max_u64(best, red);
  if (tid == 0) w.cand[blockIdx.x] = best;
}

__device__ __forceinline__ double block_sum_f64(double v, double* scratch) {
  // fixed-order tree: the result does not depend on scheduling
  __syncthreads();
  scratch[threadIdx.x] = v;
  __syncthreads();
  for (int o = kRoundThreads / 2; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) scratch[threadIdx.x] += scratch[threadIdx.x + o];
    __syncthreads();
  }
  return scratch[0];
}

__global__ __launch_bounds__(kRoundThreads) void k_round_commit(Tables tb, Window w, int32_t* __restrict__ ids_out) {
  __shared__ unsigned long long red[kRoundThreads / 64];
  __shared__ double dsum[kRoundThreads];
  State* st = w.st;
  if (st->done || st->err) return;
  const int tid = threadIdx.x;
  unsigned long long best = 0ull;
  const int n_cand = tb.A * tb.Mmax;
  for (int i = tid; i < n_cand; i += kRoundThreads) {
    const unsigned long long c = w.cand[i];
    best = c > best ? c : best;
  }
  best = block_max_u64(best, red);
  if (best == 0ull) {                 // nothing live anywhere
    if (tid == 0) st->done = 1;
    return;
  }
  const uint32_t cid = 0xFFFFFFFFu - (uint32_t)(best & 0xFFFFFFFFull);
  const float score = __uint_as_float((uint32_t)(best >> 32));
  const int B = tb.B;
  const int b = (int)(cid % (uint32_t)B) + 1;
  const int am = (int)(cid / (uint32_t)B);
  const int m = am % tb.Mmax, a = am / tb.Mmax;
  const int kind = tb.penalty[a];
  const int r = st->round;
  const double t = st->t;
  const int next_order = st->next_order;
  const double E = t + (double)tb.lat[((int64_t)a * tb.Mmax + m) * B + (b - 1)];
  double wu = 0.0, su = 0.0, viol = 0.0;
  for (int j = tid; j < b; j += kRoundThreads) {
    const int pos = w.win_pos[a * B + j];
    const int id = w.id_s[pos];
    const float D = w.D_s[pos];
    const float u = w.ea[(int64_t)id * tb.Mmax + m] * one_minus_penalty(kind, D, 1.0f / D, E);
    w.model[id] = m;
    w.round_of[id] = r;
    w.order_of[id] = next_order + j;
    w.util[id] = u;
    w.alive_s[pos] = 0;
    w.last_ids[j] = id;
    if (ids_out) ids_out[j] = id;
    wu += (double)w.w_s[pos] * (double)u;
    su += (double)u;
    viol += fmax(0.0, E - (double)D);
  }
  wu = block_sum_f64(wu, dsum);
  su = block_sum_f64(su, dsum);
  viol = block_sum_f64(viol, dsum);
  if (tid == 0) {
    Decision dc;
    dc.app = a; dc.model = m; dc.batch = b; dc.round = r;
    dc.t_start = t; dc.t_end = E;
    dc.score = score; dc.batch_utility = (float)wu;
    if (r < w.log_cap) w.log[r] = dc;
    st->last = dc;
    st->t = E;
    st->round = r + 1;
    st->next_order = next_order + b;
    st->n_sched += b;
    st->total_wu += wu;
    st->total_u += su;
    st->total_viol += viol;
  }
}

// Window state at the start of a window.
__global__ void k_reset_state(State* st) {
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    st->t = 0.0; st->total_wu = 0.0; st->total_u = 0.0; st->total_viol = 0.0;
    st->round = 0; st->next_order = 1; st->n_sched = 0; st->done = 0; st->err = 0u; st->pad = 0;
  }
}

__global__ void k_fill_f32(float* p, int64_t n, float v) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

}  // namespace sp
