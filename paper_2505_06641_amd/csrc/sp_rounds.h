// One greedy batch-selection round as two kernels (Alg. 1 generalised to batch-capped rounds; eq. (2)
// utility; eq. (13) arg max; eq. (1) clock with the batch as the unit), and the device functions that the
// one-launch rounds kernel shares with them (triangle_best, commit_members, start_time, ...).
//
// A group is what a round iterates over: an application, or (Sec. 5.3.2) one of its subgroups.
// k_round_score: one workgroup per (group, variant).  It walks the group's service order from the head
// pointer, keeps the first B live requests (pending, and penalty on the earliest possible completion
// below 1) as the candidate window, and evaluates
//   Score[g,m,b] = sum_{j<=b} key_j * EA[j,m] * (1 - gamma_a(D_j, t + L[a][m][b]))
// for every b, pairing batch sizes b and B+1-b on the same lanes so that all lanes do the same amount
// of work.  Its best (score, candidate id) goes to cand[g,m] as one 64-bit word whose unsigned order is
// (score ascending, candidate id descending): the maximum is the best score and, among equal scores,
// the smallest (g, m, b).  The policy knobs of Sec. 6.1 change what is summed (weights, penalty used
// for the comparison), which batch sizes are candidates, and how the maximum is taken (group first).
// k_round_commit: one workgroup.  Takes the maximum over cand, assigns the chosen requests, clears their
// pending flags, appends the decision to the log and advances the clock.
#pragma once
#include "sp_common.h"
#include "sp_wave.h"

namespace sp {

constexpr int kRoundThreads = 512;
constexpr int kSmallGroup = 256;                  // remaining range up to which one wavefront scores a subgroup
// Lanes that share one pair of batch sizes in the triangle: 8 when the largest batch gives every group of 8
// lanes of a 512-thread workgroup a pair (more than 64 requests), else 16, so that half the workgroup does not
// sit idle.  A function of the largest batch alone: every kernel sums a score over the same lanes in the same
// order, whatever the number of threads it brings.
__device__ __forceinline__ int pair_lanes(int B) { return B > 64 ? 8 : 16; }

// nthr: the threads of the workgroup that are still running (a power of two; the others have left).
__device__ __forceinline__ double block_sum_f64(double v, double* scratch, int nthr = kRoundThreads) {
  // fixed-order tree: the result does not depend on scheduling
  __syncthreads();
  scratch[threadIdx.x] = v;
  __syncthreads();
  for (int o = nthr / 2; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) scratch[threadIdx.x] += scratch[threadIdx.x + o];
    __syncthreads();
  }
  return scratch[0];
}

// When a batch on variant m of application a starts computing: now, plus the variant's swap-in cost
// unless the previous batch of the window ran the same variant (Sec. 3.1 "context switch time";
// Sec. 5.2 model locality).  prev.app is -1 before the first batch.
__device__ __forceinline__ double start_time(const Tables& tb, const Decision& prev, double t, int a, int m) {
  return (prev.app == a && prev.model == m) ? t : t + (double)tb.swap[a * tb.Mmax + m];
}

__device__ __forceinline__ unsigned long long pack_candidate(float score, uint32_t cand_id) {
  return ((unsigned long long)__float_as_uint(score) << 32) | (unsigned long long)(0xFFFFFFFFu - cand_id);
}

__device__ __forceinline__ unsigned long long block_max_u64(unsigned long long v, unsigned long long* scratch,
                                                           int nwaves = 0 /* 0: the whole workgroup */) {
  v = wave_max_u64(v);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  __syncthreads();
  if (lane == 0) scratch[wave] = v;
  __syncthreads();
  unsigned long long r = scratch[0];
  if (nwaves == 0) nwaves = (int)(blockDim.x >> 6);
  for (int i = 1; i < nwaves; ++i) r = scratch[i] > r ? scratch[i] : r;
  return r;
}

// Score[a,m,b] for every batch size b over a candidate window of nb entries, and the best of them as a
// packed candidate.  ent[j] = (key_j * EA[j,m], D_j, 1/D_j, 2 D_j); lat[b-1] = L[a][m][b].
// Groups of kPairLanes = pair_lanes(B) lanes own the batch sizes (p+1, B-p), so all groups do the same amount of work;
// both batch sizes of a pair run in the same loop (two independent chains per lane), and the completion
// time of each batch size is carried as a float pair so that the loop stays in float32.
// Every kernel that scores rounds calls this function: their scores agree bit for bit.
template <int KIND, int kPairLanes>
__device__ __forceinline__ unsigned long long triangle_best_kind(const float4* ent, const float* lat, int nb, int B,
                                                                double t, uint32_t cid0, float* cube_out, int only_b,
                                                                int nthr, int tid) {
  static_assert(kPairLanes == 8 || kPairLanes == 16, "the sums below add over groups of 8 or 16 lanes");
  const int sub = tid % kPairLanes, grp = tid / kPairLanes;
  const int n_pairs = (B + 1) / 2;
  unsigned long long best = 0ull;
  for (int p = grp; p < n_pairs; p += nthr / kPairLanes) {
    const int b1 = p + 1, b2 = B - p;                 // b1 <= b2; equal for the middle size of an odd B
    const double E1 = t + (double)lat[b1 - 1], E2 = t + (double)lat[b2 - 1];
    const float e1h = (float)E1, e1l = (float)(E1 - (double)e1h);
    const float e2h = (float)E2, e2l = (float)(E2 - (double)e2h);
    // only_b > 0: that batch size alone is a candidate ("the group runs whole")
    const int n1 = (b1 <= nb && (only_b == 0 || b1 == only_b)) ? b1 : 0;
    const int n2 = (b2 <= nb && b2 != b1 && (only_b == 0 || b2 == only_b)) ? b2 : 0;
    float s1 = 0.f, s2 = 0.f, s3 = 0.f;
    int j = sub;
    for (; j < n1 && j < n2; j += kPairLanes) {                 // both batch sizes use request j
      const float4 e = ent[j];
      s1 += e.x * one_minus_penalty_f32<KIND>(e.y, e.w, e.z, e1h, e1l);
      s2 += e.x * one_minus_penalty_f32<KIND>(e.y, e.w, e.z, e2h, e2l);
    }
    for (; j < n1; j += kPairLanes) {
      const float4 e = ent[j];
      s1 += e.x * one_minus_penalty_f32<KIND>(e.y, e.w, e.z, e1h, e1l);
    }
    for (; j + kPairLanes < n2; j += 2 * kPairLanes) {          // only the larger one: two requests per trip
      const float4 e = ent[j], f = ent[j + kPairLanes];
      s2 += e.x * one_minus_penalty_f32<KIND>(e.y, e.w, e.z, e2h, e2l);
      s3 += f.x * one_minus_penalty_f32<KIND>(f.y, f.w, f.z, e2h, e2l);
    }
    if (j < n2) {
      const float4 e = ent[j];
      s2 += e.x * one_minus_penalty_f32<KIND>(e.y, e.w, e.z, e2h, e2l);
    }
    s2 += s3;
    s1 = kPairLanes == 8 ? sum8(s1) : sum16(s1);
    s2 = kPairLanes == 8 ? sum8(s2) : sum16(s2);
    if (sub == 0) {
      if (n1 > 0) {
        const unsigned long long pk = pack_candidate(s1, cid0 + (uint32_t)(b1 - 1));
        best = pk > best ? pk : best;
        if (cube_out) cube_out[cid0 + b1 - 1] = s1;
      }
      if (n2 > 0) {
        const unsigned long long pk = pack_candidate(s2, cid0 + (uint32_t)(b2 - 1));
        best = pk > best ? pk : best;
        if (cube_out) cube_out[cid0 + b2 - 1] = s2;
      }
    }
  }
  return best;
}

// nthr: the threads taking part (a multiple of 64), numbered tid = 0 .. nthr - 1 (by default the first nthr
// threads of the workgroup; a single wavefront passes its lane number).  A score is summed by the same
// pair_lanes(B) lanes in the same order however many take part, so the result does not depend on it.
__device__ __forceinline__ unsigned long long triangle_best(int kind, const float4* ent, const float* lat, int nb, int B,
                                                           double t, uint32_t cid0, float* cube_out, int only_b,
                                                           int nthr = kRoundThreads, int tid = -1) {
  if (tid < 0) tid = threadIdx.x;
  if (pair_lanes(B) == 8) {
    if (kind == 0) return triangle_best_kind<0, 8>(ent, lat, nb, B, t, cid0, cube_out, only_b, nthr, tid);
    if (kind == 1) return triangle_best_kind<1, 8>(ent, lat, nb, B, t, cid0, cube_out, only_b, nthr, tid);
    return triangle_best_kind<2, 8>(ent, lat, nb, B, t, cid0, cube_out, only_b, nthr, tid);
  }
  if (kind == 0) return triangle_best_kind<0, 16>(ent, lat, nb, B, t, cid0, cube_out, only_b, nthr, tid);
  if (kind == 1) return triangle_best_kind<1, 16>(ent, lat, nb, B, t, cid0, cube_out, only_b, nthr, tid);
  return triangle_best_kind<2, 16>(ent, lat, nb, B, t, cid0, cube_out, only_b, nthr, tid);
}

// Utility evaluations (terms key * EA * (1 - penalty)) behind the candidates of one (group, variant) pair
// over a window of nb requests: every batch size b sums its first b requests, or only the whole window does.
__device__ __forceinline__ unsigned long long triangle_evals(int nb, int whole) {
  return whole ? (unsigned long long)nb : (unsigned long long)nb * (unsigned long long)(nb + 1) / 2ull;
}

// Penalty kind the candidates of application a are compared under: its own (eq. 13), or the step penalty
// when variants are compared by accuracy among those that meet the deadline (Sec. 6.1 "Max Accuracy").
__device__ __forceinline__ int scoring_penalty(const Tables& tb, int kind) { return tb.pol_max_accuracy ? 0 : kind; }

// What orders the requests of an application and what a group's priority averages (eq. 14): the key of
// eq. (12), or the negated deadline (earliest deadline first).
__device__ __forceinline__ float ordering_value(const Tables& tb, const Window& w, int pos) {
  return tb.pol_edf ? -w.D_s[pos] : w.key_s[pos];
}

// Order-preserving map of a float onto unsigned integers (negative values included).
__device__ __forceinline__ uint32_t ordered_bits(float v) {
  const uint32_t b = __float_as_uint(v);
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

// One window entry from the request at service position pos, for variant m.
__device__ __forceinline__ float4 window_entry(const Tables& tb, const Window& w, int pos, int m) {
  const float D = w.D_s[pos];
  const float wgt = tb.pol_unit_weight ? 1.0f : w.key_s[pos];
  return make_float4(wgt * w.ea[(int64_t)w.id_s[pos] * tb.Mmax + m], D, 1.0f / D, 2.0f * D);
}

__global__ __launch_bounds__(kRoundThreads) void k_round_score(Tables tb, Window w, float* __restrict__ cube_out) {
  __shared__ int32_t win[kMaxBatch];
  __shared__ float4 ent[kMaxBatch];
  __shared__ int32_t wave_cnt[kRoundThreads / 64];
  __shared__ unsigned long long red[kRoundThreads / 64];
  __shared__ double dsum[kRoundThreads];
  State* st = w.st;
  if (st->done || st->err) return;
  const int grp = blockIdx.x / tb.Mmax, m = blockIdx.x % tb.Mmax;   // group: an application, or one of its subgroups
  if (grp >= *w.grp_n) return;
  const int a = w.grp_app[grp];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int M = tb.n_models[a], B = tb.B, Bw = tb.Bcap;   // B: row stride of the tables; Bw: largest batch
  if (m >= M) {
    if (tid == 0) w.cand[blockIdx.x] = 0ull;
    return;
  }
  const int r = st->round;
  const double t = st->t;
  const int kind = tb.penalty[a];
  const double E0 = t + (double)tb.lmin[a];
  const int seg_e = w.grp_end[grp];
  const int head = w.head[(r & 1) * w.gcap + grp];
  // With the requests split into subgroups (Sec. 5.3.2) most groups hold a handful of requests: one
  // wavefront then does the whole workgroup's job and the others leave (a barrier counts only the
  // wavefronts that are still running).
  const int nthr = (tb.pol_split && seg_e - head <= kSmallGroup) ? 64 : kRoundThreads;
  if (tid >= nthr) return;

  // ---- candidate window: first B live requests in service order ----
  // The first step looks at 4 positions per thread (1024 per workgroup, enough while most of the queue
  // is live), later steps at 16 per thread, so that even an application whose queue is almost entirely
  // dead is walked in a handful of dependent memory round trips.  D_s and alive_s are padded by 16
  // entries, so whole vectors can always be loaded.
  int found = 0;
  int base = head & ~3;
  for (int step = 0; base < seg_e && found < Bw; ++step) {
    const int nq = step == 0 ? 1 : 4;                  // groups of 4 positions per thread
    const int p0 = base + 4 * nq * tid;
    uint32_t mask = 0;
    if (p0 < seg_e) {
      for (int q = 0; q < nq; ++q) {
        const uint32_t alw = *reinterpret_cast<const uint32_t*>(w.alive_s + p0 + 4 * q);
        const float4 dv = *reinterpret_cast<const float4*>(w.D_s + p0 + 4 * q);
        const float dd[4] = {dv.x, dv.y, dv.z, dv.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int pos = p0 + 4 * q + j;
          const bool live = ((alw >> (8 * j)) & 0xffu) != 0 && !is_dead(kind, dd[j], E0) && pos >= head && pos < seg_e;
          mask |= live ? (1u << (4 * q + j)) : 0u;
        }
      }
    }
    // exclusive prefix of the per-thread counts over the workgroup
    const int cnt = __popc(mask);
    const int incl = (int)wave_scan_incl((uint32_t)cnt);
    if (lane == 63) wave_cnt[wave] = incl;
    __syncthreads();
    int before = found, total = found;
    for (int i = 0; i < nthr / 64; ++i) {
      if (i < wave) before += wave_cnt[i];
      total += wave_cnt[i];
    }
    int rank = before + incl - cnt;
    uint32_t mk = mask;
    while (mk != 0 && rank < Bw) {
      const int j = __ffs((int)mk) - 1;
      mk &= mk - 1;
      win[rank++] = p0 + j;
    }
    found = total;
    base += 4 * nq * nthr;
    __syncthreads();
  }
  const int nb = min(found, Bw);
  if (m == 0) {
    for (int j = tid; j < nb; j += nthr) w.win_pos[grp * B + j] = win[j];
    if (tid == 0) {
      w.win_n[grp] = nb;
      w.head[((r + 1) & 1) * w.gcap + grp] = nb > 0 ? win[0] : seg_e;
    }
  }
  if (nb == 0) {
    if (tid == 0) w.cand[blockIdx.x] = 0ull;
    return;
  }
  for (int j = tid; j < nb; j += nthr) ent[j] = window_entry(tb, w, win[j], m);
  if (tid == 0) atomicAdd(&st->n_evals, triangle_evals(nb, tb.pol_whole));
  __syncthreads();
  const float* lat = tb.lat + ((int64_t)a * tb.Mmax + m) * B;
  const double t0 = start_time(tb, st->last, t, a, m);
  unsigned long long best = triangle_best(scoring_penalty(tb, kind), ent, lat, nb, Bw, t0,
                                          (uint32_t)((grp * tb.Mmax + m) * B), cube_out, tb.pol_whole ? nb : 0, nthr);
  if (tb.pol_group_first) {
    // the group's priority (eq. 14) over the window; the same fixed-order sum in every kernel that forms it
    double part = 0.0;                                   // one term per thread when the whole workgroup runs
    for (int j = tid; j < nb; j += nthr) part += (double)ordering_value(tb, w, win[j]);
    const double ps = block_sum_f64(part, dsum, nthr);
    if (tid == 0) w.cand_prio[blockIdx.x] = (float)(ps / (double)nb);
  }
  best = block_max_u64(best, red, nthr / 64);
  if (tid == 0) w.cand[blockIdx.x] = best;
}

// Members of one batch: outputs, pending flags and the three sums.  pos_of(j) gives the service position
// of the j-th member.  All threads of the workgroup call it; the sums come back on every thread.
template <class PosFn>
__device__ __forceinline__ void commit_members(const Tables& tb, const Window& w, int a, int m, int b, int r,
                                               int next_order, double E, PosFn pos_of, int32_t* ids_out,
                                               double* dsum, double& wu, double& su, double& viol) {
  const int kind = tb.penalty[a];
  wu = 0.0; su = 0.0; viol = 0.0;
  for (int j = threadIdx.x; j < b; j += kRoundThreads) {
    const int pos = pos_of(j);
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
}

// The window state as the host will read it after this kernel: written straight into pinned host memory by
// the one thread that owns the state, so that a round per call needs no copy behind the kernel.
__device__ __forceinline__ void mirror_state(const Window& w) {
  if (w.st_host == nullptr) return;
  const unsigned long long* src = reinterpret_cast<const unsigned long long*>(w.st);
  unsigned long long* dst = reinterpret_cast<unsigned long long*>(w.st_host);
  static_assert(sizeof(State) % 8 == 0, "State is copied in 8-byte words");
#pragma unroll
  for (int i = 0; i < (int)(sizeof(State) / 8); ++i) dst[i] = src[i];
}

__global__ __launch_bounds__(kRoundThreads) void k_round_commit(Tables tb, Window w, int32_t* __restrict__ ids_out) {
  __shared__ unsigned long long red[kRoundThreads / 64];
  __shared__ double dsum[kRoundThreads];
  State* st = w.st;
  const int tid = threadIdx.x;
  if (st->done || st->err) {
    if (tid == 0) mirror_state(w);
    return;
  }
  unsigned long long best = 0ull;
  const int n_cand = *w.grp_n * tb.Mmax;
  for (int i = tid; i < n_cand; i += kRoundThreads) {
    const unsigned long long c = w.cand[i];
    best = c > best ? c : best;
  }
  best = block_max_u64(best, red);
  if (best == 0ull) {                 // nothing live anywhere
    if (tid == 0) {
      st->done = 1;
      mirror_state(w);
    }
    return;
  }
  if (tb.pol_group_first) {
    // Alg. 1: first the application with the highest group priority (ties: the smallest application),
    // then the best candidate of that application alone
    unsigned long long top = 0ull;
    for (int i = tid; i < n_cand; i += kRoundThreads)
      if (w.cand[i] != 0ull) {
        const unsigned long long pk = ((unsigned long long)ordered_bits(w.cand_prio[i]) << 32) |
                                      (unsigned long long)(0xFFFFFFFFu - (uint32_t)(i / tb.Mmax));
        top = pk > top ? pk : top;
      }
    top = block_max_u64(top, red);
    const int g_star = (int)(0xFFFFFFFFu - (uint32_t)(top & 0xFFFFFFFFull));
    best = 0ull;
    for (int i = g_star * tb.Mmax + tid; i < (g_star + 1) * tb.Mmax; i += kRoundThreads) {
      const unsigned long long c = w.cand[i];
      best = c > best ? c : best;
    }
    best = block_max_u64(best, red);
  }
  const uint32_t cid = 0xFFFFFFFFu - (uint32_t)(best & 0xFFFFFFFFull);
  const float score = __uint_as_float((uint32_t)(best >> 32));
  const int B = tb.B;
  const int b = (int)(cid % (uint32_t)B) + 1;
  const int am = (int)(cid / (uint32_t)B);
  const int m = am % tb.Mmax, grp = am / tb.Mmax;
  const int a = w.grp_app[grp];
  const int r = st->round;
  const double t = st->t;
  const int next_order = st->next_order;
  const double E = start_time(tb, st->last, t, a, m) + (double)tb.lat[((int64_t)a * tb.Mmax + m) * B + (b - 1)];
  double wu, su, viol;
  const int32_t* row = w.win_pos + grp * B;
  commit_members(tb, w, a, m, b, r, next_order, E, [&](int j) { return row[j]; }, ids_out, dsum, wu, su, viol);
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
    mirror_state(w);
  }
}

// Window state at the start of a window, and the one-segment plan of the pass over the application ids.
__global__ void k_reset_state(State* st, int n, int32_t* seg1, uint32_t* dtot_app, int dtot_words) {
  for (int i = threadIdx.x; i < dtot_words; i += blockDim.x) dtot_app[i] = 0u;    // digit totals of the pass(es) over the application ids
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    seg1[0] = 0;
    seg1[1] = n;
    st->t = 0.0; st->total_wu = 0.0; st->total_u = 0.0; st->total_viol = 0.0;
    st->round = 0; st->next_order = 1; st->n_sched = 0; st->done = 0; st->err = 0u; st->pad = 0;
    st->n_evals = 0ull;
    st->last.app = -1; st->last.model = -1;      // nothing resident yet
  }
}

__global__ void k_fill_f32(float* p, int64_t n, float v) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

}  // namespace sp
