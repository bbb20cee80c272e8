// All greedy rounds of a chunk in one launch (Alg. 1 generalised to batch-capped rounds; eq. (2),
// eq. (13), eq. (1) as in sp_rounds.h, which this kernel reproduces decision for decision).
//
// One workgroup per (application, variant) pair stays resident for the whole chunk; two more take the
// maximum over the pairs and do the commits.  What a round costs on the two-kernel path is mostly latency: two kernel
// boundaries, the walk over the service order and the gathers behind it.  Here
//   * each pair keeps its application's candidate window in LDS between rounds, with look-ahead entries
//     behind it (kWinCap in all).  A round removes the entries the previous decision consumed (always a
//     prefix: the greedy takes the first b live requests) and those whose penalty has reached 1 at the
//     new clock (they never come back: the clock only advances).  The walk over the service order that
//     refills the look-ahead runs one step per round while the candidates are being exchanged; a round
//     waits for it only when fewer than B entries remain while the application still has unvisited
//     requests.  Every position of the service order is visited once per launch, not once per round;
//   * the arg max over all pairs goes through one slot per pair and a reducing workgroup: every pair
//     publishes its best candidate, the reducer polls the slots (one per thread), takes the maximum and
//     publishes the decision, which one thread of every pair polls.  With few pairs (kAllToAllPairs) there
//     is no reducer: every pair polls all slots itself and takes the maximum, which halves the trips
//     through the fabric between a round's last candidate and its decision (the decisions are the same:
//     every pair applies the reducer's rule to the same words; pair 0 passes the decision on to the commit
//     workgroup).  Slots and the decision are pairs of
//     64-bit words, each carrying the generation number of the round it belongs to, written and polled
//     with relaxed device-scope atomics: a word is valid exactly when its generation matches, so no
//     fence is needed and a stale value can never be mistaken for the current one.  Both are double
//     buffered by generation parity (nobody can be more than one round ahead of anybody else: the
//     reducer needs every pair's slot of a round, every pair needs the reducer's decision of it);
//   * clock, round counter and window shifts follow from the decision and are replicated in every pair;
//   * the commit workgroup receives each decision through a ring entry, and the members of the chosen
//     batch through a ring of generation-tagged window positions written by the chosen application's
//     first pair, so the commits (outputs, totals, decision log) run beside the next round's scoring.
// With data-aware subgroups (Sec. 5.3.2) a pair serves every group of its application: the largest one
// (the "primary") keeps the LDS-resident window described above; the others are walked afresh every round,
// one wavefront per group (they are small: a handful of requests behind a head pointer kept in LDS), before
// the primary's block-wide work; the pair publishes the best candidate over its groups together with the
// group's index.  The chosen batch's positions reach the commit workgroup after the decision: the chosen
// application's first pair writes them into the ring (from the primary's window, or from one more walk of
// the chosen secondary group, which every pair of that application does anyway to move its head pointer).
// The workgroups wait for each other, so all of them must be resident at once: the host launches this
// kernel only when the device can hold the whole grid (occupancy query), and every wait is bounded: a
// wait that runs out (the device was shared with other long-running work) raises kErrSync, every
// workgroup leaves its loop, and the call fails instead of hanging.
#pragma once
#include "sp_rounds.h"

namespace sp {

constexpr int kWinCap = 2 * kMaxBatch;          // window + look-ahead entries, one per thread
constexpr int kPersistRounds = 64;              // rounds per launch (ring depth)
constexpr int kSpinLimit = 1 << 20;             // polls before a wait is given up (about a second)
constexpr uint32_t kGenMask = 0x7FFFFFu;        // generation bits carried in a slot's first word
constexpr int kMaxPairs = 1024;                 // (application, variant) pairs the reducer can hold
constexpr int kSlotsPerThread = kMaxPairs / kRoundThreads;
constexpr int kMaxAppGroups = 64;               // groups of one application a resident pair can serve
constexpr int kAllToAllPairs = 128;             // up to this many pairs, every pair polls every slot itself
static_assert(kWinCap <= kRoundThreads, "one window entry per thread");

struct Persist {
  const int32_t* pair_app;      // [n_pairs] application of each pair
  const int32_t* pair_model;    // [n_pairs] variant of each pair
  int32_t n_pairs;
  int32_t all_to_all;           // 1: every pair reads all pairs' slots and takes the maximum itself (no reducing workgroup)
  int32_t n_rounds;             // rounds this launch may run (<= kPersistRounds)
  int32_t spin_limit;           // polls before a wait between workgroups is given up (kSpinLimit unless a test shortens it)
  uint32_t gen_base;            // generations used by earlier launches
  unsigned long long* slots;    // [2 (parity), n_pairs, 4 (word)]
  unsigned long long* decision; // [2 (parity), 4 (word)]: latency bits << 32 | gen; (candidate id + 1, 0 = none)
                                //   << 32 | gen; swap-in cost bits << 32 | gen; unused
  unsigned long long* ring;     // [kPersistRounds, A, B]: generation << 32 | service position
  unsigned long long* dec;      // [kPersistRounds]: decision of each round, bit 63 set; zero once consumed
  long long* ticks;             // [kPersistRounds + 1]: constant-rate timestamps, launch start then each decision
};

__device__ __forceinline__ unsigned long long ld_dev(const unsigned long long* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_dev(unsigned long long* p, unsigned long long v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// slot word 0: score bits << 32 | generation (23 bits) << 9 | valid << 8 | (b - 1)
// slot word 1: latency bits of the candidate (float) << 32 | group of the candidate (16 bits) << 16 | generation (16 bits)
//              (a slot is rewritten every round, so a stale word is two generations old: 16 bits tell)
// slot word 2: swap-in cost the pair would pay in this round (float bits) << 32 | generation (32 bits)
// slot word 3: group priority of the pair's application (eq. 14; float bits) << 32 | generation (32 bits)
__device__ __forceinline__ unsigned long long slot_word0(float score, uint32_t gen, bool valid, int b) {
  return ((unsigned long long)__float_as_uint(score) << 32) | ((unsigned long long)(gen & kGenMask) << 9) |
         (valid ? 0x100ull : 0ull) | (unsigned long long)((b - 1) & 0xff);
}

__device__ void persist_commit_loop(const Tables& tb, const Window& w, const Persist& ps, double* dsum,
                                    unsigned long long* bcast) {
  State* st = w.st;
  const int tid = threadIdx.x;
  int r = st->round, next_order = st->next_order, n_sched = st->n_sched;
  double t = st->t, twu = st->total_wu, tu = st->total_u, tv = st->total_viol;
  bool done = false, failed = false, any = false;
  Decision last = st->last;                 // app -1 before the window's first batch
  for (int rl = 0; rl < ps.n_rounds; ++rl) {
    const uint32_t gen = ps.gen_base + (uint32_t)rl + 1u;
    if (tid == 0) {
      unsigned long long v = 0ull;
      for (int i = 0; i < ps.spin_limit; ++i) {
        v = ld_dev(ps.dec + rl);
        if (v != 0ull) break;
        __builtin_amdgcn_s_sleep(4);
      }
      if (v != 0ull) st_dev(ps.dec + rl, 0ull);
      bcast[0] = v;
    }
    __syncthreads();
    const unsigned long long v = bcast[0];
    __syncthreads();
    if (v == 0ull) { failed = true; break; }
    const unsigned long long best = v & ~(1ull << 63);
    if (best == 0ull) { done = true; break; }
    const uint32_t cid = 0xFFFFFFFFu - (uint32_t)(best & 0xFFFFFFFFull);
    const float score = __uint_as_float((uint32_t)(best >> 32));
    const int B = tb.B;
    const int b = (int)(cid % (uint32_t)B) + 1;
    const int am = (int)(cid / (uint32_t)B);
    const int m = am % tb.Mmax, grp = am / tb.Mmax;
    const int a = w.grp_app[grp];                     // group = application unless the requests are split into subgroups
    const double E = start_time(tb, last, t, a, m) + (double)tb.lat[((int64_t)a * tb.Mmax + m) * B + (b - 1)];
    const unsigned long long* row = ps.ring + ((size_t)rl * tb.A + a) * B;
    bool lost = false;
    double wu, su, viol;
    commit_members(tb, w, a, m, b, r, next_order, E,
                   [&](int j) {
                     unsigned long long e = 0ull;
                     for (int i = 0; i < ps.spin_limit; ++i) {
                       e = ld_dev(row + j);
                       if ((uint32_t)(e >> 32) == gen) break;
                       __builtin_amdgcn_s_sleep(4);
                     }
                     if ((uint32_t)(e >> 32) != gen) { lost = true; return 0; }   // position 0 exists: b >= 1 request
                     return (int)(uint32_t)(e & 0xFFFFFFFFull);
                   },
                   nullptr, dsum, wu, su, viol);
    if (__syncthreads_or(lost ? 1 : 0)) { failed = true; break; }
    last.app = a; last.model = m; last.batch = b; last.round = r;
    last.t_start = t; last.t_end = E; last.score = score; last.batch_utility = (float)wu;
    any = true;
    if (tid == 0 && r < w.log_cap) w.log[r] = last;
    t = E; r += 1; next_order += b; n_sched += b;
    twu += wu; tu += su; tv += viol;
  }
  if (tid == 0) {
    st->t = t; st->round = r; st->next_order = next_order; st->n_sched = n_sched;
    st->total_wu = twu; st->total_u = tu; st->total_viol = tv;
    if (any) st->last = last;
    if (done) st->done = 1;
    if (failed) atomicOr(&st->err, kErrSync);
  }
}

// The reducing workgroup: maximum over the pairs' slots of every round, published as the decision.
__device__ void persist_reduce_loop(const Tables& tb, const Window& w, const Persist& ps, unsigned long long* red,
                                    float* lat_win, float* swap_win, int* timed_out) {
  const int tid = threadIdx.x;
  const int B = tb.B;
  if (ps.all_to_all) return;                      // every pair takes the maximum itself
  const int my_slot = tid < ps.n_pairs ? tid : 0;
  const int my_m = ps.pair_model[my_slot];
  if (tid == 0) {
    *timed_out = 0;
    ps.ticks[0] = wall_clock64();
  }
  __syncthreads();
  for (int rl = 0; rl < ps.n_rounds; ++rl) {
    const uint32_t gen = ps.gen_base + (uint32_t)rl + 1u;
    unsigned long long mine = 0ull;
    float mine_lat = 0.f, mine_swap = 0.f;
    // with the group-first rule the slots are read once and compared twice: group priorities, then the
    // candidates of the winning application (a thread holds at most kSlotsPerThread slots)
    unsigned long long held[kSlotsPerThread];
    float held_lat[kSlotsPerThread], held_swap[kSlotsPerThread];
    unsigned long long top = 0ull;
#pragma unroll
    for (int q = 0; q < kSlotsPerThread; ++q) {
      held[q] = 0ull;
      const int i = tid + q * kRoundThreads;
      if (i >= ps.n_pairs) continue;
      const unsigned long long* slot = ps.slots + ((size_t)(gen & 1u) * ps.n_pairs + i) * 4;
      unsigned long long v0 = 0ull, v1 = 0ull, v2 = 0ull, v3 = 0ull;
      bool ok = false;
      for (int k = 0; k < ps.spin_limit; ++k) {
        v0 = ld_dev(slot);
        v1 = ld_dev(slot + 1);
        v2 = ld_dev(slot + 2);
        v3 = ld_dev(slot + 3);
        ok = ((uint32_t)(v0 >> 9) & kGenMask) == (gen & kGenMask) && (uint32_t)(v1 & 0xFFFFull) == (gen & 0xFFFFu) &&
             (uint32_t)(v2 & 0xFFFFFFFFull) == gen && (uint32_t)(v3 & 0xFFFFFFFFull) == gen;
        if (ok) break;
        __builtin_amdgcn_s_sleep(1);
      }
      if (!ok) {
        *timed_out = 1;
      } else if (v0 & 0x100ull) {
        const int pm = q == 0 ? my_m : ps.pair_model[i];
        const int pg = (int)((uint32_t)(v1 >> 16) & 0xFFFFu);      // the candidate's group (the pair's application when unsplit)
        const uint32_t cid = (uint32_t)((pg * tb.Mmax + pm) * B) + (uint32_t)(v0 & 0xffull);
        const unsigned long long pk = pack_candidate(__uint_as_float((uint32_t)(v0 >> 32)), cid);
        held[q] = pk;
        held_lat[q] = __uint_as_float((uint32_t)(v1 >> 32));
        held_swap[q] = __uint_as_float((uint32_t)(v2 >> 32));
        const unsigned long long pt = ((unsigned long long)ordered_bits(__uint_as_float((uint32_t)(v3 >> 32))) << 32) |
                                      (unsigned long long)(0xFFFFFFFFu - (uint32_t)pg);
        top = pt > top ? pt : top;
      }
    }
    int a_star = -1;                                           // -1: every group competes
    if (tb.pol_group_first) {
      top = block_max_u64(top, red);
      if (top != 0ull) a_star = (int)(0xFFFFFFFFu - (uint32_t)(top & 0xFFFFFFFFull));
    }
#pragma unroll
    for (int q = 0; q < kSlotsPerThread; ++q) {
      if (held[q] == 0ull) continue;
      const uint32_t cid = 0xFFFFFFFFu - (uint32_t)(held[q] & 0xFFFFFFFFull);
      if (a_star >= 0 && (int)(cid / (uint32_t)B) / tb.Mmax != a_star) continue;
      if (held[q] > mine) { mine = held[q]; mine_lat = held_lat[q]; mine_swap = held_swap[q]; }
    }
    const unsigned long long all = block_max_u64(mine, red);
    if (all != 0ull && mine == all) {                         // candidate ids are unique: one writer
      *lat_win = mine_lat;
      *swap_win = mine_swap;
    }
    __syncthreads();
    if (*timed_out) {
      if (tid == 0) atomicOr(&w.st->err, kErrSync);
      break;
    }
    if (tid == 0) {
      unsigned long long* d = ps.decision + (size_t)(gen & 1u) * 4;
      const uint32_t cidp1 = all != 0ull ? (0xFFFFFFFFu - (uint32_t)(all & 0xFFFFFFFFull)) + 1u : 0u;
      st_dev(d, ((unsigned long long)__float_as_uint(all != 0ull ? *lat_win : 0.f) << 32) | (unsigned long long)gen);
      st_dev(d + 1, ((unsigned long long)cidp1 << 32) | (unsigned long long)gen);
      st_dev(d + 2, ((unsigned long long)__float_as_uint(all != 0ull ? *swap_win : 0.f) << 32) | (unsigned long long)gen);
      st_dev(ps.dec + rl, all | (1ull << 63));
      ps.ticks[rl + 1] = wall_clock64();
    }
    if (all == 0ull) break;                                    // nothing live anywhere
    __syncthreads();                                           // lat_win and swap_win are rewritten next round
  }
}

// The first (up to) Bw live requests of a group from position `head` on, found by one wavefront: their
// service positions go to wpos (LDS of that wavefront), the count is returned.  Same rule as the walks of
// the other round kernels: pending, and the penalty on the earliest possible completion E0 below 1.
__device__ __forceinline__ int wave_window(const Window& w, int kind, int head, int seg_e, double E0, int Bw,
                                           int32_t* wpos, int lane) {
  int found = 0;
  for (int base = head & ~3; base < seg_e && found < Bw; base += 4 * kWave) {
    const int p0 = base + 4 * lane;
    uint32_t mask = 0;
    if (p0 < seg_e) {
      const uint32_t alw = *reinterpret_cast<const uint32_t*>(w.alive_s + p0);
      const float4 dv = *reinterpret_cast<const float4*>(w.D_s + p0);
      const float dd[4] = {dv.x, dv.y, dv.z, dv.w};
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int pos = p0 + j;
        const bool live = ((alw >> (8 * j)) & 0xffu) != 0 && !is_dead(kind, dd[j], E0) && pos >= head && pos < seg_e;
        mask |= live ? (1u << j) : 0u;
      }
    }
    const int cnt = __popc(mask);
    const int incl = (int)wave_scan_incl((uint32_t)cnt);
    int rank = found + incl - cnt;
    uint32_t mk = mask;
    while (mk != 0 && rank < Bw) {
      const int j = __ffs((int)mk) - 1;
      mk &= mk - 1;
      wpos[rank++] = p0 + j;
    }
    found += __shfl(incl, kWave - 1);
  }
  wave_sync();
  return min(found, Bw);
}

// SPLIT: the window's groups are subgroups of the applications (tb.pol_split); the plain instantiation holds
// none of the secondary-group code, so that it keeps its registers (three workgroups per CU must fit).
template <bool SPLIT>
__global__ __launch_bounds__(kRoundThreads, 6) void k_rounds_persistent(Tables tb, Window w, Persist ps) {
  __shared__ int32_t win[kWinCap];
  __shared__ float4 ent[kWinCap];
  __shared__ float om[kWinCap];              // ordering value of each entry (for the group priority)
  __shared__ float lat_s[kMaxBatch];
  __shared__ int32_t wave_cnt[kRoundThreads / 64], keep_cnt[kRoundThreads / 64];
  __shared__ unsigned long long red[kRoundThreads / 64];
  __shared__ double dsum[kRoundThreads];
  __shared__ float lat_win, swap_win;
  __shared__ uint32_t cid_win;
  __shared__ int timed_out;
  __shared__ int32_t head_s[kMaxAppGroups];                     // head pointer of each group of the application
  __shared__ unsigned long long sec_best[kRoundThreads / 64], sec_top[kRoundThreads / 64];   // per wavefront: its secondary groups' best
  __shared__ float sec_prio[kRoundThreads / 64];
  extern __shared__ __align__(16) unsigned char sec_lds[];      // with subgroups: per wavefront B window entries and B positions
  State* st = w.st;
  if (st->done || st->err) return;          // the state is rewritten only when the commit workgroup ends
  if ((int)blockIdx.x >= ps.n_pairs) {
    if ((int)blockIdx.x == ps.n_pairs) persist_reduce_loop(tb, w, ps, red, &lat_win, &swap_win, &timed_out);
    if ((int)blockIdx.x == ps.n_pairs + 1) persist_commit_loop(tb, w, ps, dsum, red);
    return;
  }
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int pair = blockIdx.x;
  const int a = ps.pair_app[pair], m = ps.pair_model[pair];
  const int B = tb.B, Bw = tb.Bcap, cap = kWinCap;   // B: row stride of the tables; Bw: largest batch
  const int kind = tb.penalty[a];
  const float lmin = tb.lmin[a];
  const float my_swap = tb.swap[a * tb.Mmax + m];
  bool prev_mine = st->last.app == a;                       // the previous batch ran a variant of this application ...
  int prev_m = st->last.model;                              // ... namely this one (-1 before the window's first batch)
  int r = st->round;
  double t = st->t;
  // the groups of this application: itself, or (Sec. 5.3.2) its non-empty subgroups, consecutive in the group table
  int glo = a, ng = 1;
  if (SPLIT) {
    const int G = w.grp_n[0];
    int lo = 0, hi = G;
    while (lo < hi) {                                        // first group of an application >= a
      const int mid = (lo + hi) >> 1;
      if (w.grp_app[mid] < a) lo = mid + 1; else hi = mid;
    }
    glo = lo;
    hi = G;
    while (lo < hi) {                                        // first group of an application > a
      const int mid = (lo + hi) >> 1;
      if (w.grp_app[mid] <= a) lo = mid + 1; else hi = mid;
    }
    ng = lo - glo;
    if (ng > kMaxAppGroups) {                                // the host launches this kernel only when every application fits
      if (tid == 0) atomicOr(&st->err, kErrSync);
      ng = 0;
    }
  }
  // the primary group (largest remaining range; ties: the first) keeps the LDS-resident window
  int prim = 0, prim_size = -1;
  for (int i = 0; i < ng; ++i) {
    const int sz = w.grp_end[glo + i] - w.head[(r & 1) * w.gcap + glo + i];
    if (sz > prim_size) { prim_size = sz; prim = i; }
  }
  for (int i = tid; i < ng; i += kRoundThreads) head_s[i] = w.head[(r & 1) * w.gcap + glo + i];
  const int gprim = glo + prim;
  const int seg_e = ng > 0 ? w.grp_end[gprim] : 0;
  int scan_end = ng > 0 ? w.head[(r & 1) * w.gcap + gprim] : 0;   // everything before it is consumed or dead
  int nb = 0, shift = 0;
  unsigned long long evals = 0ull;               // utility evaluations counted by this thread (lane 0 of a wavefront)
  for (int j = tid; j < B; j += kRoundThreads) lat_s[j] = tb.lat[((int64_t)a * tb.Mmax + m) * B + j];
  if (tid == 0) {
    timed_out = 0;
    if (ps.all_to_all && pair == 0) ps.ticks[0] = wall_clock64();
  }
  const int slot_model = ps.all_to_all && tid < ps.n_pairs ? ps.pair_model[tid] : 0;   // variant behind the slot this thread polls
  float4* went = reinterpret_cast<float4*>(sec_lds) + (size_t)wave * B;
  int32_t* wpos = reinterpret_cast<int32_t*>(sec_lds + (size_t)(kRoundThreads / 64) * B * sizeof(float4)) + (size_t)wave * B;
  __syncthreads();

  for (int rl = 0; rl < ps.n_rounds; ++rl) {
    const uint32_t gen = ps.gen_base + (uint32_t)rl + 1u;
    const double E0 = t + (double)lmin;
    const float swap_now = (prev_mine && prev_m == m) ? 0.f : my_swap;

    // ---- secondary groups: one wavefront each, walked afresh from their head pointers ----
    unsigned long long wbest = 0ull, wtop = 0ull;
    float wprio = 0.f;
    if (SPLIT && ng > 1) {
      for (int i = wave; i < ng; i += kRoundThreads / 64) {
        if (i == prim) continue;
        const int g = glo + i, se = w.grp_end[g];
        const int nbs = wave_window(w, kind, head_s[i], se, E0, Bw, wpos, lane);
        if (lane == 0) head_s[i] = nbs > 0 ? wpos[0] : se;       // what lies before has been consumed or has died
        if (nbs == 0) continue;
        for (int j = lane; j < nbs; j += kWave) went[j] = window_entry(tb, w, wpos[j], m);
        wave_sync();
        if (lane == 0) evals += triangle_evals(nbs, tb.pol_whole);
        unsigned long long cand = triangle_best(scoring_penalty(tb, kind), went, lat_s, nbs, Bw, t + (double)swap_now,
                                                (uint32_t)((g * tb.Mmax + m) * B), nullptr, tb.pol_whole ? nbs : 0, kWave, lane);
        cand = wave_max_u64(cand);
        if (tb.pol_group_first) {
          // eq. (14) over the window: the fixed-order sum a single wavefront forms in k_round_score
          double part = 0.0;
          for (int j = lane; j < nbs; j += kWave) part += (double)ordering_value(tb, w, wpos[j]);
#pragma unroll
          for (int o = kWave / 2; o > 0; o >>= 1) part += __shfl_down(part, o);
          const float pr = (float)(__shfl(part, 0) / (double)nbs);
          const unsigned long long top = ((unsigned long long)ordered_bits(pr) << 32) | (unsigned long long)(0xFFFFFFFFu - (uint32_t)g);
          if (cand != 0ull && top > wtop) { wtop = top; wbest = cand; wprio = pr; }
        } else if (cand > wbest) {
          wbest = cand;
        }
        wave_sync();                                              // wpos and went are reused by the next group
      }
    }

    // ---- primary group: drop what the last decision consumed and what has died since ----
    {
      const bool has = tid < nb;
      int pos = 0;
      float4 e = make_float4(0.f, 1.f, 0.f, 0.f);
      float ov = 0.f;
      if (has) { pos = win[tid]; e = ent[tid]; ov = om[tid]; }
      const bool keep = has && tid >= shift && !is_dead(kind, e.y, E0);
      const unsigned long long bal = __ballot(keep);
      if (lane == 0) keep_cnt[wave] = __popcll(bal);
      __syncthreads();
      int before = 0, total = 0;
      for (int i = 0; i < kRoundThreads / 64; ++i) {
        const int c = keep_cnt[i];
        if (i < wave) before += c;
        total += c;
      }
      if (total != nb) {
        before += __popcll(bal & ((1ull << lane) - 1ull));
        if (keep) { win[before] = pos; ent[before] = e; om[before] = ov; }
        nb = total;
      }
      shift = 0;
      __syncthreads();
    }

    // Walks on through the service order from scan_end and appends the live requests it meets, for at
    // most max_steps steps of 4 * nq positions per thread, until the window is full or the group's
    // range ends.  Uniform over the workgroup.
    auto walk = [&](int max_steps, int first_nq) {
      const int nb_old = nb;
      for (int step = 0; step < max_steps && nb < cap && scan_end < seg_e; ++step) {
        const int nq = step == 0 ? first_nq : 4;           // groups of 4 positions per thread
        const int base = scan_end & ~3;
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
              const bool live = ((alw >> (8 * j)) & 0xffu) != 0 && !is_dead(kind, dd[j], E0) && pos >= scan_end && pos < seg_e;
              mask |= live ? (1u << (4 * q + j)) : 0u;
            }
          }
        }
        const int cnt = __popc(mask);
        const int incl = (int)wave_scan_incl((uint32_t)cnt);
        if (lane == 63) wave_cnt[wave] = incl;
        __syncthreads();
        int before = nb, total = nb;
        for (int i = 0; i < kRoundThreads / 64; ++i) {
          if (i < wave) before += wave_cnt[i];
          total += wave_cnt[i];
        }
        int rank = before + incl - cnt;
        uint32_t mk = mask;
        while (mk != 0 && rank < cap) {
          const int j = __ffs((int)mk) - 1;
          mk &= mk - 1;
          win[rank++] = p0 + j;
        }
        __syncthreads();
        if (total >= cap) {
          scan_end = win[cap - 1] + 1;                     // the rest of this step is looked at again later
          nb = cap;
        } else {
          scan_end = min(base + 4 * nq * kRoundThreads, seg_e);
          nb = total;
        }
      }
      for (int j = nb_old + tid; j < nb; j += kRoundThreads) {
        ent[j] = window_entry(tb, w, win[j], m);
        om[j] = ordering_value(tb, w, win[j]);
      }
      __syncthreads();
    };

    // ---- fewer than B entries left: the round has to wait for the walk ----
    if (nb < Bw && scan_end < seg_e) walk(1 << 30, 1);
    const int nbe = min(nb, Bw);

    // ---- the window's positions for the commit workgroup (with subgroups: after the decision) ----
    if (!SPLIT && m == 0 && tid < nbe)
      st_dev(ps.ring + ((size_t)rl * tb.A + a) * B + tid, ((unsigned long long)gen << 32) | (unsigned long long)(uint32_t)win[tid]);

    // ---- triangle: the same code as k_round_score ----
    unsigned long long best = 0ull;
    if (tid == 0) evals += triangle_evals(nbe, tb.pol_whole);
    if (nbe > 0)
      best = triangle_best(scoring_penalty(tb, kind), ent, lat_s, nbe, Bw, t + (double)swap_now,
                           (uint32_t)((gprim * tb.Mmax + m) * B), nullptr, tb.pol_whole ? nbe : 0);
    float prio = 0.f;
    if (tb.pol_group_first) {          // eq. (14) over the window, the same fixed-order sum as in k_round_score
      const double psum = block_sum_f64(tid < nbe ? (double)om[tid] : 0.0, dsum);
      prio = nbe > 0 ? (float)(psum / (double)nbe) : 0.f;
    }
    if (SPLIT && ng > 1 && lane == 0) {
      sec_best[wave] = wbest;
      sec_top[wave] = wtop;
      sec_prio[wave] = wprio;
    }
    best = block_max_u64(best, red);     // (its barriers also make the wavefronts' secondary results visible)

    // ---- publish this pair's best candidate over its groups ----
    if (tid == 0) {
      if (SPLIT && ng > 1) {
        if (tb.pol_group_first) {
          // first the group with the highest priority among those that have a candidate, then its candidate
          unsigned long long ftop = best != 0ull ? (((unsigned long long)ordered_bits(prio) << 32) |
                                                    (unsigned long long)(0xFFFFFFFFu - (uint32_t)gprim)) : 0ull;
          for (int i = 0; i < kRoundThreads / 64; ++i)
            if (sec_best[i] != 0ull && sec_top[i] > ftop) { ftop = sec_top[i]; best = sec_best[i]; prio = sec_prio[i]; }
        } else {
          for (int i = 0; i < kRoundThreads / 64; ++i) best = sec_best[i] > best ? sec_best[i] : best;
        }
      }
      unsigned long long* slot = ps.slots + ((size_t)(gen & 1u) * ps.n_pairs + pair) * 4;
      const bool valid = best != 0ull;
      const uint32_t bcid = 0xFFFFFFFFu - (uint32_t)(best & 0xFFFFFFFFull);
      const int b = valid ? (int)(bcid % (uint32_t)B) + 1 : 1;
      const uint32_t bg = valid ? (bcid / (uint32_t)B) / (uint32_t)tb.Mmax : (uint32_t)a;
      st_dev(slot + 3, ((unsigned long long)__float_as_uint(prio) << 32) | (unsigned long long)gen);
      st_dev(slot + 2, ((unsigned long long)__float_as_uint(swap_now) << 32) | (unsigned long long)gen);
      st_dev(slot + 1, ((unsigned long long)__float_as_uint(lat_s[b - 1]) << 32) | ((unsigned long long)(bg & 0xFFFFu) << 16) |
                           (unsigned long long)(gen & 0xFFFFu));
      st_dev(slot, slot_word0(__uint_as_float((uint32_t)(best >> 32)), gen, valid, b));
    }

    // ---- look-ahead: one step of the walk while the candidates are exchanged ----
    // (three dependent trips to memory, about twice the exchange: only once less than two windows are left)
    if (nb < min(2 * Bw, cap) && scan_end < seg_e) walk(1, 4);

    // ---- few pairs: the maximum over all pairs' slots, taken here (the reducer's rule on the same words) ----
    if (ps.all_to_all) {
      unsigned long long mine = 0ull, top = 0ull;
      float mine_lat = 0.f, mine_swap = 0.f;
      if (tid < ps.n_pairs) {
        const unsigned long long* slot = ps.slots + ((size_t)(gen & 1u) * ps.n_pairs + tid) * 4;
        unsigned long long v0 = 0ull, v1 = 0ull, v2 = 0ull, v3 = 0ull;
        bool ok = false;
        for (int k = 0; k < ps.spin_limit; ++k) {
          v0 = ld_dev(slot);
          v1 = ld_dev(slot + 1);
          v2 = ld_dev(slot + 2);
          v3 = ld_dev(slot + 3);
          ok = ((uint32_t)(v0 >> 9) & kGenMask) == (gen & kGenMask) && (uint32_t)(v1 & 0xFFFFull) == (gen & 0xFFFFu) &&
               (uint32_t)(v2 & 0xFFFFFFFFull) == gen && (uint32_t)(v3 & 0xFFFFFFFFull) == gen;
          if (ok) break;
          __builtin_amdgcn_s_sleep(1);
        }
        if (!ok) {
          timed_out = 1;
        } else if (v0 & 0x100ull) {
          const int pg = (int)((uint32_t)(v1 >> 16) & 0xFFFFu);
          const uint32_t c2 = (uint32_t)((pg * tb.Mmax + slot_model) * B) + (uint32_t)(v0 & 0xffull);
          mine = pack_candidate(__uint_as_float((uint32_t)(v0 >> 32)), c2);
          mine_lat = __uint_as_float((uint32_t)(v1 >> 32));
          mine_swap = __uint_as_float((uint32_t)(v2 >> 32));
          top = ((unsigned long long)ordered_bits(__uint_as_float((uint32_t)(v3 >> 32))) << 32) |
                (unsigned long long)(0xFFFFFFFFu - (uint32_t)pg);
        }
      }
      if (tb.pol_group_first) {
        top = block_max_u64(top, red);
        if (top != 0ull && mine != 0ull) {
          const int g_star = (int)(0xFFFFFFFFu - (uint32_t)(top & 0xFFFFFFFFull));
          const uint32_t c2 = 0xFFFFFFFFu - (uint32_t)(mine & 0xFFFFFFFFull);
          if ((int)(c2 / (uint32_t)B) / tb.Mmax != g_star) mine = 0ull;
        }
      }
      const unsigned long long all = block_max_u64(mine, red);
      if (all != 0ull && mine == all) {                          // candidate ids are unique: one writer
        lat_win = mine_lat;
        swap_win = mine_swap;
      }
      if (tid == 0) {
        cid_win = all != 0ull ? (0xFFFFFFFFu - (uint32_t)(all & 0xFFFFFFFFull)) + 1u : 0u;
        if (pair == 0) {                                         // for the commit workgroup, and the round's timestamp
          st_dev(ps.dec + rl, all | (1ull << 63));
          ps.ticks[rl + 1] = wall_clock64();
        }
      }
    } else if (tid == 0) {
      // ---- wait for the decision ----
      const unsigned long long* d = ps.decision + (size_t)(gen & 1u) * 4;
      unsigned long long v0 = 0ull, v1 = 0ull, v2 = 0ull;
      bool ok = false;
      for (int k = 0; k < ps.spin_limit; ++k) {
        v0 = ld_dev(d);
        v1 = ld_dev(d + 1);
        v2 = ld_dev(d + 2);
        ok = (uint32_t)(v0 & 0xFFFFFFFFull) == gen && (uint32_t)(v1 & 0xFFFFFFFFull) == gen &&
             (uint32_t)(v2 & 0xFFFFFFFFull) == gen;
        if (ok) break;
        __builtin_amdgcn_s_sleep(1);
      }
      if (!ok) timed_out = 1;
      lat_win = __uint_as_float((uint32_t)(v0 >> 32));
      cid_win = (uint32_t)(v1 >> 32);
      swap_win = __uint_as_float((uint32_t)(v2 >> 32));
    }
    __syncthreads();
    if (timed_out) {
      if (tid == 0) atomicOr(&st->err, kErrSync);
      break;
    }
    const uint32_t cidp1 = cid_win;
    const float lat_sel = lat_win, swap_sel = swap_win;
    __syncthreads();                                         // both are rewritten next round
    if (cidp1 == 0u) break;                                  // nothing live anywhere
    const uint32_t cid = cidp1 - 1u;
    const int bsel = (int)(cid % (uint32_t)B) + 1;
    const int gsel = (int)(cid / (uint32_t)B) / tb.Mmax, msel = (int)(cid / (uint32_t)B) % tb.Mmax;
    const bool mine = gsel >= glo && gsel < glo + ng;        // a group of this application
    if (mine && gsel == gprim) {
      shift = bsel;
      if (SPLIT && m == 0 && tid < bsel)
        st_dev(ps.ring + ((size_t)rl * tb.A + a) * B + tid, ((unsigned long long)gen << 32) | (unsigned long long)(uint32_t)win[tid]);
    } else if (SPLIT && mine) {
      // a secondary group was chosen: its window once more (same clock, nothing of it has changed since it was
      // scored), to move the head pointer past the batch and to hand the batch's positions to the commit workgroup
      const int isel = gsel - glo;
      if (wave == 0) {
        const int nbs = wave_window(w, kind, head_s[isel], w.grp_end[gsel], E0, Bw, wpos, lane);
        if (m == 0)
          for (int j = lane; j < bsel && j < nbs; j += kWave)
            st_dev(ps.ring + ((size_t)rl * tb.A + a) * B + j, ((unsigned long long)gen << 32) | (unsigned long long)(uint32_t)wpos[j]);
        const int last = bsel <= nbs ? wpos[bsel - 1] : w.grp_end[gsel] - 1;
        wave_sync();
        if (lane == 0) head_s[isel] = last + 1;
      }
      __syncthreads();
    }
    t = (t + (double)swap_sel) + (double)lat_sel;
    prev_mine = mine;
    prev_m = msel;
    r += 1;
  }
  {
    unsigned long long ev = evals;                           // lanes 0 of the wavefronts hold the counts
    if (lane == 0 && ev != 0ull) atomicAdd(&st->n_evals, ev);
  }
  // first position of every group of this application that may still be live, for whoever continues the window
  __syncthreads();
  if (m == 0)
    for (int i = tid; i < ng; i += kRoundThreads)
      w.head[(r & 1) * w.gcap + glo + i] = i == prim ? (shift < nb ? win[shift] : scan_end) : head_s[i];
}

__global__ void k_fill_u64(unsigned long long* p, int64_t n, unsigned long long v) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

}  // namespace sp
