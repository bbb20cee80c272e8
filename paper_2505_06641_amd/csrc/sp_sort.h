// Stable least-significant-digit radix passes (8-bit digits) over (key, value)
// pairs, run independently inside each segment of the array.  Used twice per
// window: once over the whole queue with the application id as the key (the
// request groups of Alg. 1, "HashMap<app : request list>"), then four times
// inside each application's range with the inverted bits of the priority key
// (Alg. 1, "requests in g sorted by priority"; eq. (12)) or the bits of the
// deadline (earliest deadline first), and, with data-aware subgroups
// (Sec. 5.3.2), once or twice more with the subgroup label.
//
// The unit of work is one wavefront walking `unit` consecutive elements of one
// segment 64 at a time, in order; units never straddle segments.  A pass is
// three kernels: per-unit digit histograms, a scan down every (segment, digit)
// column, and the scatter, in which every wavefront first redoes the small scan
// over its segment's 256 column totals, then ranks its elements 64 at a time per
// digit with ballots (equal digits keep their order) and bumps a
// wavefront-private running offset table in LDS.  A unit's keys and values are
// all requested before the first is used.  No inter-workgroup waiting.
#pragma once
#include "sp_common.h"
#include "sp_wave.h"
#include "sp_score_generic.h"   // find_segment

namespace sp {

constexpr int kSortWaves = 4;
constexpr int kMaxUnit = 1024;                  // largest sort unit (elements per wavefront and pass)

struct SortPlan {
  const int32_t* seg;          // [nseg+1] segment starts
  const int32_t* unit_start;   // [nseg+1] prefix of units per segment
  int32_t nseg;
  int32_t unit;                // elements per unit, multiple of 64
};

// Orders this wavefront's LDS accesses around it (compiler fence; the hardware
// already runs one wavefront's LDS operations in issue order).
__device__ __forceinline__ void wave_sync() {
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
}

// mask of lanes whose 8-bit digit equals mine
__device__ __forceinline__ unsigned long long match_digit(uint32_t digit, bool valid) {
  unsigned long long m = __ballot(valid);
#pragma unroll
  for (int b = 0; b < 8; ++b) {
    const bool bit = (digit >> b) & 1u;
    const unsigned long long vote = __ballot(bit);
    m &= bit ? vote : ~vote;
  }
  return m;
}

__device__ __forceinline__ bool unit_range(const SortPlan& sp, int u, int& beg, int& end) {
  if (u >= sp.unit_start[sp.nseg]) return false;
  const int s = find_segment(sp.unit_start, sp.nseg, u);
  beg = sp.seg[s] + (u - sp.unit_start[s]) * sp.unit;
  end = min(beg + sp.unit, sp.seg[s + 1]);
  return true;
}

// Clamp application ids into [0, A] (A = "invalid") and flag bad ones.
__global__ void k_app_keys(int n, const int32_t* __restrict__ app, int A, uint32_t* __restrict__ keys, State* st) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const int a = app[i];
  const bool ok = a >= 0 && a < A;
  keys[i] = ok ? (uint32_t)a : (uint32_t)A;
  if (!ok) atomicOr(&st->err, kErrApp);
}

__global__ __launch_bounds__(kSortWaves* kWave) void k_radix_hist(SortPlan sp, const uint32_t* __restrict__ keys,
                                                                  int shift, uint32_t* __restrict__ hist) {
  __shared__ uint32_t cnt[kSortWaves][256];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int i = lane; i < 256; i += 64) cnt[wave][i] = 0;
  wave_sync();
  const int u = blockIdx.x * kSortWaves + wave;
  int beg = 0, end = 0;
  const bool have = unit_range(sp, u, beg, end);
  if (have) {
    uint32_t kbuf[kMaxUnit / 64];                          // all of the unit's keys in flight together
#pragma unroll
    for (int c = 0; c < kMaxUnit / 64; ++c) {
      const int i = beg + c * 64 + lane;
      kbuf[c] = i < end ? keys[i] : 0u;
    }
#pragma unroll
    for (int c = 0; c < kMaxUnit / 64; ++c)
      if (beg + c * 64 + lane < end) atomicAdd(&cnt[wave][(kbuf[c] >> shift) & 255u], 1u);
    wave_sync();
    for (int i = lane; i < 256; i += 64) hist[(int64_t)u * 256 + i] = cnt[wave][i];
  }
}

// Destination offsets from the per-unit counts, in two small kernels.
// k_radix_scan_cols: a workgroup takes 256 / LPC digit columns of one segment and turns each column
// hist[.][digit] of the segment's units into exclusive prefixes down the column (LPC lanes per column, each
// walking every LPC-th unit) and stores the column totals.  LPC = 16 suits the short segments of the key
// passes (one trip for up to 256 units); a long segment (the pass over the application ids has a single one)
// takes a whole wavefront per column, so that 1024 units are still one trip to memory.  The exclusive scan
// over a segment's 256 totals is cheap enough for every scattering wavefront to redo it for itself
// (wave_digit_bases), which saves a launch per pass.
// Offset of (unit u, digit d) = seg[s] + (totals of s before d) + hist[u][d].
constexpr int kScanUnroll = 16;
constexpr int kSegTable = 1024;                        // applications whose tile prefixes k_segments keeps in LDS

template <int LPC>
__global__ __launch_bounds__(256) void k_radix_scan_cols(SortPlan sp, uint32_t* __restrict__ hist,
                                                         uint32_t* __restrict__ tot /*[nseg,256]*/) {
  static_assert(LPC == 16 || LPC == 64, "a column is scanned by a row of 16 lanes or by a wavefront");
  constexpr int kCols = 256 / LPC;                       // digit columns per workgroup
  constexpr int kGroups = 256 / kCols;                   // workgroups per segment
  const int s = blockIdx.x / kGroups, dg = blockIdx.x % kGroups;
  const int col = threadIdx.x / LPC, j = threadIdx.x % LPC;
  const int dgt = dg * kCols + col;
  const int u0 = sp.unit_start[s], u1 = sp.unit_start[s + 1];
  uint32_t carry = 0;                                    // total of the column over the chunks done so far
  // kScanUnroll chunks per trip: their loads are independent of the carry and go out together, so a
  // long column costs one memory round trip per kScanUnroll * LPC units instead of one per LPC
  for (int ub = u0; ub < u1; ub += LPC * kScanUnroll) {
    uint32_t c[kScanUnroll];
#pragma unroll
    for (int q = 0; q < kScanUnroll; ++q) {
      const int u = ub + q * LPC + j;
      c[q] = u < u1 ? hist[(int64_t)u * 256 + dgt] : 0u;
    }
#pragma unroll
    for (int q = 0; q < kScanUnroll; ++q) {
      const int u = ub + q * LPC + j;
      if (ub + q * LPC < u1) {                           // uniform: the rest of the trip is past the segment
        const uint32_t incl = wave_scan_incl<LPC == 16>(c[q]);   // LPC lanes per column: a row, or the wavefront
        if (u < u1) hist[(int64_t)u * 256 + dgt] = carry + incl - c[q];
        carry += __shfl(incl, LPC - 1, LPC);
      }
    }
  }
  if (j == 0) tot[(int64_t)s * 256 + dgt] = carry;
}

// Start of every digit of segment s, given the segment's 256 digit totals: lane l returns the starts of
// digits 4l .. 4l+3.
__device__ __forceinline__ uint4 wave_digit_bases(const uint32_t* __restrict__ tot_s, uint32_t seg_start, int lane) {
  const uint4 t = *reinterpret_cast<const uint4*>(tot_s + 4 * lane);
  const uint32_t mine = t.x + t.y + t.z + t.w;
  const uint32_t incl = wave_scan_incl(mine);
  uint4 b;
  b.x = seg_start + incl - mine;
  b.y = b.x + t.x;
  b.z = b.y + t.y;
  b.w = b.z + t.z;
  return b;
}

// vals_in == nullptr means the identity (value = element index).
__global__ __launch_bounds__(kSortWaves* kWave) void k_radix_scatter(
    SortPlan sp, const uint32_t* __restrict__ keys_in, const int32_t* __restrict__ vals_in, int shift,
    const uint32_t* __restrict__ offs, const uint32_t* __restrict__ tot, uint32_t* __restrict__ keys_out,
    int32_t* __restrict__ vals_out) {
  __shared__ __align__(16) uint32_t run[kSortWaves][256];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int u = blockIdx.x * kSortWaves + wave;
  int beg = 0, end = 0;
  const bool have = unit_range(sp, u, beg, end);
  if (!have) return;   // no block-wide barrier below: wavefronts are independent
  const int sg = find_segment(sp.unit_start, sp.nseg, u);
  {
    const uint4 b = wave_digit_bases(tot + (int64_t)sg * 256, (uint32_t)sp.seg[sg], lane);
    const uint4 o = *reinterpret_cast<const uint4*>(offs + (int64_t)u * 256 + 4 * lane);
    *reinterpret_cast<uint4*>(&run[wave][4 * lane]) = make_uint4(o.x + b.x, o.y + b.y, o.z + b.z, o.w + b.w);
  }
  wave_sync();
  const unsigned long long lt = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
  // the whole unit's keys and values are requested before the first one is used: one trip to memory per
  // unit instead of one per 64 elements (the ranking below is a dependent chain through LDS)
  uint32_t kbuf[kMaxUnit / 64];
  int32_t vbuf[kMaxUnit / 64];
#pragma unroll
  for (int c = 0; c < kMaxUnit / 64; ++c) {
    const int i = beg + c * 64 + lane;
    kbuf[c] = i < end ? keys_in[i] : 0u;
    vbuf[c] = i < end ? (vals_in ? vals_in[i] : i) : 0;
  }
#pragma unroll
  for (int c = 0; c < kMaxUnit / 64; ++c) {
    if (beg + c * 64 >= end) break;                        // uniform
    const int i = beg + c * 64 + lane;
    const bool valid = i < end;
    const uint32_t key = kbuf[c];
    const int32_t val = vbuf[c];
    const uint32_t dg = (key >> shift) & 255u;
    const unsigned long long same = match_digit(dg, valid);
    const int rank = __popcll(same & lt);
    // the first lane of each digit group reserves the group's slots, then hands the base to its group
    const int leader = valid ? (__ffsll((long long)same) - 1) : lane;
    uint32_t base_off = 0;
    if (valid && lane == leader) base_off = atomicAdd(&run[wave][dg], (uint32_t)__popcll(same));
    base_off = __shfl(base_off, leader);
    const uint32_t dst = base_off + (uint32_t)rank;
    if (valid) {
      keys_out[dst] = key;
      vals_out[dst] = val;
    }
  }
}

// Segment starts from the application-sorted keys (values in [0, A], A =
// invalid): seg[a] = first position with key >= a; then the prefixes of
// scoring tiles and sort units per application and the scoring tiles' descriptors.  One workgroup.
// digit_tot, when given, holds the count of every digit of a single radix pass over the application ids
// (wavefront 0 turns them into the segment starts without any search).
__global__ __launch_bounds__(256) void k_segments(int n, int A, const uint32_t* __restrict__ sorted_app,
                                                  const uint32_t* __restrict__ digit_tot, int tile, int unit,
                                                  int32_t* seg, int32_t* tile_start, int32_t* unit_start,
                                                  int4* tile_desc, Window w) {
  if (digit_tot != nullptr) {
    if (threadIdx.x < 64) {
      const int lane = threadIdx.x;
      const uint4 b = wave_digit_bases(digit_tot, 0u, lane);
      const uint32_t bb[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
      for (int q = 0; q < 4; ++q)
        if (4 * lane + q <= A) seg[4 * lane + q] = (int)bb[q];
      if (lane == 0) seg[A + 1] = n;
    }
  }
  for (int a = threadIdx.x; a <= A + 1 && digit_tot == nullptr; a += blockDim.x) {
    int lo = 0, hi = n;                     // lower_bound(sorted_app, a)
    while (lo < hi) {
      const int mid = (lo + hi) >> 1;
      if (sorted_app[mid] < (uint32_t)a) lo = mid + 1; else hi = mid;
    }
    seg[a] = lo;                            // seg[A] = number of valid requests, seg[A+1] = n
  }
  __syncthreads();
  // until (and unless) the requests are split into subgroups, group g is application g
  for (int a = threadIdx.x; a < A; a += blockDim.x) {
    w.head[a] = seg[a];
    w.head[w.gcap + a] = seg[a];
    w.grp_app[a] = a;
    w.grp_end[a] = seg[a + 1];
  }
  if (threadIdx.x == 0) *w.grp_n = A;
  // prefixes of tiles and units over the applications: every thread takes a run of consecutive
  // applications, the runs' totals are scanned across the workgroup (launched with 256 threads)
  __shared__ int run_t[256], run_u[256];
  __shared__ int s_tile[kSegTable + 1], s_seg[kSegTable + 1];   // used when A <= kSegTable
  const int tid = threadIdx.x;
  const int per = (A + 255) / 256;
  const int a_lo = min(A, tid * per), a_hi = min(A, a_lo + per);
  int ts = 0, us = 0;
  for (int a = a_lo; a < a_hi; ++a) {
    const int na = seg[a + 1] - seg[a];
    ts += (na + tile - 1) / tile;
    us += (na + unit - 1) / unit;
  }
  run_t[tid] = ts;
  run_u[tid] = us;
  __syncthreads();
  for (int o = 1; o < 256; o <<= 1) {
    const int t_up = tid >= o ? run_t[tid - o] : 0;
    const int u_up = tid >= o ? run_u[tid - o] : 0;
    __syncthreads();
    run_t[tid] += t_up;
    run_u[tid] += u_up;
    __syncthreads();
  }
  const int ts0 = run_t[tid] - ts, us0 = run_u[tid] - us;   // exclusive prefixes of this thread's run
  const bool table = A <= kSegTable;
  ts = ts0;
  us = us0;
  for (int a = a_lo; a < a_hi; ++a) {
    tile_start[a] = ts;
    unit_start[a] = us;
    const int sb = seg[a], na = seg[a + 1] - sb;
    if (table) {
      s_tile[a] = ts;
      s_seg[a] = sb;
    }
    ts += (na + tile - 1) / tile;
    us += (na + unit - 1) / unit;
  }
  if (tid == 255) {
    tile_start[A] = run_t[255];
    unit_start[A] = run_u[255];
    if (table) {
      s_tile[A] = run_t[255];
      s_seg[A] = seg[A];
    }
  }
  __syncthreads();
  // one descriptor per scoring tile, so that a scoring workgroup finds its place with a single load
  if (table) {
    // few applications: every thread places tiles by searching the prefixes in LDS
    const int n_tiles = s_tile[A];
    for (int t = tid; t < n_tiles; t += 256) {
      int lo = 0, hi = A;                                // last a with s_tile[a] <= t (empty applications share a start)
      while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (s_tile[mid] <= t) lo = mid; else hi = mid;
      }
      tile_desc[t] = make_int4(lo, s_seg[lo] + (t - s_tile[lo]) * tile, s_seg[lo + 1], 0);
    }
  } else {
    ts = ts0;
    for (int a = a_lo; a < a_hi; ++a) {
      const int sb = seg[a], se = seg[a + 1], nt = (se - sb + tile - 1) / tile;
      for (int t = 0; t < nt; ++t) tile_desc[ts + t] = make_int4(a, sb + t * tile, se, 0);
      ts += nt;
    }
  }
}

// Subgroup codes as sort keys, in the current order of the passes' values (grouped positions).
__global__ void k_gather_sub_keys(int n_valid_at, const int32_t* __restrict__ seg, const int32_t* __restrict__ grouped_pos,
                                  const int32_t* __restrict__ sub_g, uint32_t* __restrict__ keys) {
  const int pos = blockIdx.x * blockDim.x + threadIdx.x;
  if (pos < seg[n_valid_at]) keys[pos] = (uint32_t)sub_g[grouped_pos[pos]];
}

// Range of every possible (application, subgroup code) pair in the service order: two binary searches on
// the sorted codes inside the application's range.  Slot s belongs to application slot_app[s] and code
// s - slot_base[application].
__global__ void k_slot_ranges(int n_slots, const int32_t* __restrict__ slot_app, const int32_t* __restrict__ slot_base,
                              const int32_t* __restrict__ seg, const uint32_t* __restrict__ sub_sorted,
                              int32_t* __restrict__ slot_beg, int32_t* __restrict__ slot_end) {
  const int s = blockIdx.x * blockDim.x + threadIdx.x;
  if (s >= n_slots) return;
  const int a = slot_app[s];
  const uint32_t code = (uint32_t)(s - slot_base[a]);
  const int b0 = seg[a], e0 = seg[a + 1];
  int lo = b0, hi = e0;
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if (sub_sorted[mid] < code) lo = mid + 1; else hi = mid;
  }
  const int beg = lo;
  hi = e0;
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if (sub_sorted[mid] <= code) lo = mid + 1; else hi = mid;
  }
  slot_beg[s] = beg;
  slot_end[s] = lo;
}

// The non-empty slots, in slot order, become the groups of the rounds.  One workgroup.
__global__ __launch_bounds__(1024) void k_groups_compact(int n_slots, const int32_t* __restrict__ slot_app,
                                                         const int32_t* __restrict__ slot_beg,
                                                         const int32_t* __restrict__ slot_end, Window w) {
  __shared__ int wave_cnt[16];
  __shared__ int base_s;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (tid == 0) base_s = 0;
  __syncthreads();
  for (int s0 = 0; s0 < n_slots; s0 += 1024) {
    const int s = s0 + tid;
    const bool full = s < n_slots && slot_end[s] > slot_beg[s];
    const unsigned long long bal = __ballot(full);
    if (lane == 0) wave_cnt[wave] = __popcll(bal);
    __syncthreads();
    int before = base_s, total = 0;
    for (int i = 0; i < 16; ++i) {
      if (i < wave) before += wave_cnt[i];
      total += wave_cnt[i];
    }
    if (full) {
      const int j = before + __popcll(bal & ((1ull << lane) - 1ull));
      if (j < w.gcap) {
        w.grp_app[j] = slot_app[s];
        w.grp_end[j] = slot_end[s];
        w.head[j] = slot_beg[s];
        w.head[w.gcap + j] = slot_beg[s];
      }
    }
    __syncthreads();
    if (tid == 0) base_s += total;
    __syncthreads();
  }
  if (tid == 0) *w.grp_n = min(base_s, w.gcap);
}

// The four per-request outputs into the caller's arrays (any of them may be null), one launch.
__global__ void k_copy_outputs(int n, Window w, int32_t* __restrict__ model, int32_t* __restrict__ round_of,
                               int32_t* __restrict__ order_of, float* __restrict__ util) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  if (model) model[i] = w.model[i];
  if (round_of) round_of[i] = w.round_of[i];
  if (order_of) order_of[i] = w.order_of[i];
  if (util) util[i] = w.util[i];
}

// After the last pass.  The passes carried positions of the application-grouped array as values and the
// inverted key bits as keys, so per service position: id, deadline and weight come with one gather of the
// record the scoring kernel left at the grouped position, the key straight from the sorted key bits.
__global__ void k_finish_order(int n, int n_valid_at /*index into seg*/, const int32_t* __restrict__ seg,
                               const int32_t* __restrict__ grouped_pos, const uint32_t* __restrict__ sorted_keys,
                               Window w, int edf) {
  const int pos = blockIdx.x * blockDim.x + threadIdx.x;
  if (pos >= n) return;
  const int nv = seg[n_valid_at];
  if (pos < nv) {
    const float4 rc = w.rec_g[grouped_pos[pos]];          // one 16-byte gather per request
    const int id = __float_as_int(rc.x);
    w.id_s[pos] = id;
    w.D_s[pos] = rc.y;
    w.w_s[pos] = rc.z;
    // the passes sorted the inverted key bits, or (earliest deadline first) the deadline bits
    w.key_s[pos] = edf ? w.key[id] : __uint_as_float(~sorted_keys[pos]);
    w.alive_s[pos] = 1;
  } else {
    w.alive_s[pos] = 0;
  }
  // per-request outputs back to "not served" (indexed by request id: every id in [0, n) once)
  w.model[pos] = -1;
  w.round_of[pos] = -1;
  w.order_of[pos] = 0;
  w.util[pos] = 0.f;
}

}  // namespace sp
