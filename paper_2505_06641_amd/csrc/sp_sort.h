// Stable least-significant-digit radix passes (8-bit digits) over (key, value)
// pairs, run independently inside each segment of the array.  Used twice per
// window: once over the whole queue with the application id as the key (the
// request groups of Alg. 1, "HashMap<app : request list>"), then four times
// inside each application's range with the inverted bits of the priority key
// (Alg. 1, "requests in g sorted by priority"; eq. (12)) or the bits of the
// deadline (earliest deadline first), and, with data-aware subgroups
// (Sec. 5.3.2), once or twice more with the subgroup label.
//
// One kernel per pass.  The unit of work is a tile of kSortTile consecutive
// elements of one segment, taken by one workgroup; tiles never straddle
// segments.  A workgroup ranks its elements by digit (ballot matching inside
// a wavefront, equal digits keep their order; per-wavefront digit counts in
// LDS, scanned across the wavefronts), publishes its 256 digit counts, and
// gets the counts of the tiles before it in its segment by looking back
// through what they have published (a tile publishes first its own counts,
// then the running prefix, so the walk ends at the first tile that already
// knows its prefix).  The published words carry the generation number of the
// pass, so a word is valid exactly when its generation matches: no clearing
// between passes, no fences.  Where each digit of a segment starts follows
// from the segment's digit totals, which one small kernel (k_digit_totals)
// counts for all passes of a sort before the first pass.  The elements go
// through LDS in sorted order, so that global writes are runs of consecutive
// addresses per digit rather than single elements.
// A tile waits only for tiles with a lower index, which the hardware starts
// no later than itself; every wait is bounded all the same (kErrSortSync).
#pragma once
#include "sp_common.h"
#include "sp_wave.h"
#include "sp_score_generic.h"   // find_segment

namespace sp {

constexpr int kSortThreads = 512;
constexpr int kSortWaves = kSortThreads / kWave;
constexpr int kSortItems = 8;                         // elements per thread
constexpr int kSortTile = kSortThreads * kSortItems;  // elements per tile
constexpr int kSortSpinLimit = 1 << 20;               // polls before a look-back is given up
constexpr uint32_t kSortCountMask = 0x3FFFFFFFu;      // a published word: generation << 32 | status << 30 | count
constexpr int kLookBack = 8;                          // tiles whose published words are requested together
constexpr int kMaxSortPasses = 6;                     // four key passes and up to two over subgroup labels

struct SortPlan {
  const int32_t* seg;          // [nseg+1] segment starts
  const int32_t* unit_start;   // [nseg+1] prefix of tiles per segment
  int32_t nseg;
  const int4* desc;            // per tile: (segment, first element, end, first tile of the segment); null = one segment
};

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

// This workgroup's tile: segment s, elements [beg, end), first tile of s.  False for a workgroup without one.
__device__ __forceinline__ bool sort_tile(const SortPlan& sp, int tile, int& s, int& beg, int& end, int& first) {
  if (sp.desc == nullptr) {
    const int n = sp.seg[1];
    s = 0; first = 0;
    beg = tile * kSortTile;
    end = min(beg + kSortTile, n);
    return beg < n;
  }
  if (tile >= sp.unit_start[sp.nseg]) return false;
  const int4 d = sp.desc[tile];
  s = d.x; beg = d.y; end = d.z; first = d.w;
  return true;
}

// The key of element i: as stored, or (clamp_a > 0) an application id clamped into [0, A] with A = "invalid".
__device__ __forceinline__ uint32_t sort_key_at(const uint32_t* __restrict__ keys, int i, int clamp_a, bool& bad) {
  const uint32_t k = keys[i];
  if (clamp_a <= 0) return k;
  const int a = (int)k;
  const bool ok = a >= 0 && a < clamp_a;
  bad |= !ok;
  return ok ? k : (uint32_t)clamp_a;
}

constexpr int kSegTable = 1024;                        // applications whose tile prefixes k_segments keeps in LDS

// Start of every digit of a segment, given its 256 digit totals: lane l returns the starts of digits
// 4l .. 4l+3.
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

// Segment starts from the application-sorted keys (values in [0, A], A =
// invalid): seg[a] = first position with key >= a; then the prefixes of
// scoring tiles and sort units per application and the scoring tiles' descriptors.  One workgroup.
// digit_tot, when given, holds the count of every digit of a single radix pass over the application ids
// (wavefront 0 turns them into the segment starts without any search).
struct SegArgs {
  int32_t n, A;
  const uint32_t* sorted_app;   // application-sorted keys (used when digit_tot is null)
  const uint32_t* digit_tot;    // or: the count of every application id (one radix pass over the ids)
  int32_t tile, unit;           // requests per scoring tile and per sort tile
  int32_t small_cap;            // applications with at most this many requests get no sort tiles (k_sort_small orders them); 0: none
  int32_t* seg;
  int32_t* tile_start;
  int32_t* unit_start;
  int4* tile_desc;
  int4* sort_desc;
};

// Body of k_segments for the first 256 threads of a workgroup (any others only keep the barriers company).
__device__ __forceinline__ void segments_body(const SegArgs& g, const Window& w) {
  const int n = g.n, A = g.A, tile = g.tile, unit = g.unit;
  const uint32_t* __restrict__ sorted_app = g.sorted_app;
  const uint32_t* __restrict__ digit_tot = g.digit_tot;
  int32_t *seg = g.seg, *tile_start = g.tile_start, *unit_start = g.unit_start;
  int4 *tile_desc = g.tile_desc, *sort_desc = g.sort_desc;
  const bool on = threadIdx.x < 256;
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
  for (int a = threadIdx.x; on && a <= A + 1 && digit_tot == nullptr; a += 256) {
    int lo = 0, hi = n;                     // lower_bound(sorted_app, a)
    while (lo < hi) {
      const int mid = (lo + hi) >> 1;
      if (sorted_app[mid] < (uint32_t)a) lo = mid + 1; else hi = mid;
    }
    seg[a] = lo;                            // seg[A] = number of valid requests, seg[A+1] = n
  }
  __syncthreads();
  // until (and unless) the requests are split into subgroups, group g is application g
  for (int a = threadIdx.x; on && a < A; a += 256) {
    w.head[a] = seg[a];
    w.head[w.gcap + a] = seg[a];
    w.grp_app[a] = a;
    w.grp_end[a] = seg[a + 1];
  }
  if (threadIdx.x == 0) {
    w.grp_n[0] = A;
    w.grp_n[1] = 1;
  }
  // prefixes of tiles and units over the applications: every thread takes a run of consecutive
  // applications, the runs' totals are scanned across the workgroup (launched with 256 threads)
  __shared__ int run_t[256], run_u[256];
  __shared__ int s_tile[kSegTable + 1], s_seg[kSegTable + 1], s_unit[kSegTable + 1];   // used when A <= kSegTable
  const int tid = on ? threadIdx.x : 0;          // threads beyond 255 shadow thread 0 and store nothing
  const int per = (A + 255) / 256;
  const int a_lo = on ? min(A, tid * per) : 0, a_hi = on ? min(A, a_lo + per) : 0;
  int ts = 0, us = 0;
  for (int a = a_lo; a < a_hi; ++a) {
    const int na = seg[a + 1] - seg[a];
    ts += (na + tile - 1) / tile;
    us += na > g.small_cap ? (na + unit - 1) / unit : 0;
  }
  if (on) {
    run_t[tid] = ts;
    run_u[tid] = us;
  }
  __syncthreads();
  for (int o = 1; o < 256; o <<= 1) {
    const int t_up = tid >= o ? run_t[tid - o] : 0;
    const int u_up = tid >= o ? run_u[tid - o] : 0;
    __syncthreads();
    if (on) {
      run_t[tid] += t_up;
      run_u[tid] += u_up;
    }
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
      s_unit[a] = us;
      s_seg[a] = sb;
    }
    ts += (na + tile - 1) / tile;
    us += na > g.small_cap ? (na + unit - 1) / unit : 0;
  }
  if (on && tid == 255) {
    tile_start[A] = run_t[255];
    unit_start[A] = run_u[255];
    if (table) {
      s_tile[A] = run_t[255];
      s_unit[A] = run_u[255];
      s_seg[A] = seg[A];
    }
  }
  __syncthreads();
  // one descriptor per scoring tile, so that a scoring workgroup finds its place with a single load
  if (table) {
    // few applications: every thread places tiles by searching the prefixes in LDS
    const int n_tiles = s_tile[A];
    for (int t = tid; on && t < n_tiles; t += 256) {
      int lo = 0, hi = A;                                // last a with s_tile[a] <= t (empty applications share a start)
      while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (s_tile[mid] <= t) lo = mid; else hi = mid;
      }
      tile_desc[t] = make_int4(lo, s_seg[lo] + (t - s_tile[lo]) * tile, s_seg[lo + 1], 0);
    }
    // and one per sort tile: (application, first element, end, first tile of the application)
    const int n_units = s_unit[A];
    for (int u = tid; on && u < n_units; u += 256) {
      int lo = 0, hi = A;
      while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (s_unit[mid] <= u) lo = mid; else hi = mid;
      }
      const int b0 = s_seg[lo] + (u - s_unit[lo]) * unit;
      sort_desc[u] = make_int4(lo, b0, min(b0 + unit, s_seg[lo + 1]), s_unit[lo]);
    }
  } else {
    ts = ts0;
    us = us0;
    for (int a = a_lo; a < a_hi; ++a) {
      const int sb = seg[a], se = seg[a + 1], nt = (se - sb + tile - 1) / tile, nu = se - sb > g.small_cap ? (se - sb + unit - 1) / unit : 0;
      for (int t = 0; t < nt; ++t) tile_desc[ts + t] = make_int4(a, sb + t * tile, se, 0);
      for (int u = 0; u < nu; ++u) sort_desc[us + u] = make_int4(a, sb + u * unit, min(sb + (u + 1) * unit, se), us);
      ts += nt;
      us += nu;
    }
  }
}

__global__ __launch_bounds__(256) void k_segments(SegArgs g, Window w) { segments_body(g, w); }

// Digit totals of every segment for n_pass consecutive passes (digits at shift0, shift0 + 8, ...):
// dtot[(p * tiles_cap + first tile of the segment) * 256 + digit], which must be zero beforehand.  Also
// clears zero_rows rows of each of zero_passes pass slabs of another totals array (the next sort's).
__global__ __launch_bounds__(kSortThreads) void k_digit_totals(SortPlan sp, const uint32_t* __restrict__ keys,
                                                               int clamp_a, int shift0, int n_pass, int64_t tiles_cap,
                                                               uint32_t* __restrict__ dtot, uint32_t* __restrict__ zero_ptr,
                                                               int zero_passes, int64_t zero_rows, int64_t zero_cap,
                                                               State* st) {
  __shared__ uint32_t h[4][256];
  const int tid = threadIdx.x;
  if (zero_ptr != nullptr) {
    const int64_t per = zero_rows * 256, stride = (int64_t)gridDim.x * kSortThreads;
    for (int p = 0; p < zero_passes; ++p)
      for (int64_t i = (int64_t)blockIdx.x * kSortThreads + tid; i < per; i += stride) zero_ptr[p * zero_cap * 256 + i] = 0u;
  }
  int s, beg, end, first;
  if (!sort_tile(sp, blockIdx.x, s, beg, end, first)) return;
  for (int i = tid; i < 4 * 256; i += kSortThreads) h[0][i] = 0u;
  __syncthreads();
  bool bad = false;
#pragma unroll
  for (int c = 0; c < kSortItems; ++c) {
    const int i = beg + c * kSortThreads + tid;
    if (i < end) {
      const uint32_t k = sort_key_at(keys, i, clamp_a, bad);
      for (int p = 0; p < n_pass; ++p) atomicAdd(&h[p][(k >> (shift0 + 8 * p)) & 255u], 1u);
    }
  }
  if (bad) atomicOr(&st->err, kErrApp);
  __syncthreads();
  for (int i = tid; i < n_pass * 256; i += kSortThreads) {
    const uint32_t c = h[0][i];
    if (c) atomicAdd(&dtot[((int64_t)(i >> 8) * tiles_cap + first) * 256 + (i & 255)], c);
  }
}

// Exclusive prefix sums of one value per thread over the first 256 threads of the workgroup (all of its
// threads call it; those beyond 255 pass 0 and get the total).
template <int WAVES = kSortWaves>
__device__ __forceinline__ uint32_t scan256_excl(uint32_t v, uint32_t* wave_tot /*[WAVES]*/) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint32_t incl = wave_scan_incl(v);
  __syncthreads();
  if (lane == 63) wave_tot[wave] = incl;
  __syncthreads();
  uint32_t before = 0;
  for (int i = 0; i < WAVES; ++i) before += i < wave ? wave_tot[i] : 0u;
  return before + incl - v;
}

// Two floats that travel with an element through a pass (the grouping pass brings every request's deadline
// and weight to its grouped position, so that the scoring kernel reads them in order instead of gathering
// them by request id, 4 useful bytes per 64-byte line): read from two arrays or from one array of pairs,
// indexed by element, written as pairs.
struct SortCarry {
  const float* in0;            // [n], with in1; or null
  const float* in1;
  const float2* in01;          // [n] pairs (a second pass); or null
  float2* out;                 // [n] pairs at the elements' new positions
};

// One stable pass: (keys_in, vals_in) -> (keys_out, vals_out) by the digit at `shift`.  vals_in == nullptr
// means the identity (value = element index).  dtot_pass: this pass's slab of digit totals.  state:
// [tiles][256] published words; gen: this launch's generation (never reused while the array lives).
template <bool CARRY>
__global__ __launch_bounds__(kSortThreads) void k_radix_pass(
    SortPlan sp, const uint32_t* __restrict__ keys_in, const int32_t* __restrict__ vals_in, int shift, int clamp_a,
    const uint32_t* __restrict__ dtot_pass, unsigned long long* __restrict__ state, uint32_t gen, int spin_limit,
    uint32_t* __restrict__ keys_out, int32_t* __restrict__ vals_out, State* st, SegArgs sg, Window sw, SortCarry cy) {
  // One extra workgroup (sg.seg != null) does k_segments' job beside the pass over the application ids,
  // which needs nothing but the ids' digit totals: a launch and its trips to memory less per window.
  if (sg.seg != nullptr && (int)blockIdx.x == (int)gridDim.x - 1) {
    segments_body(sg, sw);
    return;
  }
  __shared__ uint32_t cnt[kSortWaves][256];      // digit counts per wavefront, then their exclusive prefix over the wavefronts
  __shared__ uint32_t lstart[256];               // where each digit starts inside the sorted tile
  __shared__ uint32_t dbase[256];                // global position of the digit's first element of this tile, minus lstart
  __shared__ uint32_t wave_tot[kSortWaves];
  __shared__ uint32_t skey[kSortTile];
  __shared__ int32_t sval[kSortTile];
  __shared__ float2 spay[CARRY ? kSortTile : 1];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int s, beg, end, first;
  if (!sort_tile(sp, blockIdx.x, s, beg, end, first)) return;
  const int tile = blockIdx.x;
  for (int i = tid; i < kSortWaves * 256; i += kSortThreads) cnt[0][i] = 0u;
  // a wavefront takes kSortItems chunks of 64 consecutive elements: all loads go out before the first is used
  uint32_t key[kSortItems];
  int32_t val[kSortItems];
  bool bad = false;
#pragma unroll
  for (int c = 0; c < kSortItems; ++c) {
    const int i = beg + (wave * kSortItems + c) * 64 + lane;
    key[c] = i < end ? sort_key_at(keys_in, i, clamp_a, bad) : 0u;
    val[c] = i < end ? (vals_in ? vals_in[i] : i) : 0;
  }
  float2 pay[CARRY ? kSortItems : 1];
  if (CARRY) {
#pragma unroll
    for (int c = 0; c < kSortItems; ++c) {
      const int i = beg + (wave * kSortItems + c) * 64 + lane;
      pay[c] = make_float2(0.f, 0.f);
      if (i < end) pay[c] = cy.in01 ? cy.in01[i] : make_float2(cy.in0[i], cy.in1[i]);
    }
  }
  if (bad) atomicOr(&st->err, kErrApp);
  __syncthreads();
  // rank inside the wavefront: lanes with my digit ahead of me in this chunk, plus the wavefront's earlier chunks
  const unsigned long long lt = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
  uint32_t rank[kSortItems];
#pragma unroll
  for (int c = 0; c < kSortItems; ++c) {
    const int i = beg + (wave * kSortItems + c) * 64 + lane;
    const bool valid = i < end;
    const uint32_t dg = (key[c] >> shift) & 255u;
    const unsigned long long same = match_digit(dg, valid);
    const int leader = valid ? (__ffsll((long long)same) - 1) : lane;
    uint32_t before = 0;
    if (valid && lane == leader) before = atomicAdd(&cnt[wave][dg], (uint32_t)__popcll(same));
    before = __shfl(before, leader);
    rank[c] = before + (uint32_t)__popcll(same & lt);
  }
  __syncthreads();
  // digit counts of the tile; cnt becomes the exclusive prefix over the wavefronts
  uint32_t mine = 0;
  if (tid < 256) {
#pragma unroll
    for (int w = 0; w < kSortWaves; ++w) {
      const uint32_t c = cnt[w][tid];
      cnt[w][tid] = mine;
      mine += c;
    }
  }
  // tiles before this one in the segment: publish, look back, publish the running prefix
  uint32_t excl = 0;
  if (tid < 256) {
    unsigned long long* slot = state + (size_t)tile * 256 + tid;
    const unsigned long long tag = (unsigned long long)gen << 32;
    if (tile == first) {
      __hip_atomic_store(slot, tag | (2ull << 30) | mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    } else {
      __hip_atomic_store(slot, tag | (1ull << 30) | mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      // Look back a window of tiles at a time: all of the window's words are requested together (one trip
      // to memory for up to kLookBack tiles), then taken nearest first until one carries a running prefix.
      bool lost = false, found = false;
      for (int t2 = tile - 1; t2 >= first && !found && !lost; t2 -= kLookBack) {
        unsigned long long v[kLookBack];
#pragma unroll
        for (int q = 0; q < kLookBack; ++q) {
          const int t3 = max(t2 - q, first);
          v[q] = __hip_atomic_load(state + (size_t)t3 * 256 + tid, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
#pragma unroll
        for (int q = 0; q < kLookBack; ++q) {
          if (t2 - q < first || found || lost) continue;
          unsigned long long w = v[q];
          if (spin_limit < 0) lost = true;                             // a test's way into the failure path: give up unseen
          for (int k = 0; !lost && (uint32_t)(w >> 32) != gen; ++k) {  // not published yet: poll this one
            if (k >= spin_limit) { lost = true; break; }
            __builtin_amdgcn_s_sleep(1);
            w = __hip_atomic_load(state + (size_t)(t2 - q) * 256 + tid, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          }
          if (lost) continue;
          excl += (uint32_t)w & kSortCountMask;
          found = ((uint32_t)w >> 30) == 2u;
        }
      }
      if (lost) atomicOr(&st->err, kErrSortSync);     // the counts seen so far keep every write inside the segment
      __hip_atomic_store(slot, tag | (2ull << 30) | ((excl + mine) & kSortCountMask), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
  // where the digits start: inside the tile, and in the segment
  const uint32_t tot = tid < 256 ? dtot_pass[(size_t)first * 256 + tid] : 0u;
  const uint32_t ls = scan256_excl(mine, wave_tot);
  const uint32_t gs = scan256_excl(tot, wave_tot);
  if (tid < 256) {
    lstart[tid] = ls;
    dbase[tid] = (uint32_t)sp.seg[s] + gs + excl - ls;
  }
  __syncthreads();
  // into LDS in sorted order
#pragma unroll
  for (int c = 0; c < kSortItems; ++c) {
    const int i = beg + (wave * kSortItems + c) * 64 + lane;
    if (i < end) {
      const uint32_t dg = (key[c] >> shift) & 255u;
      const uint32_t p = lstart[dg] + cnt[wave][dg] + rank[c];
      skey[p] = key[c];
      sval[p] = val[c];
      if (CARRY) spay[p] = pay[c];
    }
  }
  __syncthreads();
  // and out: neighbouring threads hold neighbouring elements of a digit's run
  const int n_tile = end - beg;
  for (int j = tid; j < n_tile; j += kSortThreads) {
    const uint32_t k = skey[j];
    const uint32_t dst = dbase[(k >> shift) & 255u] + (uint32_t)j;
    keys_out[dst] = k;
    vals_out[dst] = sval[j];
    if (CARRY) cy.out[dst] = spay[j];
  }
}

// All four key passes of one application in one kernel, for applications whose whole range fits one
// workgroup's LDS (at most kSmallSortCap requests; k_segments gives such applications no tiles in the passes
// above).  A window of a few thousand requests is otherwise six dependent launches of a few microseconds each.
// The elements live in registers between the passes (wavefront w holds elements [1024 w, 1024 (w + 1)) in
// order, 64 per chunk); a pass ranks them like k_radix_pass, scans the counts over the wavefronts and the
// digits, places the (key, value) pairs in LDS in sorted order and reads them back.  Values are grouped
// positions, as in the passes above; the result goes to the same arrays the last of those passes writes.
constexpr int kSmallSortThreads = 1024;
constexpr int kSmallSortWaves = kSmallSortThreads / kWave;
constexpr int kSmallSortItems = 16;
constexpr int kSmallSortCap = kSmallSortThreads * kSmallSortItems;   // 16,384

__global__ __launch_bounds__(kSmallSortThreads) void k_sort_small(const int32_t* __restrict__ seg,
                                                                  const uint32_t* keys_in /* may be keys_out */,
                                                                  uint32_t* keys_out, int32_t* __restrict__ vals_out) {
  __shared__ unsigned long long buf[kSmallSortCap];            // key << 32 | value, in sorted order
  __shared__ uint32_t cnt[kSmallSortWaves][256];
  __shared__ uint32_t lstart[256];
  __shared__ uint32_t wave_tot[kSmallSortWaves];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int b0 = seg[blockIdx.x], n = seg[blockIdx.x + 1] - b0;
  if (n <= 0 || n > kSmallSortCap) return;                     // (uniform) empty, or sorted by the tiled passes
  // wavefronts and chunks that hold elements (the ranking is the expensive part: nothing is spent on empty ones)
  const int n_waves = (n + kSmallSortItems * 64 - 1) / (kSmallSortItems * 64);
  const int my_chunks = min(kSmallSortItems, max(0, (n - wave * kSmallSortItems * 64 + 63) / 64));
  uint32_t key[kSmallSortItems];
  int32_t val[kSmallSortItems];
#pragma unroll
  for (int c = 0; c < kSmallSortItems; ++c) {
    const int e = (wave * kSmallSortItems + c) * 64 + lane;
    key[c] = e < n ? keys_in[b0 + e] : 0u;
    val[c] = b0 + e;
  }
  const unsigned long long lt = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
  for (int shift = 0; shift < 32; shift += 8) {
    for (int i = tid; i < n_waves * 256; i += kSmallSortThreads) cnt[0][i] = 0u;
    __syncthreads();
    uint32_t rank[kSmallSortItems];
#pragma unroll
    for (int c = 0; c < kSmallSortItems; ++c) {
      rank[c] = 0;
      if (c < my_chunks) {                                       // uniform over the wavefront
        const int e = (wave * kSmallSortItems + c) * 64 + lane;
        const bool valid = e < n;
        const uint32_t dg = (key[c] >> shift) & 255u;
        const unsigned long long same = match_digit(dg, valid);
        const int leader = valid ? (__ffsll((long long)same) - 1) : lane;
        uint32_t before = 0;
        if (valid && lane == leader) before = atomicAdd(&cnt[wave][dg], (uint32_t)__popcll(same));
        before = __shfl(before, leader);
        rank[c] = before + (uint32_t)__popcll(same & lt);
      }
    }
    __syncthreads();
    uint32_t mine = 0;
    if (tid < 256) {
      for (int w = 0; w < n_waves; ++w) {
        const uint32_t c = cnt[w][tid];
        cnt[w][tid] = mine;
        mine += c;
      }
    }
    const uint32_t ls = scan256_excl<kSmallSortWaves>(mine, wave_tot);
    if (tid < 256) lstart[tid] = ls;
    __syncthreads();
#pragma unroll
    for (int c = 0; c < kSmallSortItems; ++c) {
      const int e = (wave * kSmallSortItems + c) * 64 + lane;
      if (e < n) {
        const uint32_t dg = (key[c] >> shift) & 255u;
        buf[lstart[dg] + cnt[wave][dg] + rank[c]] = ((unsigned long long)key[c] << 32) | (unsigned long long)(uint32_t)val[c];
      }
    }
    __syncthreads();
#pragma unroll
    for (int c = 0; c < kSmallSortItems; ++c) {
      const int e = (wave * kSmallSortItems + c) * 64 + lane;
      if (e < n) {
        const unsigned long long kv = buf[e];
        key[c] = (uint32_t)(kv >> 32);
        val[c] = (int32_t)(uint32_t)kv;
      }
    }
    __syncthreads();
  }
#pragma unroll
  for (int c = 0; c < kSmallSortItems; ++c) {
    const int e = (wave * kSmallSortItems + c) * 64 + lane;
    if (e < n) {
      keys_out[b0 + e] = key[c];
      vals_out[b0 + e] = val[c];
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
  const int G = min(base_s, w.gcap);
  // the most groups any application has (the groups of an application are consecutive): it decides whether
  // the resident rounds kernel, whose workgroups each serve all groups of one application, can take the window
  __shared__ int max_run;
  if (tid == 0) max_run = 0;
  __threadfence();
  __syncthreads();
  for (int j = tid; j < G; j += 1024) {
    const int a = w.grp_app[j];
    if (j == 0 || w.grp_app[j - 1] != a) {
      int lo = j, hi = G;                                 // first index past j whose application is not a
      while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (w.grp_app[mid] == a) lo = mid; else hi = mid;
      }
      atomicMax(&max_run, hi - j);
    }
  }
  __syncthreads();
  if (tid == 0) {
    w.grp_n[0] = G;
    w.grp_n[1] = max_run;
  }
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
