// Host runtime and C ABI of the SneakPeek HIP library: profile validation and
// upload, window buffers, kernel launch order, status codes.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "sneakpeek.h"
#include "sp_common.h"
#include "sp_rounds.h"
#include "sp_score_generic.h"
#include "sp_score_split.h"
#include "sp_score_mlp.h"
#include "sp_rounds_persist.h"
#include "sp_sort.h"
#include "sp_probe.h"

using namespace sp;

static_assert(sizeof(Decision) == sizeof(sp_decision), "device and ABI decision records must match");
static_assert(SP_MAX_MODELS == kMaxModels && SP_MAX_BATCH == kMaxBatch, "limits out of sync");

struct sp_ctx {
  int device = 0;
  Tables tb{};
  Window w{};
  std::vector<void*> dev_allocs;
  int A = 0, d = 0, H = 0, B = 0, Mmax = 0, Cmax = 0, dtype = 0;
  int64_t cap = 0;
  uint32_t* bufK[2] = {nullptr, nullptr};
  int32_t* bufV[3] = {nullptr, nullptr, nullptr};
  // ordering: digit totals, per-tile published counts and tile descriptors of the radix passes
  uint32_t* dtot_app = nullptr;      // [2 passes, 1 row, 256] pass(es) over the application ids (one segment)
  uint32_t* dtot_key = nullptr;      // [kMaxSortPasses, tiles_cap, 256] passes inside the applications' ranges
  int64_t tiles_cap = 0;             // rows per pass slab of dtot_key, tiles of sort_state and sort_desc
  unsigned long long* sort_state = nullptr;   // [tiles_cap, 256] generation-tagged words of the running pass
  int4* sort_desc = nullptr;         // [tiles_cap]
  uint32_t sort_gen = 0;             // generations handed out so far
  int32_t* seg1 = nullptr;           // [2] the one-segment plan of the pass over the application ids
  float2* dw_g[2] = {nullptr, nullptr};   // [n] (deadline, weight) at each grouped position (two for two passes over the ids)
  State* h_state = nullptr;   // pinned mirror
  bool scored = false;
  int32_t n = 0;
  int32_t rounds_done = 0;
  bool done = false;
  size_t score_lds = 0;
  int mfma_D = 0;             // > 0: logistic heads run on the matrix-core kernel with this padded feature width
  unsigned char* blocks = nullptr;   // packed (application, class tile) blocks for that kernel
  int64_t* block_off = nullptr;      // [A] byte offsets
  float* w_unscale = nullptr;        // [A] 2^-ew of each application's weight scaling
  bool mlp_bf16 = false;             // bf16 MLP heads run on the matrix-core MLP kernel
  unsigned char* w1p = nullptr;      // packed layer-1 slices for that kernel
  int64_t* w1_off = nullptr;         // [A] byte offsets
  // all rounds of a chunk in one launch, when every (application, variant) pair fits on the device at once
  bool persist = false;
  bool persist_split = false;        // ... and also with the per-wavefront windows that subgroups need in LDS
  Persist ps{};
  uint32_t gen_base = 0;             // slot generations handed out so far
  int32_t spin_limit = kSpinLimit;   // polls before a wait between resident workgroups is given up
  int32_t sort_spin_limit = kSortSpinLimit;   // polls before a radix pass's look-back is given up (< 0: at once)
  long long* h_ticks = nullptr;      // pinned mirror of ps.ticks
  double tick_ms = 0.0;              // milliseconds per timestamp tick
  std::vector<float> round_ms;       // per-round latencies of the last timed sp_schedule on that path
  int32_t rounds_in_call = 0;        // rounds the last sp_schedule call committed
  // host copies needed to fold a prior into the expected accuracies (sp_set_prior)
  std::vector<float> h_acc;
  std::vector<int32_t> h_acc_off, h_ncls, h_nmod;
  float* d_ea_gain = nullptr;
  float* d_ea_bias = nullptr;
  float* d_swap = nullptr;
  // data-aware group splitting (Sec. 5.3.2): one slot per possible (application, subgroup code)
  int32_t n_slots = 0;
  int32_t *slot_app = nullptr, *slot_base = nullptr, *slot_beg = nullptr, *slot_end = nullptr;
  int32_t* h_grp_n = nullptr;        // pinned [2]: number of groups of the scored window, most groups of one application
  hipEvent_t ev_groups = nullptr;    // recorded after the copy into h_grp_n
  int sub_passes = 0;                // 8-bit radix passes over the subgroup codes
  unsigned char* static_scratch = nullptr;   // this device's copy of the static scratch array (sp_greedy_round_static)
  std::string hip_err;
  // optional stage timing (benchmarks)
  bool timing = false;
  bool timing_stages = false;            // an event after every stage (else only around the scoring kernel)
  bool timing_rounds = false;
  bool timed_score = false, timed_rounds = false;
  hipEvent_t ev[9] = {};                 // group start, score start, score stop, order stop, rounds start, rounds stop,
                                         // finish-order start, copy-outputs start and stop
  bool timed_copy = false;
  std::vector<hipEvent_t> round_ev;      // one after each timed round
  int n_round_ev = 0;
};

constexpr int kMaxRoundEvents = 4096;

// Device memory for sp_greedy_round_static: the per-round exchange buffers of the two round kernels
// (candidate words, group priorities, window positions and sizes), for callers that must not allocate.
// One copy per GPU for the life of the process; `scratch` is only a host-side handle here: its device
// address on each GPU comes from hipGetSymbolAddress (static_scratch_for) and that address is what
// kernels and memory calls get.
constexpr size_t kStaticScratchBytes = (size_t)1 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kStaticMaxDevices = 64;
static unsigned char* g_scratch_ptr[kStaticMaxDevices];   // device address of `scratch` on each GPU seen so far
static std::mutex g_scratch_mu;

namespace {

struct DeviceGuard {
  int prev = -1;
  bool ok = true;
  explicit DeviceGuard(int dev) {
    if (hipGetDevice(&prev) != hipSuccess) prev = -1;
    if (prev != dev) ok = hipSetDevice(dev) == hipSuccess;
  }
  ~DeviceGuard() {
    if (prev >= 0) (void)hipSetDevice(prev);
  }
};

#define SP_HIP(ctx, call)                                                          \
  do {                                                                             \
    hipError_t e_ = (call);                                                        \
    if (e_ != hipSuccess) {                                                        \
      (ctx)->hip_err = std::string(#call) + ": " + hipGetErrorString(e_);          \
      return SP_EDEVICE;                                                           \
    }                                                                              \
  } while (0)

template <typename T>
sp_status dev_alloc(sp_ctx* c, T** out, size_t count) {
  void* p = nullptr;
  size_t bytes = (count ? count : 1) * sizeof(T);
  hipError_t e = hipMalloc(&p, bytes);
  if (e != hipSuccess) {
    c->hip_err = std::string("hipMalloc: ") + hipGetErrorString(e);
    return e == hipErrorOutOfMemory ? SP_ENOMEM : SP_EDEVICE;
  }
  c->dev_allocs.push_back(p);
  *out = (T*)p;
  return SP_OK;
}

template <typename T>
sp_status dev_upload(sp_ctx* c, T** out, const std::vector<T>& host) {
  sp_status s = dev_alloc(c, out, host.size());
  if (s != SP_OK) return s;
  if (!host.empty()) SP_HIP(c, hipMemcpy(*out, host.data(), host.size() * sizeof(T), hipMemcpyHostToDevice));
  return SP_OK;
}

int app_passes(int A) { return (A + 1 <= 256) ? 1 : ((A + 1 <= 65536) ? 2 : 3); }

sp_status validate_profile(const sp_profile* p) {
  if (!p || !p->n_classes || !p->n_models || !p->W1 || !p->b1 || !p->acc || !p->lat_ms || !p->penalty)
    return SP_EINVAL;
  if (p->n_apps < 1 || p->feat_dim < 1 || p->hidden_dim < 0 || p->max_batch < 1 || p->max_requests < 0)
    return SP_EINVAL;
  if (p->feat_dtype != SP_F32 && p->feat_dtype != SP_BF16) return SP_EINVAL;
  if (!(p->prio_timescale_ms > 0.f) || !std::isfinite(p->prio_timescale_ms)) return SP_EINVAL;
  if (p->hidden_dim > 0 && (!p->W2 || !p->b2)) return SP_EINVAL;
  if (p->n_apps > SP_MAX_APPS || p->max_batch > SP_MAX_BATCH) return SP_ECAPACITY;
  for (int a = 0; a < p->n_apps; ++a) {
    const int C = p->n_classes[a], M = p->n_models[a];
    if (C < 1 || M < 1) return SP_EINVAL;
    if (M > SP_MAX_MODELS) return SP_ECAPACITY;
    if (!p->W1[a] || !p->b1[a] || !p->acc[a] || !p->lat_ms[a]) return SP_EINVAL;
    if (p->hidden_dim > 0 && (!p->W2[a] || !p->b2[a])) return SP_EINVAL;
    if (p->penalty[a] < SP_PEN_STEP || p->penalty[a] > SP_PEN_SIGMOID) return SP_EINVAL;
    for (int i = 0; i < M * C; ++i) {
      const float v = p->acc[a][i];
      if (!(v >= 0.f && v <= 1.f)) return SP_EINVAL;
    }
    for (int m = 0; m < M; ++m)
      for (int b = 0; b < p->max_batch; ++b) {
        const float v = p->lat_ms[a][m * p->max_batch + b];
        if (!(v >= 0.f) || !std::isfinite(v)) return SP_EINVAL;
        if (b > 0 && v < p->lat_ms[a][m * p->max_batch + b - 1]) return SP_EINVAL;
      }
  }
  return SP_OK;
}

template <typename T>
sp_status upload_heads(sp_ctx* c, const sp_profile* p) {
  const int A = p->n_apps, d = p->feat_dim, H = p->hidden_dim;
  std::vector<T> W1, W2;
  std::vector<float> b1, b2;
  std::vector<int64_t> W1o(A), W2o(A, 0);
  std::vector<int32_t> b1o(A), b2o(A, 0);
  for (int a = 0; a < A; ++a) {
    const int C = p->n_classes[a];
    const int out1 = H > 0 ? H : C;
    W1o[a] = (int64_t)W1.size();
    b1o[a] = (int32_t)b1.size();
    const T* w1 = (const T*)p->W1[a];
    W1.insert(W1.end(), w1, w1 + (size_t)d * out1);
    b1.insert(b1.end(), p->b1[a], p->b1[a] + out1);
    if (H > 0) {
      W2o[a] = (int64_t)W2.size();
      b2o[a] = (int32_t)b2.size();
      const T* w2 = (const T*)p->W2[a];
      W2.insert(W2.end(), w2, w2 + (size_t)H * C);
      b2.insert(b2.end(), p->b2[a], p->b2[a] + C);
    }
  }
  sp_status s;
  T *dW1, *dW2;
  float *db1, *db2;
  int64_t *dW1o, *dW2o;
  int32_t *db1o, *db2o;
  if ((s = dev_upload(c, &dW1, W1)) != SP_OK) return s;
  if ((s = dev_upload(c, &dW2, W2)) != SP_OK) return s;
  if ((s = dev_upload(c, &db1, b1)) != SP_OK) return s;
  if ((s = dev_upload(c, &db2, b2)) != SP_OK) return s;
  if ((s = dev_upload(c, &dW1o, W1o)) != SP_OK) return s;
  if ((s = dev_upload(c, &dW2o, W2o)) != SP_OK) return s;
  if ((s = dev_upload(c, &db1o, b1o)) != SP_OK) return s;
  if ((s = dev_upload(c, &db2o, b2o)) != SP_OK) return s;
  c->tb.W1 = dW1; c->tb.W2 = dW2; c->tb.b1 = db1; c->tb.b2 = db2;
  c->tb.W1_off = dW1o; c->tb.W2_off = dW2o; c->tb.b1_off = db1o; c->tb.b2_off = db2o;
  return SP_OK;
}

sp_status pack_mfma_blocks(sp_ctx* c, const sp_profile* p);
sp_status pack_mlp_blocks(sp_ctx* c, const sp_profile* p);
sp_status setup_persist(sp_ctx* c, const sp_profile* p);
sp_status ensure_split_buffers(sp_ctx* c);
int score_tile(const sp_ctx* c);

sp_status build_ctx(sp_ctx* c, const sp_profile* p) {
  const int A = p->n_apps, B = p->max_batch;
  c->A = A; c->d = p->feat_dim; c->H = p->hidden_dim; c->B = B; c->dtype = p->feat_dtype;
  c->cap = p->max_requests;
  int Mmax = 0, Cmax = 0;
  for (int a = 0; a < A; ++a) {
    Mmax = std::max(Mmax, p->n_models[a]);
    Cmax = std::max(Cmax, p->n_classes[a]);
  }
  c->Mmax = Mmax; c->Cmax = Cmax;
  c->score_lds = (size_t)kScoreWaves * kScoreRW * (size_t)(c->d + c->H) * sizeof(float);
  if (c->score_lds > 160 * 1024) return SP_ECAPACITY;

  Tables& tb = c->tb;
  tb.A = A; tb.d = c->d; tb.H = c->H; tb.B = B; tb.Mmax = Mmax; tb.Cmax = Cmax; tb.dtype = c->dtype;
  tb.inv_timescale = 1.0f / p->prio_timescale_ms;
  tb.pol_edf = tb.pol_group_first = tb.pol_whole = tb.pol_max_accuracy = tb.pol_unit_weight = 0;
  tb.Bcap = B;
  sp_status s;
  std::vector<int32_t> ncls(p->n_classes, p->n_classes + A), nmod(p->n_models, p->n_models + A),
      pen(p->penalty, p->penalty + A), acc_off(A);
  std::vector<float> acc, lat((size_t)A * Mmax * B, 0.f), lmin(A);
  for (int a = 0; a < A; ++a) {
    const int C = ncls[a], M = nmod[a];
    acc_off[a] = (int32_t)acc.size();
    acc.insert(acc.end(), p->acc[a], p->acc[a] + (size_t)M * C);
    float lm = p->lat_ms[a][0];
    for (int m = 0; m < M; ++m) {
      lm = std::min(lm, p->lat_ms[a][m * B]);
      for (int b = 0; b < B; ++b) lat[((size_t)a * Mmax + m) * B + b] = p->lat_ms[a][m * B + b];
    }
    lmin[a] = lm;
  }
  int32_t *d_ncls, *d_nmod, *d_pen, *d_acc_off;
  float *d_acc, *d_lat, *d_lmin;
  if ((s = dev_upload(c, &d_ncls, ncls)) != SP_OK) return s;
  if ((s = dev_upload(c, &d_nmod, nmod)) != SP_OK) return s;
  if ((s = dev_upload(c, &d_pen, pen)) != SP_OK) return s;
  if ((s = dev_upload(c, &d_acc_off, acc_off)) != SP_OK) return s;
  if ((s = dev_upload(c, &d_acc, acc)) != SP_OK) return s;
  if ((s = dev_upload(c, &d_lat, lat)) != SP_OK) return s;
  if ((s = dev_upload(c, &d_lmin, lmin)) != SP_OK) return s;
  tb.n_classes = d_ncls; tb.n_models = d_nmod; tb.penalty = d_pen; tb.acc_off = d_acc_off;
  tb.acc = d_acc; tb.lat = d_lat; tb.lmin = d_lmin;
  // no prior: gain 1, bias 0
  c->h_acc = acc; c->h_acc_off = acc_off; c->h_ncls = ncls; c->h_nmod = nmod;
  {
    std::vector<float> gain((size_t)A, 1.0f), bias((size_t)A * Mmax, 0.0f);
    if ((s = dev_upload(c, &c->d_ea_gain, gain)) != SP_OK) return s;
    if ((s = dev_upload(c, &c->d_ea_bias, bias)) != SP_OK) return s;
    tb.ea_gain = c->d_ea_gain; tb.ea_bias = c->d_ea_bias;
    if ((s = dev_upload(c, &c->d_swap, bias)) != SP_OK) return s;      // no swap-in costs
    tb.swap = c->d_swap;
  }
  s = (c->dtype == SP_BF16) ? upload_heads<uint16_t>(c, p) : upload_heads<float>(c, p);
  if (s != SP_OK) return s;
  if (c->H == 0 && c->dtype == SP_F32 && c->d <= 256) {
    c->mfma_D = c->d <= 64 ? 64 : (c->d <= 128 ? 128 : 256);
    if ((s = pack_mfma_blocks(c, p)) != SP_OK) return s;
  } else if (c->H > 0 && c->H <= kMlpH && c->dtype == SP_BF16 && (c->d % 8) == 0) {
    c->mlp_bf16 = true;
    if ((s = pack_mlp_blocks(c, p)) != SP_OK) return s;
  }

  // window buffers
  const size_t N = (size_t)c->cap;
  Window& w = c->w;
  if ((s = dev_alloc(c, &w.seg, A + 2)) != SP_OK) return s;
  if ((s = dev_alloc(c, &w.tile_start, A + 1)) != SP_OK) return s;
  if ((s = dev_alloc(c, &w.unit_start, A + 1)) != SP_OK) return s;
  if ((s = dev_alloc(c, &w.tile_desc, (size_t)c->cap / score_tile(c) + A + 1)) != SP_OK) return s;
  if ((s = dev_alloc(c, &w.ea, N * Mmax)) != SP_OK) return s;
  if ((s = dev_alloc(c, &w.key, N)) != SP_OK) return s;
  if ((s = dev_alloc(c, &w.D_s, N + 16)) != SP_OK) return s;      // +16: the window scan reads whole 16-groups
  if ((s = dev_alloc(c, &w.w_s, N)) != SP_OK) return s;
  if ((s = dev_alloc(c, &w.key_s, N)) != SP_OK) return s;
  if ((s = dev_alloc(c, &w.alive_s, N + 16)) != SP_OK) return s;
  if ((s = dev_alloc(c, &w.head, 2 * (size_t)A)) != SP_OK) return s;
  w.gcap = A;
  w.sub_g = nullptr;
  if ((s = dev_alloc(c, &w.grp_app, A)) != SP_OK) return s;
  if ((s = dev_alloc(c, &w.grp_end, A)) != SP_OK) return s;
  if ((s = dev_alloc(c, &w.grp_n, 2)) != SP_OK) return s;
  if ((s = dev_alloc(c, &w.model, N)) != SP_OK) return s;
  if ((s = dev_alloc(c, &w.round_of, N)) != SP_OK) return s;
  if ((s = dev_alloc(c, &w.order_of, N)) != SP_OK) return s;
  if ((s = dev_alloc(c, &w.util, N)) != SP_OK) return s;
  if ((s = dev_alloc(c, &w.cand, (size_t)A * Mmax)) != SP_OK) return s;
  if ((s = dev_alloc(c, &w.cand_prio, (size_t)A * Mmax)) != SP_OK) return s;
  if ((s = dev_alloc(c, &w.win_pos, (size_t)A * B)) != SP_OK) return s;
  if ((s = dev_alloc(c, &w.win_n, A)) != SP_OK) return s;
  w.log_cap = (int32_t)std::max<size_t>(N, 1);
  if ((s = dev_alloc(c, &w.log, (size_t)w.log_cap)) != SP_OK) return s;
  if ((s = dev_alloc(c, &w.last_ids, B)) != SP_OK) return s;
  if ((s = dev_alloc(c, &w.st, 1)) != SP_OK) return s;
  for (int i = 0; i < 2; ++i)
    if ((s = dev_alloc(c, &c->bufK[i], N)) != SP_OK) return s;
  for (int i = 0; i < 3; ++i)
    if ((s = dev_alloc(c, &c->bufV[i], N)) != SP_OK) return s;
  if ((s = dev_alloc(c, &w.id_s, N)) != SP_OK) return s;
  if ((s = dev_alloc(c, &w.rec_g, N)) != SP_OK) return s;
  c->tiles_cap = (int64_t)(N / kSortTile) + A + 2;
  if ((s = dev_alloc(c, &c->dtot_app, 2 * 256)) != SP_OK) return s;
  if ((s = dev_alloc(c, &c->dtot_key, (size_t)kMaxSortPasses * c->tiles_cap * 256)) != SP_OK) return s;
  if ((s = dev_alloc(c, &c->sort_state, (size_t)c->tiles_cap * 256)) != SP_OK) return s;
  SP_HIP(c, hipMemset(c->sort_state, 0, (size_t)c->tiles_cap * 256 * sizeof(unsigned long long)));
  if ((s = dev_alloc(c, &c->sort_desc, (size_t)c->tiles_cap)) != SP_OK) return s;
  if ((s = dev_alloc(c, &c->seg1, 2)) != SP_OK) return s;
  for (int i = 0; i < (app_passes(A) > 1 ? 2 : 1); ++i)
    if ((s = dev_alloc(c, &c->dw_g[i], N)) != SP_OK) return s;
  SP_HIP(c, hipHostMalloc((void**)&c->h_state, sizeof(State), hipHostMallocDefault));
  std::memset(c->h_state, 0, sizeof(State));
  {
    void* dp = nullptr;
    SP_HIP(c, hipHostGetDevicePointer(&dp, c->h_state, 0));
    c->w.st_host = (State*)dp;
  }
  SP_HIP(c, hipMemset(w.st, 0, sizeof(State)));
  if ((s = setup_persist(c, p)) != SP_OK) return s;
  if (c->score_lds > 64 * 1024) {
    const int bytes = (int)c->score_lds;
#define SP_SET_LDS(T, MT) \
    SP_HIP(c, hipFuncSetAttribute((const void*)k_score_generic<T, MT>, hipFuncAttributeMaxDynamicSharedMemorySize, bytes))
    SP_SET_LDS(float, 4); SP_SET_LDS(float, 8); SP_SET_LDS(float, 16);
    SP_SET_LDS(uint16_t, 4); SP_SET_LDS(uint16_t, 8); SP_SET_LDS(uint16_t, 16);
#undef SP_SET_LDS
  }
  return SP_OK;
}

template <int D>
sp_status pack_mfma_blocks_d(sp_ctx* c, const sp_profile* p) {
  using SB = SplitBlock<D>;
  std::vector<int64_t> off(p->n_apps);
  std::vector<float> unscale(p->n_apps);
  size_t total = 0;
  for (int a = 0; a < p->n_apps; ++a) {
    off[a] = (int64_t)total;
    total += (size_t)((p->n_classes[a] + kClassTile - 1) / kClassTile) * SB::kBytes;
  }
  std::vector<unsigned char> host(total);
  for (int a = 0; a < p->n_apps; ++a)
    unscale[a] = pack_split_blocks<D, kMapRows>((const float*)p->W1[a], p->b1[a], p->acc[a], p->feat_dim, p->n_classes[a],
                                      p->n_models[a], host.data() + off[a]);
  sp_status s;
  if ((s = dev_upload(c, &c->blocks, host)) != SP_OK) return s;
  if ((s = dev_upload(c, &c->block_off, off)) != SP_OK) return s;
  if ((s = dev_upload(c, &c->w_unscale, unscale)) != SP_OK) return s;
  return SP_OK;
}

// bf16 MLP heads: layer-1 slices as they are, layer 2 + table + bias as split blocks over the hidden units
sp_status pack_mlp_blocks(sp_ctx* c, const sp_profile* p) {
  using SB = SplitBlock<kMlpH>;
  const int A = p->n_apps, d = p->feat_dim, H = p->hidden_dim;
  const int nkc = (d + kL1Chunk - 1) / kL1Chunk;
  std::vector<int64_t> off1(A), off2(A);
  std::vector<float> unscale(A);
  size_t tot2 = 0;
  for (int a = 0; a < A; ++a) {
    off1[a] = (int64_t)((size_t)a * mlp_layer1_bytes(d));
    off2[a] = (int64_t)tot2;
    tot2 += (size_t)((p->n_classes[a] + kClassTile - 1) / kClassTile) * SB::kBytes;
  }
  std::vector<unsigned char> h1((size_t)A * mlp_layer1_bytes(d), 0), h2(tot2);
  std::vector<float> w2f;
  for (int a = 0; a < A; ++a) {
    pack_mlp_layer1((const uint16_t*)p->W1[a], d, H, reinterpret_cast<uint16_t*>(h1.data() + off1[a]));
    std::memcpy(h1.data() + off1[a] + (size_t)nkc * kL1Units * 16, p->b1[a], (size_t)H * sizeof(float));
    const int C = p->n_classes[a];
    const uint16_t* w2 = (const uint16_t*)p->W2[a];
    w2f.resize((size_t)H * C);
    for (size_t i = 0; i < w2f.size(); ++i) {
      const uint32_t bits = (uint32_t)w2[i] << 16;
      std::memcpy(&w2f[i], &bits, 4);
    }
    unscale[a] = pack_split_blocks<kMlpH, kMapTile>(w2f.data(), p->b2[a], p->acc[a], H, C, p->n_models[a],
                                                    h2.data() + off2[a]);
  }
  sp_status s;
  if ((s = dev_upload(c, &c->w1p, h1)) != SP_OK) return s;
  if ((s = dev_upload(c, &c->w1_off, off1)) != SP_OK) return s;
  if ((s = dev_upload(c, &c->blocks, h2)) != SP_OK) return s;
  if ((s = dev_upload(c, &c->block_off, off2)) != SP_OK) return s;
  if ((s = dev_upload(c, &c->w_unscale, unscale)) != SP_OK) return s;
  return SP_OK;
}


// The one-launch rounds path needs every (application, variant) pair plus the commit workgroup resident at
// once; contexts too large for that keep the two-kernels-per-round path.
sp_status setup_persist(sp_ctx* c, const sp_profile* p) {
  c->persist = false;
  const int A = p->n_apps;
  std::vector<int32_t> pa, pm;
  {
    // Which pair a workgroup takes.  Consecutive workgroup ids go to the chip's eight dies in turn, each
    // with an L2 of its own, and the variants of an application gather the same rows (deadline, key, the
    // request's line of expected accuracies): the pairs, application-major, are dealt to the dies in
    // contiguous runs, so that an application's variants share one L2 (two where a run ends inside it).
    std::vector<int32_t> na, nm;
    for (int a = 0; a < A; ++a)
      for (int m = 0; m < p->n_models[a]; ++m) { na.push_back(a); nm.push_back(m); }
    const size_t np = na.size();
    pa.resize(np); pm.resize(np);
    size_t next = 0;
    for (size_t x = 0; x < (size_t)kXcds; ++x)
      for (size_t b = x; b < np; b += kXcds, ++next) { pa[b] = na[next]; pm[b] = nm[next]; }
  }
  const size_t n_pairs = pa.size();
  const size_t ring = (size_t)kPersistRounds * A * c->B;
  if (n_pairs == 0 || n_pairs > (size_t)kMaxPairs || ring > ((size_t)32 << 20)) return SP_OK;
  int cus = 0, per_cu = 0, rate_khz = 0;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, c->device) != hipSuccess) return SP_OK;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, k_rounds_persistent<false>, kRoundThreads, 0) != hipSuccess) {
    (void)hipGetLastError();
    return SP_OK;
  }
  if ((size_t)per_cu * (size_t)cus < n_pairs + 2) return SP_OK;
  if (hipDeviceGetAttribute(&rate_khz, hipDeviceAttributeWallClockRate, c->device) != hipSuccess || rate_khz <= 0)
    rate_khz = 100000;
  c->tick_ms = 1.0 / (double)rate_khz;
  Persist& ps = c->ps;
  int32_t *d_pa = nullptr, *d_pm = nullptr;
  sp_status s;
  if ((s = dev_upload(c, &d_pa, pa)) != SP_OK) return s;
  if ((s = dev_upload(c, &d_pm, pm)) != SP_OK) return s;
  ps.pair_app = d_pa; ps.pair_model = d_pm; ps.n_pairs = (int32_t)n_pairs;
  if ((s = dev_alloc(c, &ps.slots, 8 * n_pairs)) != SP_OK) return s;
  if ((s = dev_alloc(c, &ps.ring, ring)) != SP_OK) return s;
  if ((s = dev_alloc(c, &ps.dec, kPersistRounds)) != SP_OK) return s;
  if ((s = dev_alloc(c, &ps.decision, 8)) != SP_OK) return s;
  SP_HIP(c, hipMemset(ps.decision, 0, 8 * 8));
  if ((s = dev_alloc(c, &ps.ticks, kPersistRounds + 1)) != SP_OK) return s;
  SP_HIP(c, hipMemset(ps.slots, 0, 8 * n_pairs * 8));
  SP_HIP(c, hipMemset(ps.ring, 0, ring * 8));
  SP_HIP(c, hipMemset(ps.dec, 0, kPersistRounds * 8));
  SP_HIP(c, hipMemset(ps.ticks, 0, (kPersistRounds + 1) * 8));
  SP_HIP(c, hipHostMalloc((void**)&c->h_ticks, (kPersistRounds + 1) * sizeof(long long), hipHostMallocDefault));
  c->gen_base = 0;
  c->persist = true;
  return SP_OK;
}

// LDS the resident rounds kernel needs beyond its static arrays: with subgroups, B window entries and B
// positions per wavefront.
size_t persist_dynamic_lds(const sp_ctx* c) {
  return c->tb.pol_split ? (size_t)(kRoundThreads / 64) * (size_t)c->B * (sizeof(float4) + sizeof(int32_t)) : 0;
}

// Whether sp_schedule runs the rounds of the scored window in one launch: the resident grid fits the device,
// and with subgroups no application has more groups than a resident workgroup serves (known once the
// window's groups have been counted on the device).
bool rounds_in_one_launch(sp_ctx* c) {
  if (!c->persist) return false;
  if (!c->tb.pol_split) return true;
  if (!c->persist_split) return false;
  if (!c->scored) return true;
  (void)hipEventSynchronize(c->ev_groups);
  return c->h_grp_n[1] <= kMaxAppGroups;
}

void fill_u64(hipStream_t s, unsigned long long* p, size_t n) {
  hipLaunchKernelGGL(k_fill_u64, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, p, (int64_t)n, 0ull);
}

// Up to kPersistRounds rounds in one launch.  An ordinary launch: setup_persist has checked that the whole
// grid fits on the device at once, and the kernel's waits are bounded.
sp_status launch_rounds_persistent(sp_ctx* c, hipStream_t s, int n_rounds) {
  Persist& ps = c->ps;
  if (c->gen_base + (uint32_t)n_rounds + 2u >= kGenMask) {       // generation numbers about to wrap: start over
    fill_u64(s, ps.slots, 8 * (size_t)ps.n_pairs);
    fill_u64(s, ps.decision, 8);
    fill_u64(s, ps.ring, (size_t)kPersistRounds * c->A * c->B);
    c->gen_base = 0;
  }
  ps.n_rounds = n_rounds;
  ps.all_to_all = ps.n_pairs <= kAllToAllPairs ? 1 : 0;
  ps.spin_limit = c->spin_limit;
  ps.gen_base = c->gen_base;
  c->gen_base += (uint32_t)n_rounds;
  if (c->tb.pol_split)
    hipLaunchKernelGGL(k_rounds_persistent<true>, dim3(ps.n_pairs + 2), dim3(kRoundThreads), persist_dynamic_lds(c), s, c->tb, c->w, ps);
  else
    hipLaunchKernelGGL(k_rounds_persistent<false>, dim3(ps.n_pairs + 2), dim3(kRoundThreads), 0, s, c->tb, c->w, ps);
  return SP_OK;
}

// Buffers of the group-splitting mode (Sec. 5.3.2), allocated the first time it is switched on: the subgroup
// code of every request, one slot per possible (application, code) pair, and per-group arrays large enough
// for every non-empty pair.
sp_status ensure_split_buffers(sp_ctx* c) {
  if (c->w.sub_g) return SP_OK;
  const int A = c->A;
  int64_t slots = 0;
  std::vector<int32_t> base(A), app_of;
  int cmax = 0;
  for (int a = 0; a < A; ++a) {
    base[a] = (int32_t)slots;
    slots += c->h_ncls[a] + 1;
    cmax = std::max(cmax, c->h_ncls[a]);
    if (slots > 65536) return SP_ECAPACITY;
  }
  app_of.reserve((size_t)slots);
  for (int a = 0; a < A; ++a) app_of.insert(app_of.end(), (size_t)c->h_ncls[a] + 1, a);
  c->n_slots = (int32_t)slots;
  c->sub_passes = 1;
  while ((1 << (8 * c->sub_passes)) <= cmax + 1) ++c->sub_passes;
  const size_t gcap = (size_t)std::max<int64_t>(A, std::min<int64_t>(slots, std::max<int64_t>(c->cap, 1)));
  Window& w = c->w;
  sp_status s;
  if ((s = dev_alloc(c, &w.sub_g, (size_t)std::max<int64_t>(c->cap, 1))) != SP_OK) return s;
  if ((s = dev_upload(c, &c->slot_app, app_of)) != SP_OK) return s;
  if ((s = dev_upload(c, &c->slot_base, base)) != SP_OK) return s;
  if ((s = dev_alloc(c, &c->slot_beg, (size_t)slots)) != SP_OK) return s;
  if ((s = dev_alloc(c, &c->slot_end, (size_t)slots)) != SP_OK) return s;
  // per-group arrays at the larger capacity (the old ones stay allocated until the context goes)
  SP_HIP(c, hipDeviceSynchronize());
  if ((s = dev_alloc(c, &w.grp_app, gcap)) != SP_OK) return s;
  if ((s = dev_alloc(c, &w.grp_end, gcap)) != SP_OK) return s;
  if ((s = dev_alloc(c, &w.head, 2 * gcap)) != SP_OK) return s;
  if ((s = dev_alloc(c, &w.cand, gcap * c->Mmax)) != SP_OK) return s;
  if ((s = dev_alloc(c, &w.cand_prio, gcap * c->Mmax)) != SP_OK) return s;
  if ((s = dev_alloc(c, &w.win_pos, gcap * c->B)) != SP_OK) return s;
  if ((s = dev_alloc(c, &w.win_n, gcap)) != SP_OK) return s;
  w.gcap = (int32_t)gcap;
  SP_HIP(c, hipHostMalloc((void**)&c->h_grp_n, 2 * sizeof(int32_t), hipHostMallocDefault));
  c->h_grp_n[0] = A;
  c->h_grp_n[1] = 1;
  SP_HIP(c, hipEventCreate(&c->ev_groups));
  return SP_OK;
}

sp_status pack_mfma_blocks(sp_ctx* c, const sp_profile* p) {
  switch (c->mfma_D) {
    case 64: return pack_mfma_blocks_d<64>(c, p);
    case 128: return pack_mfma_blocks_d<128>(c, p);
    default: return pack_mfma_blocks_d<256>(c, p);
  }
}

template <typename T>
void launch_score_generic(sp_ctx* c, hipStream_t s, int grid, const void* x, const int32_t* ids, const float2* dw,
                          uint32_t* sortkey, float* logits) {
  const dim3 blk(kScoreWaves * kWave);
  if (c->Mmax <= 4)
    hipLaunchKernelGGL((k_score_generic<T, 4>), dim3(grid), blk, c->score_lds, s, c->tb, c->w, (const T*)x, ids, dw, sortkey, logits);
  else if (c->Mmax <= 8)
    hipLaunchKernelGGL((k_score_generic<T, 8>), dim3(grid), blk, c->score_lds, s, c->tb, c->w, (const T*)x, ids, dw, sortkey, logits);
  else
    hipLaunchKernelGGL((k_score_generic<T, 16>), dim3(grid), blk, c->score_lds, s, c->tb, c->w, (const T*)x, ids, dw, sortkey, logits);
}

int score_tile(const sp_ctx* c) { return (c->mfma_D > 0 || c->mlp_bf16) ? kMfTile : kScoreTile; }

// Address of the static scratch array on `device` (which must be current), looked up once per device.
sp_status static_scratch_for(sp_ctx* c, int device, unsigned char** out) {
  if (device < 0 || device >= kStaticMaxDevices) return SP_ECAPACITY;
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[device]) {
    void* p = nullptr;
    SP_HIP(c, hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return SP_EDEVICE;
    g_scratch_ptr[device] = (unsigned char*)p;
  }
  *out = g_scratch_ptr[device];
  return SP_OK;
}

constexpr size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

void launch_score(sp_ctx* c, hipStream_t s, const void* x, const int32_t* ids, const float2* dw, uint32_t* sortkey,
                  float* logits) {
  if (c->mlp_bf16) {
    const int grid = (c->n + kMfTile - 1) / kMfTile + c->A + kXcds;   // at least 8 * ceil(tiles / 8): see xcd_tile
#define SP_LAUNCH_MLP(DUMP, SPLIT)                                                                                \
    hipLaunchKernelGGL((k_score_mlp_bf16<DUMP, SPLIT>), dim3(grid), dim3(kMfThreads), 0, s, c->tb, c->w,          \
                       (const uint16_t*)x, ids, dw, sortkey, (const unsigned char*)c->w1p,                       \
                       (const int64_t*)c->w1_off, (const unsigned char*)c->blocks, (const int64_t*)c->block_off, \
                       (const float*)c->w_unscale, logits)
    if (logits) SP_LAUNCH_MLP(true, false);
    else if (c->tb.pol_split) SP_LAUNCH_MLP(false, true);
    else SP_LAUNCH_MLP(false, false);
#undef SP_LAUNCH_MLP
    return;
  }
  if (c->mfma_D > 0) {
    const int grid = (c->n + kMfTile - 1) / kMfTile + c->A + kXcds;   // at least 8 * ceil(tiles / 8): see xcd_tile
    const dim3 blk(kMfThreads);
#define SP_LAUNCH_MF(DD)                                                                                          \
    do {                                                                                                          \
      if (logits)                                                                                                 \
        hipLaunchKernelGGL((k_score_logistic_split<DD, true, false>), dim3(grid), blk, 0, s, c->tb, c->w,         \
                           (const float*)x, ids, dw, sortkey, (const unsigned char*)c->blocks,                    \
                           (const int64_t*)c->block_off, (const float*)c->w_unscale, logits);                     \
      else if (c->tb.pol_split)                                                                                   \
        hipLaunchKernelGGL((k_score_logistic_split<DD, false, true>), dim3(grid), blk, 0, s, c->tb, c->w,         \
                           (const float*)x, ids, dw, sortkey, (const unsigned char*)c->blocks,                    \
                           (const int64_t*)c->block_off, (const float*)c->w_unscale, logits);                     \
      else                                                                                                        \
        hipLaunchKernelGGL((k_score_logistic_split<DD, false, false>), dim3(grid), blk, 0, s, c->tb, c->w,        \
                           (const float*)x, ids, dw, sortkey, (const unsigned char*)c->blocks,                    \
                           (const int64_t*)c->block_off, (const float*)c->w_unscale, logits);                     \
    } while (0)
    if (c->mfma_D == 64) SP_LAUNCH_MF(64);
    else if (c->mfma_D == 128) SP_LAUNCH_MF(128);
    else SP_LAUNCH_MF(256);
#undef SP_LAUNCH_MF
    return;
  }
  const int grid = (c->n + kScoreTile - 1) / kScoreTile + c->A;
  if (c->dtype == SP_BF16)
    launch_score_generic<uint16_t>(c, s, grid, x, ids, dw, sortkey, logits);
  else
    launch_score_generic<float>(c, s, grid, x, ids, dw, sortkey, logits);
}

// One stable radix pass over the tiles of `plan`; (keys, vals) -> (keys_out, vals_out).
void radix_pass(sp_ctx* c, hipStream_t s, const SortPlan& plan, int tiles, const uint32_t* keys, const int32_t* vals,
                int shift, int clamp_a, const uint32_t* dtot_pass, uint32_t* keys_out, int32_t* vals_out,
                const SegArgs* fused_segments = nullptr, const SortCarry* carry = nullptr) {
  if (c->sort_gen == 0xFFFFFFFFu) {                       // generation numbers about to wrap: start over
    hipLaunchKernelGGL(k_fill_u64, dim3((unsigned)((c->tiles_cap * 256 + 255) / 256)), dim3(256), 0, s, c->sort_state,
                       (int64_t)c->tiles_cap * 256, 0ull);
    c->sort_gen = 0;
  }
  const uint32_t gen = ++c->sort_gen;
  SegArgs sg{};                                            // seg == null: no segment bookkeeping in this launch
  if (fused_segments) sg = *fused_segments;
  if (carry)
    hipLaunchKernelGGL(k_radix_pass<true>, dim3(tiles + (fused_segments ? 1 : 0)), dim3(kSortThreads), 0, s, plan, keys, vals,
                       shift, clamp_a, dtot_pass, c->sort_state, gen, c->sort_spin_limit, keys_out, vals_out, c->w.st, sg, c->w, *carry);
  else
    hipLaunchKernelGGL(k_radix_pass<false>, dim3(tiles + (fused_segments ? 1 : 0)), dim3(kSortThreads), 0, s, plan, keys, vals,
                       shift, clamp_a, dtot_pass, c->sort_state, gen, c->sort_spin_limit, keys_out, vals_out, c->w.st, sg, c->w,
                       SortCarry{});
}

// Number of groups of the scored window: the applications, or the non-empty (application, subgroup) pairs.
int group_count(sp_ctx* c) {
  if (!c->tb.pol_split) return c->A;
  (void)hipEventSynchronize(c->ev_groups);
  return std::max(1, (int)*c->h_grp_n);
}

void launch_round(sp_ctx* c, const Window& w, hipStream_t s, int32_t* ids_out, float* cube) {
  hipLaunchKernelGGL(k_round_score, dim3(group_count(c) * c->Mmax), dim3(kRoundThreads), 0, s, c->tb, w, cube);
  if (cube == nullptr)
    hipLaunchKernelGGL(k_round_commit, dim3(1), dim3(kRoundThreads), 0, s, c->tb, w, ids_out);
}

// Brings the window state to the host.  mirrored: the last kernel on the stream was k_round_commit, which
// has written the state into the pinned copy itself; otherwise it is copied here.
sp_status fetch_state(sp_ctx* c, hipStream_t s, bool mirrored = false) {
  if (!mirrored) SP_HIP(c, hipMemcpyAsync(c->h_state, c->w.st, sizeof(State), hipMemcpyDeviceToHost, s));
  SP_HIP(c, hipStreamSynchronize(s));
  SP_HIP(c, hipGetLastError());
  c->rounds_done = c->h_state->round;
  c->done = c->h_state->done != 0;
  if (c->h_state->err & kErrSortSync) {
    c->hip_err = "ordering: a look-back between tiles of a radix pass ran out";
    c->scored = false;
    return SP_EDEVICE;
  }
  if (c->h_state->err & kErrSync) {
    // resident workgroups lost each other: leave the exchange buffers clean and stop using that path
    c->hip_err = "rounds kernel: a wait between workgroups ran out";
    fill_u64(s, c->ps.slots, 8 * (size_t)c->ps.n_pairs);
    fill_u64(s, c->ps.dec, kPersistRounds);
    (void)hipStreamSynchronize(s);
    c->persist = false;
    c->scored = false;                 // the window's state is not trustworthy any more: score it again
    return SP_EDEVICE;
  }
  return c->h_state->err ? SP_EINVAL : SP_OK;
}

}  // namespace

extern "C" {

sp_status sp_create(const sp_profile* profile, int device_id, sp_ctx** out) {
  if (!out) return SP_EINVAL;
  *out = nullptr;
  sp_status s = validate_profile(profile);
  if (s != SP_OK) return s;
  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess || device_id < 0 || device_id >= ndev) return SP_EDEVICE;
  sp_ctx* c = new (std::nothrow) sp_ctx();
  if (!c) return SP_ENOMEM;
  c->device = device_id;
  DeviceGuard g(device_id);
  if (!g.ok) {
    delete c;
    return SP_EDEVICE;
  }
  s = build_ctx(c, profile);
  if (s == SP_OK) s = static_scratch_for(c, device_id, &c->static_scratch);
  if (s != SP_OK) {
    sp_destroy(c);
    return s;
  }
  *out = c;
  return SP_OK;
}

void sp_destroy(sp_ctx* c) {
  if (!c) return;
  DeviceGuard g(c->device);
  (void)hipDeviceSynchronize();
  for (void* p : c->dev_allocs) (void)hipFree(p);
  if (c->h_state) (void)hipHostFree(c->h_state);
  if (c->h_ticks) (void)hipHostFree(c->h_ticks);
  if (c->h_grp_n) (void)hipHostFree(c->h_grp_n);
  if (c->ev_groups) (void)hipEventDestroy(c->ev_groups);
  for (hipEvent_t e : c->ev)
    if (e) (void)hipEventDestroy(e);
  for (hipEvent_t e : c->round_ev) (void)hipEventDestroy(e);
  delete c;
}

sp_status sp_score(sp_ctx* c, int32_t n, const void* x_dev, const int32_t* app_dev, const float* deadline_ms_dev,
                   const float* weight_dev, void* stream, float* ea_out_dev, float* key_out_dev) {
  if (!c || n < 0) return SP_EINVAL;
  if (n > 0 && (!x_dev || !app_dev || !deadline_ms_dev || !weight_dev)) return SP_EINVAL;
  if ((int64_t)n > c->cap) return SP_ECAPACITY;
  DeviceGuard g(c->device);
  if (!g.ok) return SP_EDEVICE;
  hipStream_t s = (hipStream_t)stream;
  Window& w = c->w;
  w.n = n;
  c->n = n;
  c->rounds_done = 0;
  c->done = false;
  const int A = c->A;
  hipLaunchKernelGGL(k_reset_state, dim3(1), dim3(256), 0, s, w.st, n, c->seg1, c->dtot_app, 2 * 256);
  const bool tm = c->timing && n > 0;
  c->timed_score = false;
  c->timed_rounds = false;
  const bool tms = tm && c->timing_stages;
  if (tms) SP_HIP(c, hipEventRecord(c->ev[0], s));

  uint32_t *curK = c->bufK[0], *altK = c->bufK[1];
  int32_t *curV = c->bufV[0], *altV = c->bufV[1];
  const int n_app_passes = app_passes(A);
  const int tiles2 = n / kSortTile + A;                       // upper bound on the tiles inside the applications' ranges
  const int64_t slab = c->tiles_cap * 256;                    // words per pass of dtot_key
  // a single pass over the application ids: every application's count is one of its digit totals
  // Applications whose whole range fits one workgroup's LDS are ordered by one kernel (k_sort_small) and get
  // no tiles in the passes; not with subgroups (their passes over the labels need the tiles) and not with more
  // applications than that kernel is worth a workgroup each.
  const int small_cap = (!c->tb.pol_split && A <= 1024) ? kSmallSortCap : 0;
  SegArgs seg_args{n, A, nullptr, c->dtot_app, score_tile(c), kSortTile, small_cap, w.seg, w.tile_start, w.unit_start,
                   w.tile_desc, c->sort_desc};
  if (n > 0) {
    // requests grouped by application: stable pass(es) over the application id, read straight from the
    // caller's array (ids outside [0, A) become A and raise the error flag)
    SortPlan whole{c->seg1, nullptr, 1, nullptr};
    const int tiles1 = (n + kSortTile - 1) / kSortTile;
    hipLaunchKernelGGL(k_digit_totals, dim3(tiles1), dim3(kSortThreads), 0, s, whole, (const uint32_t*)app_dev, A, 0,
                       n_app_passes, (int64_t)1, c->dtot_app, c->dtot_key, kMaxSortPasses, (int64_t)tiles2 + 1, c->tiles_cap,
                       w.st);
    const uint32_t* kin = (const uint32_t*)app_dev;
    const int32_t* vin = nullptr;
    for (int p = 0; p < n_app_passes; ++p) {
      // a single pass: the segment bookkeeping (which needs only the ids' digit totals) rides along;
      // every request's deadline and weight travel with it to its grouped position
      const SortCarry cy = p == 0 ? SortCarry{deadline_ms_dev, weight_dev, nullptr, c->dw_g[n_app_passes - 1 - p]}
                                  : SortCarry{nullptr, nullptr, c->dw_g[n_app_passes - p], c->dw_g[n_app_passes - 1 - p]};
      radix_pass(c, s, whole, tiles1, kin, vin, 8 * p, p == 0 ? A : 0, c->dtot_app + 256 * p, altK, altV,
                 n_app_passes == 1 ? &seg_args : nullptr, &cy);
      std::swap(curK, altK);
      std::swap(curV, altV);
      kin = curK;
      vin = curV;
    }
  }
  if (n == 0 || n_app_passes > 1) {
    // no pass to ride along with, or two passes (the segment starts then come from the sorted ids)
    seg_args.sorted_app = curK;
    seg_args.digit_tot = nullptr;
    hipLaunchKernelGGL(k_segments, dim3(1), dim3(256), 0, s, seg_args, w);
  }
  if (n > 0) {
    // posterior -> EA -> key, one pass over the features
    uint32_t* sortkey = altK;
    if (tm) SP_HIP(c, hipEventRecord(c->ev[1], s));
    launch_score(c, s, x_dev, curV, c->dw_g[0], sortkey, nullptr);
    if (tm) SP_HIP(c, hipEventRecord(c->ev[2], s));
    // service order: inside each application by (key descending, id ascending).  The passes carry
    // positions of the grouped array (identity to start with), the grouped ids stay where they are.
    SortPlan per_app{w.seg, w.unit_start, A, c->sort_desc};
    // with n <= small_cap every application is small: the tiled passes have nothing to do and are not launched
    const bool tiled = !(small_cap > 0 && n <= small_cap);
    if (tiled)
      hipLaunchKernelGGL(k_digit_totals, dim3(tiles2), dim3(kSortThreads), 0, s, per_app, (const uint32_t*)sortkey, 0, 0, 4,
                         c->tiles_cap, c->dtot_key, (uint32_t*)nullptr, 0, (int64_t)0, (int64_t)0, w.st);
    uint32_t *k_in = sortkey, *k_out = curK;
    const int32_t* v_in = nullptr;
    int32_t *v_out = altV, *v_spare = c->bufV[2];
    for (int p = 0; p < 4; ++p) {
      if (tiled) radix_pass(c, s, per_app, tiles2, k_in, v_in, 8 * p, 0, c->dtot_key + slab * p, k_out, v_out);
      std::swap(k_in, k_out);
      v_in = v_out;
      std::swap(v_out, v_spare);
    }
    // the small applications, straight into the arrays the fourth pass has written (or would have)
    if (small_cap > 0)
      hipLaunchKernelGGL(k_sort_small, dim3(A), dim3(kSmallSortThreads), 0, s, (const int32_t*)w.seg, (const uint32_t*)sortkey,
                         k_in, const_cast<int32_t*>(v_in));
    if (c->tb.pol_split) {
      // subgroups: further stable passes over the subgroup codes make the order (subgroup, key) inside
      // every application; then the non-empty (application, subgroup) pairs become the rounds' groups
      hipLaunchKernelGGL(k_gather_sub_keys, dim3((n + 255) / 256), dim3(256), 0, s, A, (const int32_t*)w.seg, v_in,
                         (const int32_t*)w.sub_g, k_in);
      hipLaunchKernelGGL(k_digit_totals, dim3(tiles2), dim3(kSortThreads), 0, s, per_app, (const uint32_t*)k_in, 0, 0,
                         c->sub_passes, c->tiles_cap, c->dtot_key + slab * 4, (uint32_t*)nullptr, 0, (int64_t)0, (int64_t)0, w.st);
      for (int p = 0; p < c->sub_passes; ++p) {
        radix_pass(c, s, per_app, tiles2, k_in, v_in, 8 * p, 0, c->dtot_key + slab * (4 + p), k_out, v_out);
        std::swap(k_in, k_out);
        v_in = v_out;
        std::swap(v_out, v_spare);
      }
    }
    if (tms) SP_HIP(c, hipEventRecord(c->ev[6], s));
    hipLaunchKernelGGL(k_finish_order, dim3((n + 255) / 256), dim3(256), 0, s, n, A, (const int32_t*)w.seg, v_in,
                       (const uint32_t*)k_in, w, c->tb.pol_edf | c->tb.pol_split);
    if (c->tb.pol_split) {
      hipLaunchKernelGGL(k_slot_ranges, dim3((c->n_slots + 255) / 256), dim3(256), 0, s, c->n_slots,
                         (const int32_t*)c->slot_app, (const int32_t*)c->slot_base, (const int32_t*)w.seg,
                         (const uint32_t*)k_in, c->slot_beg, c->slot_end);
      hipLaunchKernelGGL(k_groups_compact, dim3(1), dim3(1024), 0, s, c->n_slots, (const int32_t*)c->slot_app,
                         (const int32_t*)c->slot_beg, (const int32_t*)c->slot_end, w);
    }
    if (tms) SP_HIP(c, hipEventRecord(c->ev[3], s));
    if (tm) c->timed_score = true;
    if (ea_out_dev)
      SP_HIP(c, hipMemcpyAsync(ea_out_dev, w.ea, (size_t)n * c->Mmax * sizeof(float), hipMemcpyDeviceToDevice, s));
    if (key_out_dev)
      SP_HIP(c, hipMemcpyAsync(key_out_dev, w.key, (size_t)n * sizeof(float), hipMemcpyDeviceToDevice, s));
  }
  if (c->tb.pol_split) {
    // the rounds' launch grids depend on the number of groups
    SP_HIP(c, hipMemcpyAsync(c->h_grp_n, w.grp_n, 2 * sizeof(int32_t), hipMemcpyDeviceToHost, s));
    SP_HIP(c, hipEventRecord(c->ev_groups, s));
  }
  SP_HIP(c, hipGetLastError());
  c->scored = true;
  return SP_OK;
}

sp_status sp_greedy_round(sp_ctx* c, void* stream, sp_decision* out_host, int32_t* req_ids_out_dev) {
  if (!c) return SP_EINVAL;
  if (!c->scored) return SP_ESTATE;
  DeviceGuard g(c->device);
  if (!g.ok) return SP_EDEVICE;
  hipStream_t s = (hipStream_t)stream;
  const int32_t before = c->rounds_done;
  launch_round(c, c->w, s, req_ids_out_dev, nullptr);
  sp_status st = fetch_state(c, s, true);
  if (st != SP_OK) return st;
  if (c->rounds_done == before) return SP_DONE;
  if (out_host) std::memcpy(out_host, &c->h_state->last, sizeof(sp_decision));
  return SP_OK;
}

sp_status sp_greedy_round_static(sp_ctx* c, void* stream, sp_decision* out_host, int32_t* req_ids_out_dev) {
  if (!c) return SP_EINVAL;
  if (!c->scored) return SP_ESTATE;
  // the round kernels' exchange buffers, carved out of the static array instead of the context's own
  const size_t G = (size_t)c->w.gcap, GM = G * (size_t)c->Mmax;
  const size_t o_cand = 0, o_prio = o_cand + align256(GM * sizeof(unsigned long long));
  const size_t o_pos = o_prio + align256(GM * sizeof(float));
  const size_t o_n = o_pos + align256(G * (size_t)c->B * sizeof(int32_t));
  const size_t need = o_n + align256(G * sizeof(int32_t));
  if (need > kStaticScratchBytes) {
    c->hip_err = "sp_greedy_round_static: groups x variants x batch sizes exceed the static scratch array";
    return SP_ECAPACITY;
  }
  if (!c->static_scratch) return SP_EDEVICE;
  DeviceGuard g(c->device);
  if (!g.ok) return SP_EDEVICE;
  hipStream_t s = (hipStream_t)stream;
  Window w = c->w;
  unsigned char* base = c->static_scratch;
  w.cand = reinterpret_cast<unsigned long long*>(base + o_cand);
  w.cand_prio = reinterpret_cast<float*>(base + o_prio);
  w.win_pos = reinterpret_cast<int32_t*>(base + o_pos);
  w.win_n = reinterpret_cast<int32_t*>(base + o_n);
  const int32_t before = c->rounds_done;
  launch_round(c, w, s, req_ids_out_dev, nullptr);
  sp_status st = fetch_state(c, s, true);
  if (st != SP_OK) return st;
  if (c->rounds_done == before) return SP_DONE;
  if (out_host) std::memcpy(out_host, &c->h_state->last, sizeof(sp_decision));
  return SP_OK;
}

sp_status sp_schedule(sp_ctx* c, int32_t max_rounds, void* stream, int32_t* model_out_dev, int32_t* round_out_dev,
                      int32_t* order_out_dev, float* util_out_dev, sp_decision* round_log_host,
                      int32_t log_capacity, sp_summary* out_host) {
  if (!c || log_capacity < 0 || (log_capacity > 0 && !round_log_host)) return SP_EINVAL;
  if (!c->scored) return SP_ESTATE;
  DeviceGuard g(c->device);
  if (!g.ok) return SP_EDEVICE;
  hipStream_t s = (hipStream_t)stream;
  const int32_t start = c->rounds_done;
  sp_status st = SP_OK;
  bool fetched = false, outputs_copied = false;
  const bool tm = c->timing && c->timing_stages;
  c->n_round_ev = 0;
  c->timed_rounds = false;
  c->timed_copy = false;
  if (tm) SP_HIP(c, hipEventRecord(c->ev[4], s));
  c->round_ms.clear();
  while (!c->done) {
    const bool persist = rounds_in_one_launch(c);
    int chunk = persist ? kPersistRounds : 64;
    if (max_rounds > 0) chunk = std::min(chunk, start + max_rounds - c->rounds_done);
    if (chunk <= 0) break;
    const int32_t before = c->rounds_done;
    if (persist) {
      if ((st = launch_rounds_persistent(c, s, chunk)) != SP_OK) return st;
      if (tm && c->timing_rounds)
        SP_HIP(c, hipMemcpyAsync(c->h_ticks, c->ps.ticks, (kPersistRounds + 1) * sizeof(long long), hipMemcpyDeviceToHost, s));
    } else {
      for (int i = 0; i < chunk; ++i) {
        launch_round(c, c->w, s, nullptr, nullptr);
        if (tm && c->timing_rounds && c->n_round_ev < kMaxRoundEvents) SP_HIP(c, hipEventRecord(c->round_ev[c->n_round_ev++], s));
      }
    }
    if (tm) SP_HIP(c, hipEventRecord(c->ev[5], s));
    // the per-request outputs go out right behind the rounds, so that the one host synchronisation of
    // fetch_state covers them too (a later chunk simply copies again)
    if (c->n > 0 && (model_out_dev || round_out_dev || order_out_dev || util_out_dev)) {
      const bool tc = tm && !outputs_copied;
      if (tc) SP_HIP(c, hipEventRecord(c->ev[7], s));
      hipLaunchKernelGGL(k_copy_outputs, dim3((c->n + 255) / 256), dim3(256), 0, s, c->n, c->w, model_out_dev,
                         round_out_dev, order_out_dev, util_out_dev);
      if (tc) {
        SP_HIP(c, hipEventRecord(c->ev[8], s));
        c->timed_copy = true;
      }
      outputs_copied = true;
    }
    st = fetch_state(c, s);          // tells how far the device got and whether the queue ran dry
    fetched = true;
    if (st != SP_OK) return st;
    if (persist && tm && c->timing_rounds)
      for (int i = 0; i < c->rounds_done - before; ++i)
        c->round_ms.push_back((float)((double)(c->h_ticks[i + 1] - c->h_ticks[i]) * c->tick_ms));
  }
  if (!fetched && (st = fetch_state(c, s)) != SP_OK) return st;
  c->timed_rounds = tm && fetched;
  c->rounds_in_call = c->rounds_done - start;
  bool pending = false;
  if (c->n > 0 && !outputs_copied && (model_out_dev || round_out_dev || order_out_dev || util_out_dev)) {
    hipLaunchKernelGGL(k_copy_outputs, dim3((c->n + 255) / 256), dim3(256), 0, s, c->n, c->w, model_out_dev,
                       round_out_dev, order_out_dev, util_out_dev);
    pending = true;
  }
  const int32_t n_log = std::min(std::min(c->rounds_done, log_capacity), c->w.log_cap);
  if (n_log > 0) {
    SP_HIP(c, hipMemcpyAsync(round_log_host, c->w.log, (size_t)n_log * sizeof(sp_decision), hipMemcpyDeviceToHost, s));
    pending = true;
  }
  if (pending) SP_HIP(c, hipStreamSynchronize(s));
  if (out_host) {
    const State& h = *c->h_state;
    out_host->total_weighted_utility = h.total_wu;
    out_host->mean_utility = c->n > 0 ? h.total_u / (double)c->n : 0.0;
    out_host->total_violation_ms = h.total_viol;
    out_host->n_rounds = h.round;
    out_host->n_scheduled = h.n_sched;
    out_host->n_dropped = c->n - h.n_sched;
    out_host->done = h.done;
  }
  return c->done ? SP_DONE : SP_OK;
}

sp_status sp_debug_dump(sp_ctx* c, int32_t kind, void* stream, const void* x_dev, const int32_t* app_dev,
                        void* dst_dev) {
  (void)app_dev;
  if (!c || !dst_dev) return SP_EINVAL;
  if (!c->scored) return SP_ESTATE;
  DeviceGuard g(c->device);
  if (!g.ok) return SP_EDEVICE;
  hipStream_t s = (hipStream_t)stream;
  const size_t n = (size_t)c->n;
  switch (kind) {
    case SP_DUMP_ORDER:
      if (n) SP_HIP(c, hipMemcpyAsync(dst_dev, c->w.id_s, n * 4, hipMemcpyDeviceToDevice, s));
      break;
    case SP_DUMP_SEGMENTS:
      SP_HIP(c, hipMemcpyAsync(dst_dev, c->w.seg, (size_t)(c->A + 1) * 4, hipMemcpyDeviceToDevice, s));
      break;
    case SP_DUMP_SCORE_CUBE: {
      const int64_t cnt = (int64_t)group_count(c) * c->Mmax * c->B;
      hipLaunchKernelGGL(k_fill_f32, dim3((unsigned)((cnt + 255) / 256)), dim3(256), 0, s, (float*)dst_dev, cnt, -1.0f);
      launch_round(c, c->w, s, nullptr, (float*)dst_dev);
      break;
    }
    case SP_DUMP_LOGITS: {
      if (n == 0) break;
      if (!x_dev) return SP_EINVAL;
      const int64_t cnt = (int64_t)n * c->Cmax;
      hipLaunchKernelGGL(k_fill_f32, dim3((unsigned)((cnt + 255) / 256)), dim3(256), 0, s, (float*)dst_dev, cnt, 0.0f);
      // same kernel as the scoring pass, with the EA / key epilogue switched off
      launch_score(c, s, x_dev, c->w.id_s, nullptr, nullptr, (float*)dst_dev);
      break;
    }
    default:
      return SP_EINVAL;
  }
  SP_HIP(c, hipStreamSynchronize(s));
  SP_HIP(c, hipGetLastError());
  return SP_OK;
}

sp_status sp_set_timing(sp_ctx* c, int32_t enable) {
  if (!c) return SP_EINVAL;
  DeviceGuard g(c->device);
  if (!g.ok) return SP_EDEVICE;
  if (enable && !c->ev[0]) {
    for (hipEvent_t& e : c->ev) SP_HIP(c, hipEventCreate(&e));
    c->round_ev.resize(kMaxRoundEvents);
    for (hipEvent_t& e : c->round_ev) SP_HIP(c, hipEventCreate(&e));
  }
  c->timing = enable != 0;
  c->timing_stages = enable == 1 || enable == 2;
  c->timing_rounds = enable == 2;
  c->timed_score = c->timed_rounds = false;
  return SP_OK;
}

sp_status sp_get_timing(sp_ctx* c, sp_timing* out) {
  if (!c || !out) return SP_EINVAL;
  if (!c->timing || (!c->timed_score && !c->timed_rounds)) return SP_ESTATE;
  DeviceGuard g(c->device);
  if (!g.ok) return SP_EDEVICE;
  sp_timing t{};
  if (c->timed_score) {
    SP_HIP(c, hipEventSynchronize(c->ev[2]));
    SP_HIP(c, hipEventElapsedTime(&t.score_kernel_ms, c->ev[1], c->ev[2]));
    if (c->timing_stages) {
      SP_HIP(c, hipEventSynchronize(c->ev[3]));
      SP_HIP(c, hipEventElapsedTime(&t.group_ms, c->ev[0], c->ev[1]));
      SP_HIP(c, hipEventElapsedTime(&t.order_ms, c->ev[2], c->ev[3]));
      SP_HIP(c, hipEventElapsedTime(&t.finish_order_ms, c->ev[6], c->ev[3]));
    }
  }
  if (c->timed_rounds) {
    SP_HIP(c, hipEventSynchronize(c->ev[5]));
    SP_HIP(c, hipEventElapsedTime(&t.rounds_ms, c->ev[4], c->ev[5]));
    t.n_rounds_timed = c->round_ms.empty() ? std::min(c->n_round_ev, c->rounds_in_call) : (int32_t)c->round_ms.size();
    if (c->timed_copy) {
      SP_HIP(c, hipEventSynchronize(c->ev[8]));
      SP_HIP(c, hipEventElapsedTime(&t.copy_outputs_ms, c->ev[7], c->ev[8]));
    }
    t.utility_evaluations = (int64_t)c->h_state->n_evals;
  }
  *out = t;
  return SP_OK;
}

sp_status sp_get_round_times(sp_ctx* c, float* ms_out, int32_t capacity, int32_t* n_out) {
  if (!c || !n_out || capacity < 0 || (capacity > 0 && !ms_out)) return SP_EINVAL;
  if (!c->timing || !c->timed_rounds) return SP_ESTATE;
  DeviceGuard g(c->device);
  if (!g.ok) return SP_EDEVICE;
  if (!c->round_ms.empty()) {          // the one-launch path times its rounds itself
    const int n = std::min(capacity, (int)c->round_ms.size());
    for (int i = 0; i < n; ++i) ms_out[i] = c->round_ms[i];
    *n_out = n;
    return SP_OK;
  }
  // an event follows every round that was launched; only those that committed a batch count
  const int n = std::min(capacity, std::min(c->n_round_ev, c->rounds_in_call));
  for (int i = 0; i < n; ++i) {
    SP_HIP(c, hipEventSynchronize(c->round_ev[i]));
    SP_HIP(c, hipEventElapsedTime(&ms_out[i], i == 0 ? c->ev[4] : c->round_ev[i - 1], c->round_ev[i]));
  }
  *n_out = n;
  return SP_OK;
}

const char* sp_strerror(sp_status s) {
  switch (s) {
    case SP_OK: return "ok";
    case SP_DONE: return "no live request left";
    case SP_EINVAL: return "invalid argument, profile or request data";
    case SP_ENOMEM: return "out of memory";
    case SP_EDEVICE: return "HIP call failed";
    case SP_ESTATE: return "call order: score the window first";
    case SP_ECAPACITY: return "size beyond the context's or the library's capacity";
  }
  return "unknown status";
}

const char* sp_last_hip_error(const sp_ctx* c) { return c ? c->hip_err.c_str() : ""; }
sp_status sp_set_prior(sp_ctx* c, int32_t app, const float* alpha_host, float evidence_k) {
  if (!c || app < 0 || app >= c->A) return SP_EINVAL;
  DeviceGuard g(c->device);
  if (!g.ok) return SP_EDEVICE;
  const int C = c->h_ncls[app], M = c->h_nmod[app];
  float gain = 1.0f;
  std::vector<float> bias((size_t)c->Mmax, 0.0f);
  if (alpha_host) {
    if (!(evidence_k >= 0.f) || !std::isfinite(evidence_k)) return SP_EINVAL;
    double sum = 0.0;
    for (int cl = 0; cl < C; ++cl) {
      if (!(alpha_host[cl] >= 0.f) || !std::isfinite(alpha_host[cl])) return SP_EINVAL;
      sum += (double)alpha_host[cl];
    }
    const double den = sum + (double)evidence_k;
    if (!(den > 0.0)) return SP_EINVAL;
    // EA'[m] = (sum_c alpha_c Acc[m][c] + k EA[m]) / (sum alpha + k)
    gain = (float)((double)evidence_k / den);
    const float* acc = c->h_acc.data() + c->h_acc_off[app];
    for (int m = 0; m < M; ++m) {
      double t = 0.0;
      for (int cl = 0; cl < C; ++cl) t += (double)alpha_host[cl] * (double)acc[(size_t)m * C + cl];
      bias[m] = (float)(t / den);
    }
  }
  // ordered after whatever the device is still doing with the old values
  SP_HIP(c, hipDeviceSynchronize());
  SP_HIP(c, hipMemcpy(c->d_ea_gain + app, &gain, sizeof(float), hipMemcpyHostToDevice));
  SP_HIP(c, hipMemcpy(c->d_ea_bias + (size_t)app * c->Mmax, bias.data(), bias.size() * sizeof(float), hipMemcpyHostToDevice));
  return SP_OK;
}

sp_status sp_set_policy(sp_ctx* c, const sp_policy* p) {
  if (!c) return SP_EINVAL;
  sp_policy def{};
  if (!p) p = &def;
  if (p->order < 0 || p->order > 1 || p->select < 0 || p->select > 1 || p->batch_rule < 0 || p->batch_rule > 1 ||
      p->choice < 0 || p->choice > 1 || p->weight < 0 || p->weight > 1 || p->batch_cap < 0 || p->split_groups < 0 ||
      p->split_groups > 1)
    return SP_EINVAL;
  Tables& tb = c->tb;
  tb.pol_edf = p->order; tb.pol_group_first = p->select; tb.pol_whole = p->batch_rule;
  tb.pol_max_accuracy = p->choice; tb.pol_unit_weight = p->weight;
  tb.Bcap = p->batch_cap > 0 ? std::min(p->batch_cap, c->B) : c->B;
  c->scored = false;                 // the service order depends on the policy: score the window again
  if (p->split_groups) {
    DeviceGuard g(c->device);
    if (!g.ok) return SP_EDEVICE;
    sp_status s = ensure_split_buffers(c);
    if (s != SP_OK) return s;
    // the resident rounds kernel with its per-wavefront windows: does the whole grid still fit?
    c->persist_split = false;
    if (c->persist) {
      int cus = 0, per_cu = 0;
      const size_t dyn = (size_t)(kRoundThreads / 64) * (size_t)c->B * (sizeof(float4) + sizeof(int32_t));
      if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, c->device) == hipSuccess &&
          hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, k_rounds_persistent<true>, kRoundThreads, dyn) == hipSuccess)
        c->persist_split = (size_t)per_cu * (size_t)cus >= (size_t)c->ps.n_pairs + 2;
      else
        (void)hipGetLastError();
    }
  }
  tb.pol_split = p->split_groups;
  return SP_OK;
}

sp_status sp_set_swap_cost(sp_ctx* c, int32_t app, const float* swap_ms_host) {
  if (!c || app < 0 || app >= c->A) return SP_EINVAL;
  DeviceGuard g(c->device);
  if (!g.ok) return SP_EDEVICE;
  const int M = c->h_nmod[app];
  std::vector<float> v((size_t)c->Mmax, 0.0f);
  if (swap_ms_host)
    for (int m = 0; m < M; ++m) {
      if (!(swap_ms_host[m] >= 0.f) || !std::isfinite(swap_ms_host[m])) return SP_EINVAL;
      v[m] = swap_ms_host[m];
    }
  SP_HIP(c, hipDeviceSynchronize());
  SP_HIP(c, hipMemcpy(c->d_swap + (size_t)app * c->Mmax, v.data(), v.size() * sizeof(float), hipMemcpyHostToDevice));
  return SP_OK;
}

int32_t sp_max_models(const sp_ctx* c) { return c ? c->Mmax : 0; }
int32_t sp_max_classes(const sp_ctx* c) { return c ? c->Cmax : 0; }
int32_t sp_rounds_in_one_launch(const sp_ctx* c) {
  if (!c) return 0;
  DeviceGuard g(c->device);
  return (g.ok && rounds_in_one_launch(const_cast<sp_ctx*>(c))) ? 1 : 0;
}

sp_status sp_debug_set_spin_limit(sp_ctx* c, int32_t polls) {
  if (!c || polls < 0) return SP_EINVAL;
  c->spin_limit = polls == 0 ? kSpinLimit : polls;
  return SP_OK;
}

sp_status sp_debug_set_sort_spin_limit(sp_ctx* c, int32_t polls) {
  if (!c) return SP_EINVAL;
  c->sort_spin_limit = polls == 0 ? kSortSpinLimit : polls;
  return SP_OK;
}

sp_status sp_debug_set_generation(sp_ctx* c, uint32_t generation) {
  if (!c || generation >= kGenMask) return SP_EINVAL;
  if (c->persist) {
    // words tagged by earlier launches must not match a generation that is handed out again
    DeviceGuard g(c->device);
    if (!g.ok) return SP_EDEVICE;
    SP_HIP(c, hipDeviceSynchronize());
    fill_u64(nullptr, c->ps.slots, 8 * (size_t)c->ps.n_pairs);
    fill_u64(nullptr, c->ps.decision, 8);
    fill_u64(nullptr, c->ps.ring, (size_t)kPersistRounds * c->A * c->B);
    fill_u64(nullptr, c->ps.dec, kPersistRounds);
    SP_HIP(c, hipDeviceSynchronize());
  }
  c->gen_base = generation;
  return SP_OK;
}

sp_status sp_debug_mfma_rate(int device_id, int32_t random_bits, int32_t idle, int32_t iters, void* stream,
                             double* tflops_out, double* clock_ghz_out) {
  if (iters < 1 || iters > (1 << 20) || !tflops_out) return SP_EINVAL;
  if (idle != 0 && idle != 1 && idle != 2 && idle != 4 && idle != 8) return SP_EINVAL;
  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess || device_id < 0 || device_id >= ndev) return SP_EDEVICE;
  DeviceGuard g(device_id);
  if (!g.ok) return SP_EDEVICE;
  hipStream_t s = (hipStream_t)stream;
  float* out = nullptr;
  long long* clk = nullptr;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  sp_status rc = SP_EDEVICE;
  float ms = 0.f;
  long long h[2] = {0, 0};
  const int threads = idle > 0 ? kProbeIdleThreads : kProbeThreads;
  auto launch = [&] {
    const dim3 grd(kProbeBlocks), blk(threads);
    switch (idle) {
      case 0: hipLaunchKernelGGL(k_mfma_rate<0>, grd, blk, 0, s, (int)random_bits, (int)iters, out, clk); break;
      case 1: hipLaunchKernelGGL(k_mfma_rate<1>, grd, blk, 0, s, (int)random_bits, (int)iters, out, clk); break;
      case 2: hipLaunchKernelGGL(k_mfma_rate<2>, grd, blk, 0, s, (int)random_bits, (int)iters, out, clk); break;
      case 4: hipLaunchKernelGGL(k_mfma_rate<4>, grd, blk, 0, s, (int)random_bits, (int)iters, out, clk); break;
      default: hipLaunchKernelGGL(k_mfma_rate<8>, grd, blk, 0, s, (int)random_bits, (int)iters, out, clk); break;
    }
  };
  if (hipMalloc((void**)&out, (size_t)kProbeBlocks * kProbeThreads * sizeof(float)) != hipSuccess) goto end;
  if (hipMalloc((void**)&clk, 2 * sizeof(long long)) != hipSuccess) goto end;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) goto end;
  // one untimed launch brings the clocks to their steady state, the second is timed
  launch();
  if (hipEventRecord(e0, s) != hipSuccess) goto end;
  launch();
  if (hipEventRecord(e1, s) != hipSuccess) goto end;
  if (hipEventSynchronize(e1) != hipSuccess || hipGetLastError() != hipSuccess) goto end;
  if (hipEventElapsedTime(&ms, e0, e1) != hipSuccess || !(ms > 0.f)) goto end;
  if (hipMemcpy(h, clk, sizeof(h), hipMemcpyDeviceToHost) != hipSuccess) goto end;
  // 2 * 32 * 32 * 16 flops per instruction and wavefront
  *tflops_out = (double)kProbeBlocks * (threads / 64) * (double)iters * kProbeMfmaPerIter * 32768.0 / ((double)ms * 1e-3) / 1e12;
  if (clock_ghz_out) *clock_ghz_out = h[1] > 0 ? (double)h[0] / ((double)h[1] * 10.0) : 0.0;
  rc = SP_OK;
end:
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  if (out) (void)hipFree(out);
  if (clk) (void)hipFree(clk);
  return rc;
}

sp_status sp_debug_copy_rate(int device_id, int64_t bytes, void* stream, double* gbs_out) {
  if (bytes < 16 || bytes > ((int64_t)1 << 34) || !gbs_out) return SP_EINVAL;
  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess || device_id < 0 || device_id >= ndev) return SP_EDEVICE;
  DeviceGuard g(device_id);
  if (!g.ok) return SP_EDEVICE;
  hipStream_t s = (hipStream_t)stream;
  const int64_t n = bytes / 16;
  float4 *src = nullptr, *dst = nullptr;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  sp_status rc = SP_EDEVICE;
  float ms = 0.f;
  const unsigned grid = (unsigned)std::min<int64_t>((n + 255) / 256, 256 * 64);
  if (hipMalloc((void**)&src, (size_t)n * 16) != hipSuccess) { rc = SP_ENOMEM; goto end; }
  if (hipMalloc((void**)&dst, (size_t)n * 16) != hipSuccess) { rc = SP_ENOMEM; goto end; }
  if (hipMemsetAsync(src, 1, (size_t)n * 16, s) != hipSuccess) goto end;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) goto end;
  hipLaunchKernelGGL(k_copy_rate, dim3(grid), dim3(256), 0, s, (const float4*)src, dst, n);   // untimed: page the buffers in
  if (hipEventRecord(e0, s) != hipSuccess) goto end;
  for (int i = 0; i < 4; ++i) hipLaunchKernelGGL(k_copy_rate, dim3(grid), dim3(256), 0, s, (const float4*)src, dst, n);
  if (hipEventRecord(e1, s) != hipSuccess) goto end;
  if (hipEventSynchronize(e1) != hipSuccess || hipGetLastError() != hipSuccess) goto end;
  if (hipEventElapsedTime(&ms, e0, e1) != hipSuccess || !(ms > 0.f)) goto end;
  *gbs_out = 4.0 * 2.0 * (double)n * 16.0 / ((double)ms * 1e-3) / 1e9;     // bytes read + bytes written
  rc = SP_OK;
end:
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  if (src) (void)hipFree(src);
  if (dst) (void)hipFree(dst);
  return rc;
}

}  // extern "C"
