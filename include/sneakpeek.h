/*
 * sneakpeek.h -- C ABI of the MI355X (gfx950) SneakPeek scoring / batch-aware
 * greedy scheduling library.
 *
 * The library scores every pending inference request against every model
 * variant of its application and turns the queue into a schedule by greedy
 * batch-selection rounds:
 *
 *   posterior      theta_i = softmax(f_{a_i}(x_i))            (Def. 4.1.1, 4.1.2)
 *   data-aware EA  EA[i,m] = sum_c theta_ic * Acc[a_i][m][c]  (Sec. 4.1, eq. (9))
 *   priority key   k_i = w_i (1 + Var_m EA[i,.]) exp(-D_i/T_d) (Sec. 5.1.1, eq. (12))
 *   utility        u = EA * (1 - gamma_a(D, t + L[a][m][b]))   (Sec. 3.1, eq. (2); Sec. 6.1)
 *   round          arg max over (a, m, b) of the key-weighted utility of the
 *                  first b live requests of a in key order   (eq. (13), Alg. 1)
 *
 * All entry points are plain C: opaque context, plain pointers and sizes.
 * Pointers named *_dev are DEVICE pointers owned by the caller (any HIP
 * allocation on the context's device); all others are HOST pointers.  No call
 * throws or aborts; every call returns an sp_status (or void).  Outputs are
 * left untouched when a call fails before launching work.  A context serves
 * one scheduling window at a time and must not be used from two threads at
 * once; different contexts are independent.
 */
#ifndef SNEAKPEEK_H
#define SNEAKPEEK_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct sp_ctx sp_ctx;

typedef enum {
  SP_OK = 0,
  SP_DONE = 1,        /* no live request is left: not an error                   */
  SP_EINVAL = -1,     /* bad argument, bad profile, or bad request data          */
  SP_ENOMEM = -2,     /* host or device allocation failed                        */
  SP_EDEVICE = -3,    /* a HIP call failed, or resident workgroups of the rounds
                         kernel lost each other (see sp_last_hip_error)          */
  SP_ESTATE = -4,     /* call order: rounds before any sp_score                  */
  SP_ECAPACITY = -5   /* a size exceeds what the context or library supports     */
} sp_status;

/* Deadline penalties of Sec. 6.1, with x = (e - d) / d for completion e and
 * relative deadline d; all are 0 for e <= d and capped at 1:
 *   step    1                          linear   min(1, x)
 *   sigmoid x^3 / (x^3 + (1-x)^3) for x < 1, else 1                           */
typedef enum { SP_PEN_STEP = 0, SP_PEN_LINEAR = 1, SP_PEN_SIGMOID = 2 } sp_penalty;

typedef enum { SP_F32 = 0, SP_BF16 = 1 } sp_dtype;

/* Library limits (SP_ECAPACITY beyond them). */
#define SP_MAX_MODELS 16      /* variants per application                        */
#define SP_MAX_BATCH 256      /* largest batch size B                            */
#define SP_MAX_APPS 65535

/*
 * Registered applications (Sec. 2.2 "System Model", Sec. 3.2): per
 * application a SneakPeek head, the accuracy (recall) of every model variant
 * on each of the application's classes, and each variant's profiled latency
 * per batch size.  HOST pointers; sp_create copies
 * everything, the caller keeps ownership.
 *
 * Head of application a: hidden_dim == 0 -> logistic, z = x W1 + b1 with
 * W1 [feat_dim, C_a]; otherwise z = relu(x W1 + b1) W2 + b2 with
 * W1 [feat_dim, hidden_dim], W2 [hidden_dim, C_a].  All matrices row-major.
 * W1/W2 (and the request features) hold feat_dtype elements (float, or
 * bfloat16 bit patterns in uint16_t); biases and tables are float.
 */
typedef struct {
  int32_t n_apps;               /* A >= 1                                          */
  int32_t feat_dim;             /* d >= 1                                          */
  int32_t hidden_dim;           /* H >= 0                                          */
  int32_t max_batch;            /* B: batch sizes are 1..B                         */
  int32_t feat_dtype;           /* sp_dtype                                        */
  int32_t max_requests;         /* capacity of the window buffers (>= 0)           */
  const int32_t* n_classes;     /* [A] C_a >= 1                                    */
  const int32_t* n_models;      /* [A] 1 <= M_a <= SP_MAX_MODELS                   */
  const void* const* W1;        /* [A] -> [d, H] or [d, C_a]                       */
  const float* const* b1;       /* [A] -> [H] or [C_a]                             */
  const void* const* W2;        /* [A] -> [H, C_a]; NULL when hidden_dim == 0      */
  const float* const* b2;       /* [A] -> [C_a];    NULL when hidden_dim == 0      */
  const float* const* acc;      /* [A] -> [M_a, C_a], each in [0, 1]               */
  const float* const* lat_ms;   /* [A] -> [M_a, B], >= 0, non-decreasing in b      */
  const int32_t* penalty;       /* [A] sp_penalty (penalties are per application)  */
  float prio_timescale_ms;      /* T_d > 0 of the priority key (1000 = seconds)    */
} sp_profile;

/* One committed batch.  Times are milliseconds on the worker clock, 0 at the
 * start of the window (eq. (1) with the batch as the unit).                    */
typedef struct {
  int32_t app, model, batch, round;
  double t_start_ms, t_end_ms;
  float score;                  /* sum over members of key * utility               */
  float batch_utility;          /* sum over members of weight * utility            */
} sp_decision;

typedef struct {
  double total_weighted_utility;   /* sum_i w_i u_i                                */
  double mean_utility;             /* (1/N) sum_i u_i, the objective of eq. (3)    */
  double total_violation_ms;       /* sum over served requests of max(0, e_i - D_i)*/
  int32_t n_rounds, n_scheduled, n_dropped;
  int32_t done;                    /* 1 when no live request is left               */
} sp_summary;

/* What sp_debug_dump can export (parity tests only; not on the hot path). */
typedef enum {
  SP_DUMP_ORDER = 0,      /* int32 [n]: request ids in service order, application-major        */
  SP_DUMP_SEGMENTS = 1,   /* int32 [A+1]: start of each application's range in that order      */
  SP_DUMP_SCORE_CUBE = 2, /* float [A, Mmax, B]: Score[a][m][b-1] at the current clock, -1
                             where (a, m, b) is not a candidate                                 */
  SP_DUMP_LOGITS = 3      /* float [n, Cmax]: head outputs z_i (0 beyond C_a)                   */
} sp_dump_kind;

/* Device times of the last sp_score / sp_schedule call, from HIP events that
 * the library records on the caller's stream while timing is enabled.         */
typedef struct {
  float group_ms;          /* grouping requests by application                                 */
  float score_kernel_ms;   /* the fused posterior / EA / key kernel alone (one launch)         */
  float order_ms;          /* per-application ordering by key                                  */
  float rounds_ms;         /* all rounds of the last sp_schedule call                          */
  int32_t n_rounds_timed;  /* rounds with an individual time (see sp_get_round_times)          */
  float finish_order_ms;   /* within order_ms: the kernel that gathers id, deadline, weight and
                              key per service position after the last radix pass              */
  float copy_outputs_ms;   /* the kernel that copies the four per-request outputs to the
                              caller's arrays (first chunk of the last sp_schedule call)      */
  int64_t utility_evaluations;  /* terms key * EA * (1 - penalty) summed by the rounds of the
                              window so far: per round and (group, variant), nb (nb + 1) / 2
                              for a candidate window of nb requests (nb under SP_BATCH_WHOLE) */
} sp_timing;

/* Application registration (Sec. 3.2 "System Architecture": owners upload
 * their variants with accuracy and latency profiles before any request is
 * served).  Validate and upload a profile to `device_id`, allocate window
 * buffers for max_requests.  SP_EINVAL: NULL pointers, counts out of range, acc outside
 * [0,1] or NaN, latency negative / NaN / decreasing in b, unknown enum,
 * T_d <= 0.  SP_ECAPACITY: beyond the SP_MAX_* limits.  On success *out owns
 * device memory until sp_destroy.                                              */
sp_status sp_create(const sp_profile* profile, int device_id, sp_ctx** out);
void sp_destroy(sp_ctx* ctx);

/* Scoring pass over one window of n pending requests (Sec. 3.2: requests are
 * enqueued during a window, then scheduled together): groups requests by
 * application, computes EA and the priority key of every request, orders each
 * application's requests by (key descending, request id ascending) and resets
 * the window state (everyone pending, clock 0, round 0).
 *   x_dev            [n, feat_dim] row-major, feat_dtype elements
 *   app_dev          [n] application id in [0, A)
 *   deadline_ms_dev  [n] D_i = d_i - now, > 0
 *   weight_dev       [n] w_i >= 0 (all ones recovers the paper's priority)
 *   ea_out_dev       [n, Mmax] (Mmax = max_a M_a; 0 beyond M_a) or NULL
 *   key_out_dev      [n] or NULL
 * Work is enqueued on `stream` (a hipStream_t, NULL = default stream) and the
 * call returns without waiting.  The inputs may be freed once the stream has
 * passed this call.  n == 0 is legal.  n > max_requests -> SP_ECAPACITY.  Bad
 * request data (application id out of range, deadline <= 0 or NaN, weight < 0
 * or NaN) is detected on the device and reported as SP_EINVAL by the next
 * sp_greedy_round / sp_schedule; such a window is not scheduled.              */
sp_status sp_score(sp_ctx* ctx, int32_t n, const void* x_dev, const int32_t* app_dev,
                   const float* deadline_ms_dev, const float* weight_dev, void* stream,
                   float* ea_out_dev, float* key_out_dev);

/* One greedy round at the current clock t (one pass of Alg. 1's loop over
 * groups, Sec. 5.2, with the batch as the unit: choice by eq. (13), utility
 * eq. (2), clock eq. (1)): a request is live while pending
 * and its penalty on the earliest possible completion t + min_m L[a][m][1] is
 * below 1; for every application the first min(B, n_live) live requests in
 * service order form the candidate window; every (a, m, b) is scored and the
 * best one is committed (exact ties: smallest (a, m, b)); the clock advances
 * to its completion time.  Waits for the stream.  *out_host receives the
 * decision; req_ids_out_dev (NULL or [B]) the ids of its members in service
 * order.  Returns SP_DONE (and leaves *out_host untouched) when no request is
 * live, SP_ESTATE before the first sp_score.                                   */
sp_status sp_greedy_round(sp_ctx* ctx, void* stream, sp_decision* out_host, int32_t* req_ids_out_dev);

/* sp_greedy_round for callers that must not allocate device memory and want the library to touch none
 * that was allocated for it either: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, same decision, same status codes as sp_greedy_round; the buffers the
 * two round kernels exchange through (one candidate word and one group priority per (group, variant), the
 * window positions and window size per group) live in a static device array of 1 MiB that every GPU the
 * library runs on holds until the process ends, instead of in the context.  The call allocates and frees
 * nothing.  SP_ECAPACITY (nothing launched) when
 *   G * Mmax * 12 + G * B * 4 + G * 4 bytes, each term rounded up to 256,
 * exceed 1 MiB, G being the number of groups the context can hold (A, or the (application, subgroup)
 * slots once group splitting has been switched on).  All contexts on one GPU share that array and it
 * keeps the last call's contents (every word a round reads is written by that round first, so nothing has
 * to be cleared): calls that overlap on one GPU, from different contexts or streams, race.               */
sp_status sp_greedy_round_static(sp_ctx* ctx, void* stream, sp_decision* out_host, int32_t* req_ids_out_dev);

/* Greedy rounds until nothing is live, or until max_rounds more rounds have
 * been committed (max_rounds <= 0: no limit).  Rounds run back to back on the
 * device; the call waits for the stream before returning.
 *   model_out_dev / round_out_dev / order_out_dev / util_out_dev: each NULL
 *     or [n]; variant id (-1 = not served), round id (-1), global execution
 *     order starting at 1 (0 = not served, as s_ij = 0 in Sec. 3.1), utility.
 *   round_log_host [log_capacity]: decisions of all rounds of this window so
 *     far (including earlier sp_greedy_round calls), truncated to capacity.
 *   out_host: totals over the window so far.
 * Returns SP_OK when stopped by max_rounds, SP_DONE when the queue is
 * exhausted (both fill the outputs).
 * When every (application, variant) pair fits on the device at once (see
 * sp_rounds_in_one_launch), up to 64 rounds run inside one kernel whose
 * workgroups wait for each other with bounded waits.  If the device is shared
 * with other long-running work and such a wait runs out, the call returns
 * SP_EDEVICE, the context switches to two kernels per round for good, and the
 * window has to be scored again (SP_ESTATE until then).                        */
sp_status sp_schedule(sp_ctx* ctx, int32_t max_rounds, void* stream,
                      int32_t* model_out_dev, int32_t* round_out_dev, int32_t* order_out_dev,
                      float* util_out_dev, sp_decision* round_log_host, int32_t log_capacity,
                      sp_summary* out_host);

/* Parity-test export; waits for the stream.  SP_DUMP_LOGITS recomputes the
 * heads from x_dev/app_dev (pass the same arrays as to sp_score); the other
 * kinds ignore them.  dst_dev must hold the size listed at sp_dump_kind.       */
sp_status sp_debug_dump(sp_ctx* ctx, int32_t kind, void* stream, const void* x_dev,
                        const int32_t* app_dev, void* dst_dev);

/* Benchmark aid.  sp_set_timing(ctx, 1) makes sp_score and sp_schedule record
 * HIP events around their stages; sp_set_timing(ctx, 2) additionally times
 * every round: from the rounds kernel's own constant-rate timestamps when the
 * rounds run in one launch, else from one HIP event after each of the first
 * 4096 rounds (this slows the rounds down a little); sp_set_timing(ctx, 3)
 * records the two events around the scoring kernel only (an event between two
 * kernels keeps the second from starting right behind the first: nine of them
 * cost a window about 40 us, two about 10), and sp_get_timing then fills
 * score_kernel_ms and leaves the other fields 0; 0 turns timing off.
 * sp_get_timing /
 * sp_get_round_times wait for the events and return the elapsed device times
 * (per-round times in milliseconds, HOST array of `capacity` floats, *n_out =
 * number written).  SP_ESTATE if timing is off or nothing has been recorded yet. */
sp_status sp_set_timing(sp_ctx* ctx, int32_t enable);
sp_status sp_get_timing(sp_ctx* ctx, sp_timing* out_host);
sp_status sp_get_round_times(sp_ctx* ctx, float* ms_out_host, int32_t capacity, int32_t* n_out);

/*
 * Dirichlet prior of one application (Sec. 4.2, eq. (10)-(11); the kinds of prior: Sec. 6.3 "Choice of
 * Prior").  alpha_host: HOST pointer to C_a values alpha_c >= 0 (copied), or NULL to remove the prior.
 * evidence_k >= 0: the number of multinomial draws the head's output theta stands for (the paper's k
 * neighbours; the evidence is y = k * theta).  From the next sp_score on, the posterior of that
 * application's requests is the mean of Dirichlet(alpha + y), theta' = (alpha + k theta) / (sum alpha + k),
 * and expected accuracies, keys and utilities follow from theta'.  The library folds this into an affine
 * map of the expected accuracies, EA' = (sum_c alpha_c Acc[m][c] + k EA[m]) / (sum alpha + k), which is
 * eq. (9) applied to theta'.  Synchronises the device.  SP_EINVAL: app out of range, a negative or
 * non-finite alpha_c or k, sum alpha + k == 0.
 */
sp_status sp_set_prior(sp_ctx* ctx, int32_t app, const float* alpha_host, float evidence_k);

/*
 * Scheduling policy: the approaches the paper compares (Sec. 6.1 "Baselines and Metrics") and Alg. 1 as
 * printed, as combinations of independent knobs on the same kernels.  All zero (or policy == NULL) is the
 * default: priority order, one joint arg max over (application, variant, batch size).
 *   order       SP_ORDER_PRIORITY: requests of an application are served by descending key (eq. (12));
 *               SP_ORDER_EDF: by ascending deadline (ties: ascending request id).
 *   select      SP_SELECT_JOINT: arg max of the score over all (a, m, b);
 *               SP_SELECT_GROUP_FIRST: first the application whose candidate window has the highest mean
 *               priority (eq. (14); the mean of the keys, or of the negated deadlines under EDF; ties: the
 *               smallest application), then the arg max over (m, b) for that application alone (Alg. 1).
 *   batch_rule  SP_BATCH_FREE: every batch size up to the cap is a candidate;
 *               SP_BATCH_WHOLE: only the whole candidate window ("all requests in the group", Alg. 1).
 *   choice      SP_CHOICE_UTILITY: candidates are compared by utility under the application's penalty
 *               (eq. (13)); SP_CHOICE_MAX_ACCURACY: under the step penalty, i.e. by accuracy among the
 *               variants that meet the deadline ("Max Accuracy"); utilities of served requests always use
 *               the application's own penalty.
 *   weight      SP_WEIGHT_KEY: a batch's score is the key-weighted sum of its members' utilities;
 *               SP_WEIGHT_UNIT: the plain sum ("avg group utility", Alg. 1).
 *   batch_cap   > 0: batches hold at most min(batch_cap, B) requests (1 = request-level baselines).
 * LO-Priority = {GROUP_FIRST, cap 1}; LO-EDF = {EDF, GROUP_FIRST, cap 1}; MaxAcc-EDF = LO-EDF +
 * MAX_ACCURACY; Alg. 1 = {GROUP_FIRST, WHOLE, UNIT}; the data-oblivious variants also set a prior with no
 * evidence (sp_set_prior with the profiling label mix and evidence_k = 0).
 * The window must be scored again afterwards (the service order depends on the policy): rounds return
 * SP_ESTATE until then.  SP_EINVAL: a knob out of range.
 */
typedef enum { SP_ORDER_PRIORITY = 0, SP_ORDER_EDF = 1 } sp_order;
typedef enum { SP_SELECT_JOINT = 0, SP_SELECT_GROUP_FIRST = 1 } sp_select;
typedef enum { SP_BATCH_FREE = 0, SP_BATCH_WHOLE = 1 } sp_batch_rule;
typedef enum { SP_CHOICE_UTILITY = 0, SP_CHOICE_MAX_ACCURACY = 1 } sp_choice;
typedef enum { SP_WEIGHT_KEY = 0, SP_WEIGHT_UNIT = 1 } sp_weight;
typedef struct {
  int32_t order, select, batch_rule, choice, weight, batch_cap;
  int32_t split_groups;   /* 1: data-aware subgroups (Sec. 5.3.2, "Enhancements for Grouped Scheduling"): inside an
                             application, requests whose SneakPeek head puts more than one half on a class form that
                             class's subgroup, the others stay in the application's unsplit group; every non-empty
                             (application, subgroup) pair is then a group of its own in the rounds (own service
                             order, own candidate window; batches never mix subgroups; ties go to the smaller
                             (application, subgroup)).  The label uses the head's own softmax output, also when a
                             prior is set.  SP_ECAPACITY if sum_a (C_a + 1) exceeds 65536.  SP_DUMP_SCORE_CUBE then
                             has one [Mmax, B] slab per group.  sp_schedule still runs the rounds in one launch
                             while no application of the scored window has more than 64 non-empty groups
                             (sp_rounds_in_one_launch after sp_score tells), else two kernels per round.           */
} sp_policy;
sp_status sp_set_policy(sp_ctx* ctx, const sp_policy* policy);

/*
 * Swap-in cost of the variants of one application (Sec. 3.1 counts the cost of switching to a variant as
 * part of its latency; Sec. 5.2: grouping keeps a loaded variant in use).
 * swap_ms_host: HOST pointer to M_a values >= 0 (copied), or NULL for none.  A batch on variant m of that
 * application then completes at t + swap_ms[m] + L[a][m][b] unless the previous batch of the window ran
 * the same variant of the same application, in which case it completes at t + L[a][m][b]; candidates are
 * scored with the completion time they would really have.  The first batch of a window always pays.
 * Liveness does not look at swap costs (a request is dead once t + min_m L[a][m][1] makes its penalty
 * 1), so that dead requests stay dead.  Takes effect from the next round on.  Synchronises the
 * device.  SP_EINVAL: app out of range, a negative or non-finite cost.
 */
sp_status sp_set_swap_cost(sp_ctx* ctx, int32_t app, const float* swap_ms_host);

const char* sp_strerror(sp_status s);
/* Text of the last HIP error seen by this context (empty string if none). */
const char* sp_last_hip_error(const sp_ctx* ctx);
/* max_a M_a and max_a C_a of the profile (row widths of the outputs). */
int32_t sp_max_models(const sp_ctx* ctx);
int32_t sp_max_classes(const sp_ctx* ctx);
/* How sp_schedule runs the greedy rounds (Alg. 1, Sec. 5.2) on this context: 1 = all rounds of a chunk in
 * one launch (every (application, variant) pair fits on the device at once and, with group splitting, no
 * application of the scored window has more than 64 groups: after sp_score the call waits for that count),
 * 0 = two kernels per round.  The decisions are the same either way.  sp_greedy_round always takes the
 * second way. */
int32_t sp_rounds_in_one_launch(const sp_ctx* ctx);

/*
 * Test hook, not on the hot path (implements nothing of the paper).  The one-launch rounds kernel tags the words
 * its workgroups exchange with a round generation number that grows by one per round over the life of the
 * context and starts over, with the exchange buffers cleared, before it would exceed 2^23 - 1 (after some
 * eight million rounds).  This sets the number of generations used so far, so that a test can place a window
 * across that point, and clears the exchange buffers (words tagged by earlier launches can then never match a
 * generation that is handed out again).  Synchronises the device.  Call it between windows only.
 * SP_EINVAL: ctx NULL or generation >= 2^23 - 1.
 */
sp_status sp_debug_set_generation(sp_ctx* ctx, uint32_t generation);

/*
 * Test hook, not on the hot path (implements nothing of the paper).  The workgroups of the one-launch rounds kernel wait for each other with
 * bounded polling; a wait that runs out (the device is shared with other long-running work and the grid is
 * not resident as a whole) makes every workgroup leave, sp_schedule return SP_EDEVICE, and the context use
 * two kernels per round from then on (the window has to be scored again).  polls > 0 shortens the bound so
 * that a test can take that path with every kernel still ending normally; 0 restores the default (2^20).
 * SP_EINVAL: ctx NULL or polls < 0.
 */
sp_status sp_debug_set_spin_limit(sp_ctx* ctx, int32_t polls);

/*
 * Test hook, not on the hot path (implements nothing of the paper).  A tile of a radix pass of the ordering
 * learns the digit counts of the tiles before it in its segment by polling words they publish; the polling
 * is bounded, and a look-back that runs out raises an error that the next sp_greedy_round / sp_schedule
 * reports as SP_EDEVICE (the window has to be scored again; the context stays usable).  polls > 0 sets the
 * bound, polls < 0 makes every look-back give up at once (a test's way into that path with every kernel
 * still ending normally), 0 restores the default (2^20).  SP_EINVAL: ctx NULL.
 */
sp_status sp_debug_set_sort_spin_limit(sp_ctx* ctx, int32_t polls);

/*
 * Diagnostic, not on the hot path and no part of the paper's method: the rate at which the device's matrix
 * cores run the half-precision instruction the scoring kernel is built on when nothing else competes.
 * random_bits = 0: constant operands; 1: operands with random bits.  idle in {0, 1, 2, 4, 8}: after every
 * eight instructions a wavefront sleeps about idle * 64 cycles (idle > 0 runs one wavefront per SIMD, so that
 * eight instructions are 256 busy cycles of the matrix core followed by the gap; the duty cycle reached is
 * tflops_out over 1024 SIMDs * 1024 flops per cycle * the clock; idle = 0 runs two wavefronts per SIMD back
 * to back).  The clock the device sustains depends on how many operand
 * bits toggle and on the duty cycle (the instruction runs under a power limit), so the figures with
 * random bits are the ceiling a kernel fed with real data can reach.  iters in [1, 2^20]: instructions per
 * wavefront = 8 * iters.  stream: a hipStream_t.  tflops_out (HOST, required): 2 * 32 * 32 * 16 flops per
 * instruction over the time of one launch between two events; clock_ghz_out (HOST, may be NULL): shader
 * cycles over the constant-rate counter.  Allocates and frees its own small buffers; synchronises the stream.
 * SP_EINVAL: iters or idle out of range or tflops_out NULL; SP_EDEVICE: no such device or a HIP call failed.
 */
sp_status sp_debug_mfma_rate(int device_id, int32_t random_bits, int32_t idle, int32_t iters, void* stream,
                             double* tflops_out, double* clock_ghz_out);

/*
 * Diagnostic, not on the hot path and no part of the paper's method: the memory bandwidth a plain streaming
 * copy kernel reaches on the device, bytes read plus bytes written per second over four launches between
 * two events (GB/s, 10^9), for `bytes` bytes each way (a multiple of 16, at most 16 GiB).  Allocates and
 * frees its two buffers; synchronises the stream.  SP_EINVAL: bytes out of range or gbs_out NULL;
 * SP_ENOMEM: the buffers do not fit; SP_EDEVICE: no such device or a HIP call failed.
 */
sp_status sp_debug_copy_rate(int device_id, int64_t bytes, void* stream, double* gbs_out);

#ifdef __cplusplus
}
#endif
#endif /* SNEAKPEEK_H */
