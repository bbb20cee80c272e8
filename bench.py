#!/usr/bin/env python3
"""Benchmark of the SneakPeek scoring + greedy-round hot path on one MI355X.

A step is one pass of the whole path over one window of synthetic requests:
sp_score (group by application, posterior -> expected accuracy -> priority
key, per-application ordering) followed by sp_schedule (greedy rounds).
Inputs are resident in HBM before the timed region.  Prints one JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg5]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np

METRIC = "request x model x batch candidates scored/s"

# published MI355X peaks used for the roofline fractions
PEAK_HBM_GBS = 8000.0
PEAK_MFMA_F32_TFLOPS = 157.3
PEAK_MFMA_BF16_TFLOPS = 2500.0
PEAK_MFMA_F16_TFLOPS = 2500.0
PEAK_VALU_F32_TFLOPS = 157.3

# HBM traffic of the scoring kernel per launch comes from hardware counters taken in profiler runs of this
# same script (rocprofv3 --pmc FETCH_SIZE, then WRITE_SIZE, each scaled by what the same counter reads for
# the 256 MiB copy of --calibrate-copy).  The summaries under profiles/ carry one line per workload,
#   scoring_kernel_traffic <workload> fetch_bytes=<f> write_bytes=<w> kernel_sources_sha256=<sha>
# which is read here; a figure is only reported while the kernel sources it was taken on are unchanged
# (sha256 over the files below), otherwise traffic is null.
KERNEL_SOURCES = ["sp_common.h", "sp_score_generic.h", "sp_score_split.h", "sp_score_mlp.h"]
PROFILE_FILES = {w: os.path.join("profiles", f"hot_path_{w}_kernel_stats_and_hbm_traffic.md") for w in ("cfg4", "cfg5")}


def kernel_sources_sha():
    import hashlib
    h = hashlib.sha256()
    for name in KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_2505_06641_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def measured_traffic(workload):
    """(bytes per launch or None, where the figure comes from)."""
    rel = PROFILE_FILES.get(workload)
    if rel is None:
        return None, None
    try:
        sha = kernel_sources_sha()
        with open(os.path.join(ROOT, rel)) as f:
            for line in f:
                t = line.split()
                if len(t) == 5 and t[0] == "scoring_kernel_traffic" and t[1] == workload:
                    kv = dict(x.split("=", 1) for x in t[2:])
                    if kv.get("kernel_sources_sha256") == sha:
                        return float(kv["fetch_bytes"]) + float(kv["write_bytes"]), rel
                    return None, rel + " (taken on other kernel sources: not reported)"
    except (OSError, ValueError, KeyError):
        pass
    return None, None


def scoring_flops_per_request(p, a):
    """Algorithmic flops of the head and the EA contraction for one request of application a."""
    d, H, C, M = int(p.feat_dim), int(p.hidden_dim), int(p.n_classes[a]), int(p.n_models[a])
    head = 2 * d * C if H == 0 else 2 * (d * H + H * C)
    return head + 2 * C * M


def cpu_baseline(w, n_sample, rounds, policy=None, threads=None):
    """The oracle, as it stands (NumPy float64; its matrix products run in NumPy's BLAS), on the first
    n_sample requests of the same workload; threads: None = whatever the BLAS takes, or a limit."""
    from oracle import sneakpeek_oracle as orc
    from paper_2505_06641_amd import workloads as wl
    if threads is not None:
        from threadpoolctl import threadpool_limits
        with threadpool_limits(limits=int(threads)):
            out = cpu_baseline(w, n_sample, rounds, policy, None)
        out["cores"] = int(threads)
        return out
    try:
        from threadpoolctl import threadpool_info
        cores = max([int(i.get("num_threads", 1)) for i in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    rq = w.requests
    sub = wl.Requests(x=rq.x[:n_sample], app=rq.app[:n_sample], deadline_rel_ms=rq.deadline_rel_ms[:n_sample],
                      weight=rq.weight[:n_sample])
    t0 = time.perf_counter()
    labels = None
    if policy is not None and getattr(policy, "split_groups", 0):
        ea, key, thetas = orc.score_requests(w.profile, sub, return_theta=True)
        labels = orc.split_labels(thetas)
    else:
        ea, key = orc.score_requests(w.profile, sub)
    t1 = time.perf_counter()
    win = orc.Window(w.profile, sub, ea=ea, key=key, policy=policy, sub=labels)
    win.run(max_rounds=rounds)
    t2 = time.perf_counter()
    p = w.profile
    cand = float(n_sample) * int(np.max(p.n_models)) * int(p.max_batch)
    return {"value": cand / (t2 - t0), "unit": "candidates/s", "cores": cores, "kind": "oracle",
            "sample": f"first {n_sample} of {rq.n} requests of {w.name} (full profile), scoring {t1 - t0:.2f} s + "
                      f"{win.round} rounds {t2 - t1:.2f} s, NumPy float64 with BLAS matrix products",
            "implementation": "NumPy/BLAS",
            "round_latency_us": (t2 - t1) / max(1, win.round) * 1e6}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="cfg5", choices=["cfg1", "cfg2", "cfg3", "cfg4", "cfg5"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample", type=int, default=0)
    ap.add_argument("--policy", default="sneakpeek",
                    choices=["sneakpeek", "alg1", "lo_priority", "lo_edf", "maxacc_edf"],
                    help="scheduling policy (Sec. 6.1 baselines, Alg. 1 as printed); default: the joint arg max")
    ap.add_argument("--split-groups", action="store_true", help="data-aware subgroups per predicted class (Sec. 5.3.2)")
    ap.add_argument("--priors", action="store_true", help="Dirichlet priors of the three kinds of Sec. 6.3 on the applications")
    ap.add_argument("--swap-costs", action="store_true", help="swap-in cost of 0.5-8 ms per variant")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="before the steps, run one elementwise copy of 256 MiB (reads 256 MiB, writes 256 MiB): "
                         "the known-size kernel that hardware byte counters of a profiler run are scaled by")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this library runs on one GPU only (the path would shard by application); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2505_06641_amd import binding, workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    w = wl.make(args.workload)
    p, rq = w.profile, w.requests
    n, A = rq.n, int(p.n_apps)
    m_max, B = int(np.max(p.n_models)), int(p.max_batch)
    rounds = w.rounds                      # <= 0: until the queue is exhausted
    if args.priors:
        wl.attach_priors(p, seed=1000 + w.seed)
    if args.swap_costs:
        wl.attach_swap_costs(p, seed=2000 + w.seed)
    policy = None if (args.policy == "sneakpeek" and not args.split_groups) else wl.named_policy(args.policy)
    if args.split_groups:
        policy.split_groups = 1
    ctx = binding.Context(p, n, policy=policy)
    x, app, D, wt = binding.to_device(rq)
    model = torch.empty(n, dtype=torch.int32, device="cuda:0")
    rnd = torch.empty(n, dtype=torch.int32, device="cuda:0")
    order = torch.empty(n, dtype=torch.int32, device="cuda:0")
    util = torch.empty(n, device="cuda:0")
    ctx.sp_set_timing(1)
    if args.calibrate_copy:
        src = torch.ones(64 * 1024 * 1024, device="cuda:0")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        torch.mul(src, 1.0, out=dst)
        torch.cuda.synchronize()
        del src, dst

    def step():
        ctx.sp_score(x, app, D, wt)
        return ctx.sp_schedule(rounds, model, rnd, order, util, log_capacity=0)

    # The timed steps carry the two events around the scoring kernel and nothing else: an event between two
    # kernels keeps the second from starting right behind the first, and one after every stage would add
    # about 40 us to a step.  The stage times come from a second pass of as many steps with all the events.
    ctx.sp_set_timing(3)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    k_ms, group_ms, order_ms, rounds_ms, finish_ms, copy_ms = [], [], [], [], [], []
    n_rounds = 0
    n_evals = 0
    t0 = time.perf_counter()
    for _ in range(args.steps):
        rc, summ, _ = step()
        k_ms.append(ctx.sp_get_timing()["score_kernel_ms"])   # waits only for events that the step has already waited for
        n_rounds = summ["n_rounds"]
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ctx.sp_set_timing(1)
    step()
    torch.cuda.synchronize()
    s0 = time.perf_counter()
    for _ in range(args.steps):
        step()
        tm = ctx.sp_get_timing()
        group_ms.append(tm["group_ms"]); order_ms.append(tm["order_ms"]); rounds_ms.append(tm["rounds_ms"])
        finish_ms.append(tm["finish_order_ms"]); copy_ms.append(tm["copy_outputs_ms"])
        n_evals = tm["utility_evaluations"]
    torch.cuda.synchronize()
    ms_per_step_all_events = (time.perf_counter() - s0) * 1e3 / args.steps
    # per-round latencies from one extra, untimed step with an event after every round
    ctx.sp_set_timing(2)
    step()
    per_round = [v * 1e3 for v in ctx.sp_get_round_times()][:max(1, n_rounds)]
    # and the latency of single sp_greedy_round calls (one round per call, host synchronisation included)
    ctx.sp_set_timing(0)
    ctx.sp_score(x, app, D, wt)
    torch.cuda.synchronize()
    call_us = []
    for _ in range(max(1, min(n_rounds, 64))):
        c0 = time.perf_counter()
        rc, _ = ctx.sp_greedy_round()
        call_us.append((time.perf_counter() - c0) * 1e6)
        if rc != binding.SP_OK:
            break
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    cand = float(n) * m_max * B
    value = cand / (ms_per_step * 1e-3)

    counts = np.bincount(rq.app, minlength=A)
    flops = float(sum(int(counts[a]) * scoring_flops_per_request(p, a) for a in range(A)))
    k_avg = float(np.mean(k_ms))
    elem = 2 if p.feat_dtype == wl.BF16 else 4
    k_bytes = float(n) * (int(p.feat_dim) * elem + m_max * 4 + 4 + 4 + 8)   # x row in; EA row, key, sort key out; D, w in
    tflops = flops / (k_avg * 1e-3) / 1e12
    gbs = k_bytes / (k_avg * 1e-3) / 1e9
    ai = flops / k_bytes
    split = p.feat_dtype == wl.F32 and int(p.hidden_dim) == 0 and int(p.feat_dim) <= 256
    mlp_mfma = p.feat_dtype == wl.BF16 and 0 < int(p.hidden_dim) <= 256 and int(p.feat_dim) % 8 == 0
    if mlp_mfma:
        # layer 1 is one bf16 MFMA per product; layer 2 and the table contraction take three fp16 MFMAs per
        # product (float32 hidden activations as hi + lo halves): the ceiling is the flop-weighted mix
        f1 = float(sum(int(counts[a]) * 2 * int(p.feat_dim) * int(p.hidden_dim) for a in range(A)))
        peak_c = flops / (f1 / PEAK_MFMA_BF16_TFLOPS + (flops - f1) / (PEAK_MFMA_F16_TFLOPS / 3.0))
        peak_note = "bf16 dense MFMA peak for layer 1, fp16 peak / 3 for layer 2 and the table, weighted by flops"
    elif p.feat_dtype == wl.BF16:
        peak_c, peak_note = PEAK_VALU_F32_TFLOPS, "float32 vector peak (generic kernel)"
    elif split:
        # the kernel forms every float32 product from three fp16 MFMAs (hi.hi + lo.hi + hi.lo), so its
        # ceiling for float32 flops is a third of the fp16 MFMA peak
        peak_c, peak_note = PEAK_MFMA_F16_TFLOPS / 3.0, "fp16 dense MFMA peak / 3 (three fp16 MFMAs per float32 product)"
    else:
        peak_c, peak_note = PEAK_VALU_F32_TFLOPS, "float32 vector peak (generic kernel)"
    ridge = peak_c * 1e12 / (PEAK_HBM_GBS * 1e9)
    if ai >= ridge:
        roof = {"bound": "mfma" if (split or mlp_mfma) else "alu", "achieved": tflops, "peak": peak_c, "unit": "TFLOP/s", "frac": tflops / peak_c}
    else:
        roof = {"bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS}
    if split or mlp_mfma:
        # what the matrix cores sustain on this device, measured now: the bare half-precision MFMA loop on
        # constant operands and on operands with random bits (the clock drops with the toggle rate, so the
        # second figure is the ceiling for real data); the kernel's ceiling scaled by sustained / published
        tf_const, ghz_const = binding.sp_debug_mfma_rate(False)
        tf_rand, ghz_rand = binding.sp_debug_mfma_rate(True)
        sustained = peak_c * tf_rand / PEAK_MFMA_F16_TFLOPS
        # the same loop with idle gaps (one wavefront per SIMD: 256 busy cycles, then about 64 * idle idle ones):
        # under the power limit the clock rises as the duty cycle falls, so the throughput on real data stays
        # near one level until the clock reaches its maximum
        duty = []
        for idle in (1, 2, 4, 8):
            tf_i, ghz_i = binding.sp_debug_mfma_rate(True, idle=idle)
            duty.append({"idle": idle, "tflops": tf_i, "clock_ghz": ghz_i,
                         "duty_cycle": tf_i / (1024 * 1024 * ghz_i * 1e9 / 1e12) if ghz_i > 0 else None})
        roof["mfma_f16_measured"] = {"constant_operands_tflops": tf_const, "constant_operands_clock_ghz": ghz_const,
                                     "random_operands_tflops": tf_rand, "random_operands_clock_ghz": ghz_rand,
                                     "peak_scaled_to_random_operands": sustained, "frac_of_that": tflops / sustained,
                                     "random_operands_with_idle_gaps": duty}
    traffic, traffic_source = measured_traffic(args.workload)
    roof.update({"kernel": "fused posterior/EA/key scoring kernel", "kernel_ms": k_avg, "traffic": traffic,
                 "traffic_source": traffic_source,
                 "peak_note": peak_note, "x_fp32_mfma_peak": tflops / PEAK_MFMA_F32_TFLOPS,
                 "algorithmic_flops": flops, "algorithmic_bytes": k_bytes, "hbm_gbs": gbs, "tflops": tflops})

    out = {
        "metric": METRIC, "value": value, "unit": "candidates/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16" if p.feat_dtype == wl.BF16 else ("f32 (fp16 hi/lo split MFMA, f32 accumulate)" if split else "f32"), "data": "synthetic",
        "config": {"workload": f"{w.name}: {A} applications, C={int(np.max(p.n_classes))}, M={m_max}, B={B}, "
                               f"N={n}, d={int(p.feat_dim)}, H={int(p.hidden_dim)}, seed {w.seed}; "
                               f"one scoring pass + {'greedy rounds until exhausted' if rounds <= 0 else str(rounds) + ' greedy rounds'}",
                   "n_requests": n, "rounds_run": n_rounds, "policy": args.policy, "priors": bool(args.priors),
                   "swap_costs": bool(args.swap_costs), "split_groups": bool(args.split_groups),
                   "rounds_path": "one launch" if ctx.rounds_in_one_launch else "two kernels per round"},
        "greedy_round_latency_us": {"mean": float(np.mean(per_round)) if per_round else None,
                                    "p50": float(np.percentile(per_round, 50)) if per_round else None,
                                    "p99": float(np.percentile(per_round, 99)) if per_round else None,
                                    "rounds": len(per_round),
                                    "single_call_mean": float(np.mean(call_us)), "single_call_p50": float(np.percentile(call_us, 50)),
                                    "single_call_p99": float(np.percentile(call_us, 99))},
        "stage_ms": {"group_by_app": float(np.mean(group_ms)), "score_kernel": k_avg,
                     "order_by_key": float(np.mean(order_ms)), "rounds": float(np.mean(rounds_ms)),
                     "note": "score_kernel: events in the timed steps; the other stages: a second pass of as many "
                             "steps with an event after every stage",
                     "ms_per_step_with_all_stage_events": ms_per_step_all_events},
        "roofline": roof,
    }
    # utility evaluations the rounds really performed (per round and (group, variant): nb (nb + 1) / 2 terms
    # for a candidate window of nb requests), counted by the kernels themselves
    r_ms = float(np.mean(rounds_ms))
    out["utility_evaluations"] = {"per_step": int(n_evals), "per_round_mean": float(n_evals) / max(1, n_rounds),
                                  "per_s": float(n_evals) / (r_ms * 1e-3) if r_ms > 0 else None}
    # the streaming stages against the HBM roofline: algorithmic bytes (what each has to read and write,
    # 4-byte ids / keys / positions) over the stage time from HIP events
    N = float(n)
    g_ms, o_ms, f_ms, c_ms = float(np.mean(group_ms)), float(np.mean(order_ms)), float(np.mean(finish_ms)), float(np.mean(copy_ms))

    def stream(name, nbytes, ms, note):
        gbs_ = nbytes / (ms * 1e-3) / 1e9 if ms > 0 else None
        return {"name": name, "algorithmic_bytes": nbytes, "ms": ms, "gbs": gbs_,
                "frac_of_hbm_peak": gbs_ / PEAK_HBM_GBS if gbs_ else None, "what": note}
    # applications that fit one workgroup's LDS are ordered by one kernel that reads and writes each (key,
    # position) pair once; longer ones take four radix passes over tiles (Sec. 5.2, eq. 12 ordering)
    in_lds = (not args.split_groups) and A <= 1024 and int(np.max(counts)) <= 16384
    order_b = 16 if in_lds else 68
    order_note = ("one kernel per application: (key, position) read (8 B) and written (8 B) once, four passes in LDS" if in_lds
                  else "digit totals of the keys (4 B) + four radix passes (8 B read, 8 B written each)")
    out["kernels"] = [
        stream("group_by_app", 32 * N, g_ms, "digit totals of the application ids (4 B read per request) + one radix pass (id 4 B, deadline and weight 8 B read; id, position 8 B and deadline, weight 8 B written)"),
        stream("order_by_key_passes", order_b * N, o_ms - f_ms, order_note),
        stream("finish_order", 57 * N, f_ms, "position, 16-byte record and key read; id, deadline, weight, key, pending flag written; outputs reset"),
        stream("copy_outputs", 32 * N, c_ms, "four per-request outputs read and written"),
    ]
    out["hbm_copy_measured_gbs"] = binding.sp_debug_copy_rate(1 << 28)
    # the whole step against the scoring kernel's ceilings: its algorithmic flops and the algorithmic bytes of
    # every stage over the step's wall time (the rounds work on LDS-resident windows: no bytes counted for them)
    step_bytes = k_bytes + (32 + order_b + 57 + 32) * N
    out["whole_step_roofline"] = {"algorithmic_flops": flops, "algorithmic_bytes": step_bytes,
                                  "tflops": flops / (ms_per_step * 1e-3) / 1e12,
                                  "frac_of_scoring_kernel_ceiling": flops / (ms_per_step * 1e-3) / 1e12 / peak_c,
                                  "gbs": step_bytes / (ms_per_step * 1e-3) / 1e9,
                                  "frac_of_hbm_peak": step_bytes / (ms_per_step * 1e-3) / 1e9 / PEAK_HBM_GBS}
    if not args.no_cpu_baseline:
        default_sample = {"cfg1": n, "cfg2": n, "cfg3": n, "cfg4": 65536, "cfg5": 1048576}[args.workload]
        ns = min(n, args.cpu_sample or default_sample)
        out["cpu_baseline"] = cpu_baseline(w, ns, rounds, policy)
        # and on one thread, on a sixteenth of that sample at the largest sizes so that it stays within seconds
        ns1 = ns if ns <= 65536 else ns // 16
        one = cpu_baseline(w, ns1, rounds, policy, threads=1)
        out["cpu_baseline"]["one_thread"] = {k: one[k] for k in ("value", "unit", "cores", "sample", "round_latency_us")}
    ctx.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
