"""Parity of the HIP library against the CPU oracle, through the C ABI.

Tolerances: 1e-5 relative (denominator max(|ref|, 1e-6)) on expected
accuracies, keys, scores and utilities for float32 features; for the bfloat16
config 2e-3 on posteriors (absolute) and on EA.  Decisions must match exactly
or be tolerance ties as defined in tests/parity.py.
"""
import copy

import numpy as np
import pytest

from oracle import sneakpeek_oracle as orc
from paper_2505_06641_amd import workloads as wl
from tests import parity

pytestmark = pytest.mark.gpu

TOL = 1e-5
BF16_EA_DERIVED = 1e-5      # bound on EA and key errors of the bf16 kernels that follows from their arithmetic


@pytest.fixture(scope="module")
def gpu():
    torch = pytest.importorskip("torch")
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible: the gpu-marked tests need a real MI355X")
    from paper_2505_06641_amd import binding
    binding.load_library()
    return torch, binding


def run_window(gpu, w, max_rounds, ctx=None, want_cube=False, policy=None, n_groups=None):
    """Score + schedule one workload through the C ABI; everything back on the host."""
    torch, binding = gpu
    p, rq = w.profile, w.requests
    n = rq.n
    own = ctx is None
    if own:
        ctx = binding.Context(p, max(n, 1), policy=policy)
    x, app, D, wt = binding.to_device(rq)
    ea = torch.full((n, ctx.m_max), -7.0, device="cuda:0")
    key = torch.full((n,), -7.0, device="cuda:0")
    ctx.sp_score(x, app, D, wt, ea_out=ea, key_out=key)
    out = {"ctx": ctx}
    order = torch.zeros(max(n, 1), dtype=torch.int32, device="cuda:0")
    seg = torch.zeros(p.n_apps + 1, dtype=torch.int32, device="cuda:0")
    ctx.sp_debug_dump(binding.SP_DUMP_ORDER, order)
    ctx.sp_debug_dump(binding.SP_DUMP_SEGMENTS, seg)
    out["order"], out["seg"] = order.cpu().numpy()[:n], seg.cpu().numpy()
    if want_cube:
        cube = torch.zeros((n_groups or p.n_apps, ctx.m_max, p.max_batch), device="cuda:0")
        ctx.sp_debug_dump(binding.SP_DUMP_SCORE_CUBE, cube)
        out["cube"] = cube.cpu().numpy()
    model = torch.full((max(n, 1),), 99, dtype=torch.int32, device="cuda:0")
    rnd = torch.full((max(n, 1),), 99, dtype=torch.int32, device="cuda:0")
    ordr = torch.full((max(n, 1),), 99, dtype=torch.int32, device="cuda:0")
    util = torch.full((max(n, 1),), -7.0, device="cuda:0")
    rc, summ, log = ctx.sp_schedule(max_rounds, model, rnd, ordr, util, log_capacity=max(n, 1))
    out.update(rc=rc, summary=summ, log=log, ea=ea.cpu().numpy(), key=key.cpu().numpy(),
               model=model.cpu().numpy()[:n], round_of=rnd.cpu().numpy()[:n], order_of=ordr.cpu().numpy()[:n],
               util=util.cpu().numpy()[:n], x=x, app=app)
    if own:
        out["close"] = ctx.close
    return out


def full_parity(gpu, w, max_rounds, tol=TOL, ea_tol=None, want_cube=False, policy=None):
    torch, binding = gpu
    p, rq = w.profile, w.requests
    sub, n_groups, border = None, None, []
    if policy is not None and getattr(policy, "split_groups", 0):
        # Subgroup labels (Sec. 5.3.2) from the head's own posterior.  The library sees every request.  Rule
        # for labels: they must equal the oracle's, except for requests whose largest oracle probability is
        # within 1e-4 of one half, where float32 and float64 may legitimately fall on different sides: for
        # those (`border`) either label is accepted, and the one the library took is read off its order.
        plain = copy.copy(p)
        plain.prior_alpha = None
        _, _, thetas = orc.score_requests(plain, rq, return_theta=True)
        top = np.array([float(np.max(t)) for t in thetas])
        arg = np.array([int(np.argmax(t)) for t in thetas])
        border = [int(i) for i in np.nonzero(np.abs(top - 0.5) <= 1e-4)[0]]
        assert len(border) <= 10, "too many requests at the labelling threshold for this test to resolve"
        sub = orc.split_labels(thetas)
        n_groups = len(set(zip(rq.app.tolist(), sub.tolist()))) + len(border)
    ea_ref, key_ref = orc.score_requests(p, rq)
    got = run_window(gpu, w, max_rounds, want_cube=want_cube, policy=policy, n_groups=n_groups)
    if border:
        # the labelling of the borderline requests that reproduces the library's order, if there is one
        def order_of(labels):
            w0 = orc.Window(p, rq, ea=ea_ref, key=key_ref, policy=policy, sub=labels)
            return np.concatenate([w0.order[g] for a in range(p.n_apps) for g in range(w0.G) if w0.gapp[g] == a])
        found = None
        for bits in range(1 << len(border)):
            trial = sub.copy()
            for k, i in enumerate(border):
                trial[i] = 1 + arg[i] if (bits >> k) & 1 else 0
            if np.array_equal(order_of(trial), got["order"][:got["seg"][p.n_apps]]):
                found = trial
                break
        assert found is not None, "no admissible labelling of the borderline requests gives the library's order"
        sub = found
    if sub is not None:
        n_groups = len(set(zip(rq.app.tolist(), sub.tolist())))
        if want_cube:
            got["cube"] = got["cube"][:n_groups]
    stats = {}
    stats["ea_rel"] = parity.assert_close("EA", got["ea"], ea_ref, ea_tol or tol)
    stats["key_rel"] = parity.assert_close("key", got["key"], key_ref, ea_tol or tol, floor=1e-30)
    # bfloat16 configs are allowed 2e-3 (ea_tol), but the arithmetic says they do as well as float32 ones:
    # bf16 features and weights are exact in both implementations, layer 1 multiplies them exactly and
    # accumulates in float32, the hidden activations stay float32, so only float32 roundings remain
    assert stats["ea_rel"] <= BF16_EA_DERIVED and stats["key_rel"] <= BF16_EA_DERIVED, stats
    edf = policy is not None and policy.order == wl.ORDER_EDF
    omega = -orc.widen(rq.deadline_rel_ms) if edf else key_ref
    if sub is None:
        stats["order_swaps"] = parity.check_order(got["order"], got["seg"], rq.app, omega, p.n_apps, tol)
    else:
        # inside an application: subgroups in ascending order, each by descending ordering value
        w0 = orc.Window(p, rq, ea=ea_ref, key=key_ref, policy=policy, sub=sub)
        for a in range(p.n_apps):
            want = np.concatenate([w0.order[g] for g in range(w0.G) if w0.gapp[g] == a] or [np.zeros(0, dtype=np.int64)])
            have = got["order"][got["seg"][a]:got["seg"][a + 1]]
            assert np.array_equal(have, want), f"app {a}: order inside the subgroups differs"
        stats["order_swaps"] = 0
    if want_cube:
        ref_cube = orc.Window(p, rq, ea=ea_ref, key=key_ref, policy=policy, sub=sub).score_cube()
        valid = np.isfinite(ref_cube)
        assert np.array_equal(got["cube"] >= 0, valid), "candidate sets differ"
        stats["cube_rel"] = parity.assert_close("score cube", got["cube"][valid], ref_cube[valid], tol, floor=1e-12)
    members = parity.members_by_round(got["round_of"], got["order_of"], len(got["log"]))
    win, rstats = parity.replay(p, rq, ea_ref, key_ref, got["log"], members, got["summary"]["done"] == 1, tol,
                                policy=policy, sub=sub)
    stats.update(rstats)
    stats["util_rel"] = parity.check_outputs(win, got["model"], got["round_of"], got["order_of"], got["util"],
                                             got["summary"], tol)
    got["close"]()
    got["workload"] = w
    print(w.name, stats)
    return got, stats


def test_cfg1_scoring_cube_and_one_round(gpu):
    torch, binding = gpu
    w = wl.make("cfg1")
    got, stats = full_parity(gpu, w, max_rounds=1, want_cube=True)
    assert got["rc"] == binding.SP_OK and got["summary"]["n_rounds"] == 1
    assert stats["ties"] == 0 and stats["order_swaps"] == 0


def test_cfg2_full_schedule(gpu):
    torch, binding = gpu
    w = wl.make("cfg2")
    got, stats = full_parity(gpu, w, max_rounds=0, want_cube=True)
    assert got["rc"] == binding.SP_DONE and got["summary"]["done"] == 1
    assert stats["exact"] + stats["ties"] == got["summary"]["n_rounds"] > 10
    assert stats["ties"] <= 2


def test_cfg3_full_schedule_tight_deadlines(gpu):
    torch, binding = gpu
    w = wl.make("cfg3")
    got, stats = full_parity(gpu, w, max_rounds=0, want_cube=True)
    assert got["rc"] == binding.SP_DONE
    assert got["summary"]["n_dropped"] > 0 and got["summary"]["n_scheduled"] > 0
    assert stats["ties"] <= 2


def test_cfg4_bf16_posteriors_and_rounds(gpu):
    torch, binding = gpu
    w = wl.make("cfg4")
    p, rq = w.profile, w.requests
    got, stats = full_parity(gpu, w, max_rounds=64, ea_tol=2e-3, want_cube=True)
    # the queue may run dry before the 64th round (replay has already checked that it really is dry)
    assert got["summary"]["n_rounds"] == 64 or (got["rc"] == binding.SP_DONE and 0 < got["summary"]["n_rounds"] < 64)
    # posteriors from the library's logits against the oracle's, on a sample of requests
    ctx = binding.Context(p, rq.n)
    x, app, D, wt = binding.to_device(rq)
    ctx.sp_score(x, app, D, wt)
    z = torch.zeros((rq.n, ctx.c_max), device="cuda:0")
    ctx.sp_debug_dump(binding.SP_DUMP_LOGITS, z, x=x, app=app)
    z = z.cpu().numpy()
    ctx.close()
    sample = np.random.default_rng(0).choice(rq.n, 2048, replace=False)
    for a in range(p.n_apps):
        ids = sample[rq.app[sample] == a]
        th_ref = orc.posterior(orc.head_logits(rq.x[ids], p.W1[a], p.b1[a], p.W2[a], p.b2[a]))
        th_got = orc.posterior(z[ids, : p.n_classes[a]])
        assert np.max(np.abs(th_got - th_ref)) <= 2e-3


@pytest.mark.parametrize("kind", [wl.PEN_STEP, wl.PEN_LINEAR, wl.PEN_SIGMOID])
def test_ragged_applications_all_penalties(gpu, kind):
    w = wl.tiny(seed=40 + kind, n=3000, classes=(5, 1, 130, 2), models=(3, 1, 16, 7), max_batch=37, feat_dim=19,
                hidden_dim=0, penalty=kind, deadline=(4.0, 60.0), fractions=(0.4, 0.1, 0.3, 0.2))
    got, stats = full_parity(gpu, w, max_rounds=0, want_cube=True)
    assert got["summary"]["done"] == 1


def test_ragged_mlp_head(gpu):
    w = wl.tiny(seed=50, n=1500, classes=(3, 70), models=(2, 5), max_batch=8, feat_dim=33, hidden_dim=17,
                deadline=(4.0, 80.0))
    full_parity(gpu, w, max_rounds=0, want_cube=True)


def test_bf16_ragged(gpu):
    w = wl.tiny(seed=51, n=700, classes=(3, 9), models=(2, 3), max_batch=5, feat_dim=24, hidden_dim=10,
                feat_dtype=wl.BF16, deadline=(4.0, 80.0))
    full_parity(gpu, w, max_rounds=0, ea_tol=2e-3)


@pytest.mark.parametrize("head", ["logistic", "mlp_f32", "mlp_bf16"])
def test_dirichlet_priors_on_every_scoring_kernel(gpu, head):
    """Sec. 4.2 eq. (10)-(11): priors of the three kinds of Sec. 6.3 and one application without a prior."""
    kw = dict(classes=(5, 12, 130, 2), models=(3, 1, 16, 7), max_batch=9, deadline=(4.0, 60.0), fractions=(0.4, 0.1, 0.3, 0.2))
    if head == "logistic":
        w = wl.tiny(seed=90, n=2500, feat_dim=19, hidden_dim=0, **kw)
    elif head == "mlp_f32":
        w = wl.tiny(seed=91, n=1200, feat_dim=33, hidden_dim=17, **kw)
    else:
        w = wl.tiny(seed=92, n=1500, feat_dim=24, hidden_dim=10, feat_dtype=wl.BF16, **kw)
    wl.attach_priors(w.profile, seed=93)
    plain, _ = orc.score_requests(wl.tiny(seed=w.seed, n=w.requests.app.shape[0], feat_dim=w.profile.feat_dim,
                                          hidden_dim=w.profile.hidden_dim, feat_dtype=w.profile.feat_dtype, **kw).profile,
                                  w.requests)
    smooth, _ = orc.score_requests(w.profile, w.requests)
    assert np.max(np.abs(plain - smooth)) > 1e-3          # the priors do move the estimates
    full_parity(gpu, w, max_rounds=0, ea_tol=2e-3 if head == "mlp_bf16" else None, want_cube=head != "mlp_bf16")


@pytest.mark.parametrize("name", ["sneakpeek", "alg1"])
def test_data_oblivious_baselines_are_a_prior_without_evidence(gpu, name):
    """Sec. 6.1: the data-oblivious approaches use the profiled accuracy under the profiling label mix for
    every request of an application: a prior equal to that mix and no evidence (Sec. 4.1, fallback of eq. 9)."""
    w = wl.tiny(seed=96, n=1800, classes=(5, 12, 40), models=(3, 2, 6), max_batch=7, feat_dim=21, deadline=(4.0, 90.0))
    wl.attach_priors(w.profile, seed=97, kinds=("weak", "strong"))
    w.profile.evidence_k[:] = 0.0
    ea_ref, _ = orc.score_requests(w.profile, w.requests)
    for a in range(3):
        rows = ea_ref[w.requests.app == a]
        assert np.ptp(rows, axis=0).max() == 0.0          # one row per application, whatever the request holds
    full_parity(gpu, w, max_rounds=0, policy=wl.named_policy(name), want_cube=True)


def test_prior_can_be_removed_and_bad_priors_are_rejected(gpu):
    torch, binding = gpu
    w = wl.tiny(seed=94, n=300, classes=(4, 6), models=(2, 3), max_batch=4, feat_dim=8)
    ea_plain, _ = orc.score_requests(w.profile, w.requests)
    ctx = binding.Context(w.profile, 300)
    x, app, D, wt = binding.to_device(w.requests)
    ctx.sp_set_prior(1, np.array([2.0, 0.5, 0.5, 1.0, 3.0, 0.25], dtype=np.float32), 5.0)
    ea = torch.zeros((300, ctx.m_max), device="cuda:0")
    ctx.sp_score(x, app, D, wt, ea_out=ea)
    ea1 = ea.cpu().numpy()
    ctx.sp_set_prior(1, None, 0.0)
    ctx.sp_score(x, app, D, wt, ea_out=ea)
    ea2 = ea.cpu().numpy()
    assert np.max(np.abs(ea1 - ea_plain)) > 1e-3
    parity.assert_close("EA", ea2, ea_plain, TOL)
    for bad_alpha, k in (([1.0, -0.1, 1.0, 1.0], 1.0), ([1.0, float("nan"), 1.0, 1.0], 1.0), ([0.0] * 4, 0.0),
                         ([1.0] * 4, -1.0)):
        with pytest.raises(binding.SneakPeekError) as e:
            ctx.sp_set_prior(0, np.asarray(bad_alpha, dtype=np.float32), k)
        assert e.value.status == binding.SP_EINVAL
    with pytest.raises(binding.SneakPeekError) as e:
        ctx.sp_set_prior(2, np.ones(4, dtype=np.float32), 1.0)
    assert e.value.status == binding.SP_EINVAL
    ctx.close()


def test_batch_of_one(gpu):
    w = wl.tiny(seed=52, n=200, classes=(4, 3), models=(3, 2), max_batch=1, feat_dim=8, deadline=(3.0, 40.0))
    got, stats = full_parity(gpu, w, max_rounds=0, want_cube=True)
    assert all(r["batch"] == 1 for r in got["log"])


def test_fewer_requests_than_batch_and_single_request(gpu):
    for n in (1, 3):
        w = wl.tiny(seed=60 + n, n=n, classes=(4,), models=(2,), max_batch=16, feat_dim=8, deadline=(50.0, 90.0))
        got, stats = full_parity(gpu, w, max_rounds=0, want_cube=True)
        assert got["summary"]["n_scheduled"] == n


def test_empty_window(gpu):
    torch, binding = gpu
    w = wl.tiny(seed=70, n=0, classes=(4, 2), models=(2, 2))
    got = run_window(gpu, w, max_rounds=0)
    assert got["rc"] == binding.SP_DONE
    assert got["summary"] == {"total_weighted_utility": 0.0, "mean_utility": 0.0, "total_violation_ms": 0.0,
                              "n_rounds": 0, "n_scheduled": 0, "n_dropped": 0, "done": 1}
    rc, dec = got["ctx"].sp_greedy_round()
    assert rc == binding.SP_DONE and dec is None
    got["close"]()


def test_all_dead_queue(gpu):
    torch, binding = gpu
    w = wl.tiny(seed=71, n=50, classes=(4,), models=(2,), penalty=wl.PEN_STEP, deadline=(0.01, 0.02))
    got, stats = full_parity(gpu, w, max_rounds=0)
    assert got["summary"]["n_scheduled"] == 0 and got["summary"]["n_dropped"] == 50 and got["rc"] == binding.SP_DONE
    assert np.all(got["model"] == -1) and np.all(got["round_of"] == -1) and np.all(got["order_of"] == 0)


def test_duplicate_keys_fall_back_to_request_id(gpu):
    w = wl.tiny(seed=72, n=400, classes=(3, 2), models=(2, 2), max_batch=6, feat_dim=4, deadline=(30.0, 30.0))
    rq = w.requests
    rq.x[:] = rq.x[0]                       # identical features -> identical EA within an application
    rq.deadline_rel_ms[:] = 30.0
    rq.weight[:] = np.float32(0.5)
    got, stats = full_parity(gpu, w, max_rounds=0)
    for a in range(2):
        mine = got["order"][got["seg"][a]:got["seg"][a + 1]]
        assert np.all(np.diff(mine) > 0)     # equal keys: ascending request id


@pytest.mark.parametrize("head", ["generic", "mfma"])
def test_weight_of_negative_zero_sorts_with_the_zeros(gpu, head):
    # a weight of -0.0 gives the key 0 like +0.0: such requests are served last in their application, by id
    if head == "generic":
        w = wl.tiny(seed=73, n=300, classes=(3, 2), models=(2, 2), max_batch=6, feat_dim=4, hidden_dim=3)
    else:
        w = wl.tiny(seed=74, n=300, classes=(5, 2), models=(3, 2), max_batch=6, feat_dim=8)
    rq = w.requests
    rq.weight[1::7] = np.float32(0.0)
    rq.weight[::5] = np.float32(-0.0)
    zero = rq.weight == 0
    assert np.signbit(rq.weight[::5]).all() and not np.signbit(rq.weight[1::35][rq.weight[1::35] == 0]).all()
    got, stats = full_parity(gpu, w, max_rounds=0)
    assert np.all(got["key"] == 0.0) or np.any(got["key"] > 0)
    assert not np.signbit(got["key"]).any()
    for a in range(2):
        mine = got["order"][got["seg"][a]:got["seg"][a + 1]]
        nz = int(np.sum(zero[mine]))
        assert nz > 0 and zero[mine[-nz:]].all() and not zero[mine[:-nz]].any()
        assert np.all(np.diff(mine[-nz:]) > 0)


def test_exact_score_ties_pick_smallest_candidate(gpu):
    w = wl.tiny(seed=900, n=6, classes=(3, 3), models=(2, 2), max_batch=2, deadline=(1e3, 1e3))
    p, r = w.profile, w.requests
    r.app[:] = [0, 1, 0, 1, 0, 1]
    r.x[1::2] = r.x[0::2]
    r.deadline_rel_ms[:] = 1e3
    r.weight[:] = 0.5
    p.W1[1][:] = p.W1[0]
    p.acc[0][1] = p.acc[0][0]
    p.acc[1][:] = p.acc[0]
    p.lat_ms[1][:] = p.lat_ms[0]
    got, stats = full_parity(gpu, w, max_rounds=1, want_cube=True)
    c = got["cube"]
    assert c[0, 0, 1] == c[0, 1, 1] == c[1, 0, 1] == c[1, 1, 1]
    assert (got["log"][0]["app"], got["log"][0]["model"], got["log"][0]["batch"]) == (0, 0, 2)


def test_short_circuit_variant(gpu):
    w = wl.tiny(seed=800, n=4, classes=(3,), models=(2,), max_batch=2, penalty=wl.PEN_STEP, deadline=(10.0, 10.0))
    w.requests.deadline_rel_ms[:] = 10.0
    w.profile.acc[0][0, :] = 0.9
    w.profile.acc[0][1, :] = 0.4
    w.profile.lat_ms[0][1, :] = 0.0
    w.profile.lat_ms[0][0, :] = [50.0, 60.0]
    got, stats = full_parity(gpu, w, max_rounds=1)
    assert got["log"][0]["model"] == 1 and got["log"][0]["t_end_ms"] == 0.0


def test_round_by_round_equals_schedule_and_is_deterministic(gpu):
    torch, binding = gpu
    w = wl.make("cfg2", n_requests=1500)
    a = run_window(gpu, w, max_rounds=0)
    b = run_window(gpu, w, max_rounds=0)
    for k in ("ea", "key", "order", "model", "round_of", "order_of", "util"):
        assert np.array_equal(a[k], b[k]), k
    assert a["log"] == b["log"] and a["summary"] == b["summary"]
    # the same window stepped one round at a time, with the member ids of every round
    ctx = b["ctx"]
    x, app, D, wt = binding.to_device(w.requests)
    ctx.sp_score(x, app, D, wt)
    ids = torch.zeros(w.profile.max_batch, dtype=torch.int32, device="cuda:0")
    members = parity.members_by_round(a["round_of"], a["order_of"], len(a["log"]))
    for r, rec in enumerate(a["log"]):
        rc, dec = ctx.sp_greedy_round(req_ids_out=ids)
        assert rc == binding.SP_OK and dec == rec
        assert np.array_equal(ids.cpu().numpy()[: rec["batch"]], members[r])
    rc, dec = ctx.sp_greedy_round()
    assert rc == binding.SP_DONE
    # resumable: a limited run followed by an unlimited one gives the same log
    ctx.sp_score(x, app, D, wt)
    rc, s1, log1 = ctx.sp_schedule(5, log_capacity=4096)
    assert rc == binding.SP_OK and s1["n_rounds"] == 5 and log1 == a["log"][:5]
    rc, s2, log2 = ctx.sp_schedule(0, log_capacity=4096)
    assert rc == binding.SP_DONE and log2 == a["log"] and s2 == a["summary"]
    a["close"]()
    b["close"]()


@pytest.mark.parametrize("name", ["alg1", "lo_priority", "lo_edf", "maxacc_edf", "edf_batched", "capped"])
def test_policies_of_the_evaluation_on_both_round_paths(gpu, name):
    """Sec. 6.1 "Baselines and Metrics" and Alg. 1 as printed, as knobs on the same kernels."""
    torch, binding = gpu
    policy = {"edf_batched": wl.Policy(order=wl.ORDER_EDF, weight=wl.WEIGHT_UNIT),
              "capped": wl.Policy(batch_cap=5, choice=wl.CHOICE_MAX_ACCURACY)}.get(name) or wl.named_policy(name)
    n = 600 if policy.batch_cap == 1 else 2400
    w = wl.tiny(seed=97, n=n, classes=(5, 3, 40, 2), models=(3, 2, 8, 5), max_batch=19, feat_dim=19,
                penalty=wl.PEN_LINEAR, deadline=(6.0, 150.0), fractions=(0.4, 0.1, 0.3, 0.2))
    w.profile.penalty[:] = [wl.PEN_LINEAR, wl.PEN_STEP, wl.PEN_SIGMOID, wl.PEN_LINEAR]
    got, stats = full_parity(gpu, w, max_rounds=0, want_cube=True, policy=policy)      # rounds in one launch
    assert got["summary"]["done"] == 1 and stats["rounds"] > 10
    if policy.batch_cap:
        assert max(r["batch"] for r in got["log"]) <= policy.batch_cap
    # the same window one round per call (two kernels per round)
    ctx = binding.Context(w.profile, n, policy=policy)
    x, app, D, wt = binding.to_device(w.requests)
    ctx.sp_score(x, app, D, wt)
    for rec in got["log"]:
        rc, dec = ctx.sp_greedy_round()
        assert rc == binding.SP_OK and dec == rec
    assert ctx.sp_greedy_round()[0] == binding.SP_DONE
    # back to the default policy: the window has to be scored again, and then runs as without a policy
    ctx.sp_set_policy(None)
    with pytest.raises(binding.SneakPeekError) as e:
        ctx.sp_schedule(0)
    assert e.value.status == binding.SP_ESTATE
    ctx.sp_score(x, app, D, wt)
    rc, summ, log = ctx.sp_schedule(0, log_capacity=4096)
    plain = run_window(gpu, w, 0)
    assert log == plain["log"] and summ == plain["summary"]
    plain["close"]()
    bad = wl.Policy(order=7)
    with pytest.raises(binding.SneakPeekError) as e:
        ctx.sp_set_policy(bad)
    assert e.value.status == binding.SP_EINVAL
    ctx.close()


@pytest.mark.parametrize("head", ["logistic", "mlp_f32", "mlp_bf16"])
@pytest.mark.parametrize("name", ["sneakpeek", "alg1"])
def test_data_aware_group_splitting(gpu, head, name):
    """Sec. 5.3.2: subgroups per predicted class, labelled by every scoring kernel, ordered and scheduled as
    groups of their own."""
    torch, binding = gpu
    kw = dict(classes=(2, 5, 33, 3), models=(3, 2, 6, 4), max_batch=11, deadline=(6.0, 150.0), fractions=(0.3, 0.2, 0.3, 0.2))
    if head == "logistic":
        w = wl.tiny(seed=98, n=2200, feat_dim=19, hidden_dim=0, **kw)
    elif head == "mlp_f32":
        w = wl.tiny(seed=99, n=1100, feat_dim=33, hidden_dim=17, **kw)
    else:
        w = wl.tiny(seed=100, n=1300, feat_dim=24, hidden_dim=10, feat_dtype=wl.BF16, **kw)
    for a in range(4):                          # sharper heads: a good share of confident requests
        if w.profile.feat_dtype == wl.BF16:
            w.profile.W1[a] = wl.f32_to_bf16_bits(wl.bf16_bits_to_f32(w.profile.W1[a]) * 2.0)
        else:
            w.profile.W1[a] = (w.profile.W1[a] * 3.0).astype(np.float32)
    policy = wl.named_policy(name)
    policy.split_groups = 1
    got, stats = full_parity(gpu, w, max_rounds=0, ea_tol=2e-3 if head == "mlp_bf16" else None, want_cube=True,
                             policy=policy)
    assert got["summary"]["done"] == 1 and stats["rounds"] > 10
    # round by round gives the same schedule (on the window full_parity actually ran)
    w = got["workload"]
    ctx = binding.Context(w.profile, w.requests.n, policy=policy)
    x, app, D, wt = binding.to_device(w.requests)
    ctx.sp_score(x, app, D, wt)
    # sp_schedule above ran the rounds in one launch (a resident workgroup serves all groups of its application);
    # one round per call below takes the two-kernel path: the two must agree decision for decision
    assert ctx.lib.sp_rounds_in_one_launch(ctx.h)
    for rec in got["log"]:
        rc, dec = ctx.sp_greedy_round()
        assert rc == binding.SP_OK and dec == rec
    assert ctx.sp_greedy_round()[0] == binding.SP_DONE
    ctx.close()


def test_group_splitting_beyond_what_a_resident_workgroup_serves(gpu):
    """More than 64 non-empty subgroups in one application: sp_schedule takes two kernels per round, with the
    same parity; an application with few subgroups beside it changes nothing."""
    torch, binding = gpu
    w = wl.tiny(seed=101, n=4000, classes=(120, 3), models=(3, 2), max_batch=9, feat_dim=24, deadline=(6.0, 150.0),
                fractions=(0.8, 0.2))
    w.profile.W1[0] = (w.profile.W1[0] * 8.0).astype(np.float32)       # sharp head: most requests are confident
    policy = wl.named_policy("sneakpeek")
    policy.split_groups = 1
    got, stats = full_parity(gpu, w, max_rounds=0, want_cube=True, policy=policy)
    assert got["summary"]["done"] == 1 and stats["rounds"] > 10
    ctx = binding.Context(w.profile, w.requests.n, policy=policy)
    x, app, D, wt = binding.to_device(w.requests)
    ctx.sp_score(x, app, D, wt)
    assert not ctx.lib.sp_rounds_in_one_launch(ctx.h)
    ctx.close()


@pytest.mark.parametrize("kind", [wl.PEN_STEP, wl.PEN_LINEAR, wl.PEN_SIGMOID])
def test_swap_in_costs_on_both_round_paths(gpu, kind):
    """Sec. 3.1 "context switch time" / Sec. 5.2 model locality: a batch pays its variant's swap-in cost
    unless the previous batch ran the same variant."""
    torch, binding = gpu
    w = wl.tiny(seed=95 + kind, n=2600, classes=(5, 3, 40, 2), models=(3, 2, 8, 5), max_batch=21, feat_dim=19,
                penalty=kind, deadline=(4.0, 120.0), fractions=(0.4, 0.1, 0.3, 0.2))
    wl.attach_swap_costs(w.profile, seed=96, lo=0.5, hi=9.0, skip_every=3)
    got, stats = full_parity(gpu, w, max_rounds=0, want_cube=True)       # sp_schedule: rounds in one launch
    # swap costs do show in the clock: some batch starts computing later than the previous one ended
    L = w.profile.lat_ms
    paid = [r for r in got["log"] if r["t_end_ms"] - r["t_start_ms"] > float(L[r["app"]][r["model"], r["batch"] - 1]) * (1 + 1e-6)]
    free = [r for r in got["log"] if r not in paid]
    assert paid and free
    # the same window one round per call (two kernels per round)
    ctx = binding.Context(w.profile, 2600)
    x, app, D, wt = binding.to_device(w.requests)
    ctx.sp_score(x, app, D, wt)
    for rec in got["log"]:
        rc, dec = ctx.sp_greedy_round()
        assert rc == binding.SP_OK and dec == rec
    assert ctx.sp_greedy_round()[0] == binding.SP_DONE
    # costs can be taken away again, and bad ones are rejected
    for a in range(4):
        ctx.sp_set_swap_cost(a, None)
    ctx.sp_score(x, app, D, wt)
    rc, summ, log = ctx.sp_schedule(0, log_capacity=4096)
    assert all(r["t_end_ms"] - r["t_start_ms"] == pytest.approx(float(L[r["app"]][r["model"], r["batch"] - 1]), rel=1e-6) for r in log)
    with pytest.raises(binding.SneakPeekError) as e:
        ctx.sp_set_swap_cost(0, np.array([1.0, -2.0, 0.0], dtype=np.float32))
    assert e.value.status == binding.SP_EINVAL
    with pytest.raises(binding.SneakPeekError) as e:
        ctx.sp_set_swap_cost(9, np.array([1.0], dtype=np.float32))
    assert e.value.status == binding.SP_EINVAL
    ctx.close()


def test_profile_too_large_for_the_one_launch_rounds_takes_the_two_kernel_path(gpu):
    """More (application, variant) pairs than resident workgroups fit: sp_schedule falls back to two kernels
    per round and takes the same decisions the oracle does."""
    torch, binding = gpu
    A = 90
    w = wl.tiny(seed=101, n=5000, classes=tuple(2 + (a % 5) for a in range(A)), models=tuple(9 + (a % 4) for a in range(A)),
                max_batch=7, feat_dim=12, deadline=(5.0, 90.0))
    assert int(np.sum(w.profile.n_models)) > 900
    got, stats = full_parity(gpu, w, max_rounds=0, want_cube=False)
    assert stats["rounds"] > 20 and got["summary"]["done"] == 1
    ctx = binding.Context(w.profile, 5000)
    assert not ctx.rounds_in_one_launch
    ctx.close()


def test_more_than_255_applications_two_pass_grouping(gpu):
    """Two radix passes over the application id, segment starts by search, many empty and tiny groups."""
    A = 300
    rng = np.random.default_rng(7)
    frac = rng.dirichlet(np.full(A, 0.3))
    w = wl.tiny(seed=102, n=4000, classes=tuple(2 + (a % 3) for a in range(A)), models=tuple(1 + (a % 3) for a in range(A)),
                max_batch=6, feat_dim=10, deadline=(5.0, 90.0), fractions=tuple(frac / frac.sum()))
    counts = np.bincount(w.requests.app, minlength=A)
    assert (counts == 0).any() and counts.max() > 50
    got, stats = full_parity(gpu, w, max_rounds=0, want_cube=True)
    assert got["summary"]["done"] == 1 and stats["rounds"] >= 20


def test_more_applications_than_the_segment_table_holds(gpu):
    """Beyond 1024 applications k_segments places tiles and units without its LDS tables, the scan's
    digit totals are one row per application, and the rounds run over more than a thousand groups."""
    A = 1100
    rng = np.random.default_rng(11)
    frac = rng.dirichlet(np.full(A, 0.5))
    w = wl.tiny(seed=103, n=6000, classes=tuple(2 + (a % 4) for a in range(A)), models=tuple(1 + (a % 2) for a in range(A)),
                max_batch=4, feat_dim=6, deadline=(5.0, 60.0), fractions=tuple(frac / frac.sum()))
    got, stats = full_parity(gpu, w, max_rounds=0, want_cube=False)
    assert stats["rounds"] >= 20 and got["summary"]["done"] == 1


def test_largest_batch_variant_and_class_counts(gpu):
    """B = 256 and M = 16 (the library's limits) with C well beyond one class tile, on the matrix-core kernel."""
    w = wl.tiny(seed=103, n=900, classes=(1500, 700), models=(16, 16), max_batch=256, feat_dim=64, deadline=(20.0, 900.0),
                alpha=(0.5, 3.0), beta=(0.05, 0.4))
    got, stats = full_parity(gpu, w, max_rounds=0, want_cube=True)
    assert max(r["batch"] for r in got["log"]) > 64 and got["summary"]["done"] == 1


def test_bf16_logistic_head_and_wide_fp32_head(gpu):
    """Heads outside the matrix-core kernels' shapes run on the generic kernel: bf16 without a hidden layer,
    fp32 wider than 256 features."""
    w = wl.tiny(seed=104, n=500, classes=(6, 11), models=(3, 4), max_batch=7, feat_dim=40, hidden_dim=0,
                feat_dtype=wl.BF16, deadline=(5.0, 90.0))
    full_parity(gpu, w, max_rounds=0, ea_tol=2e-3)
    w = wl.tiny(seed=105, n=300, classes=(9, 4), models=(2, 5), max_batch=5, feat_dim=300, hidden_dim=0, deadline=(5.0, 90.0))
    full_parity(gpu, w, max_rounds=0, want_cube=True)


def test_context_reuse_with_a_smaller_second_window(gpu):
    torch, binding = gpu
    big = wl.make("cfg2", n_requests=3000)
    small = wl.make("cfg2", n_requests=700, seed=5)
    small.profile = big.profile
    ctx = binding.Context(big.profile, 3000)
    first = run_window(gpu, big, 0, ctx=ctx)
    second = run_window(gpu, small, 0, ctx=ctx)
    alone = run_window(gpu, small, 0)
    for k in ("ea", "key", "order", "model", "round_of", "order_of", "util"):
        assert np.array_equal(second[k], alone[k]), k
    assert second["log"] == alone["log"] and first["summary"]["n_rounds"] > 0
    ctx.close()
    alone["close"]()


def test_error_paths(gpu):
    torch, binding = gpu
    w = wl.tiny(seed=80, n=100, classes=(4, 2), models=(2, 2), max_batch=4, feat_dim=8)
    ctx = binding.Context(w.profile, 100)
    with pytest.raises(binding.SneakPeekError) as e:
        ctx.sp_greedy_round()
    assert e.value.status == binding.SP_ESTATE
    with pytest.raises(binding.SneakPeekError) as e:
        ctx.sp_schedule(0)
    assert e.value.status == binding.SP_ESTATE
    x, app, D, wt = binding.to_device(w.requests)
    big = torch.zeros((101, 8), device="cuda:0")
    with pytest.raises(binding.SneakPeekError) as e:
        ctx.sp_score(big, torch.zeros(101, dtype=torch.int32, device="cuda:0"), torch.ones(101, device="cuda:0"),
                     torch.ones(101, device="cuda:0"))
    assert e.value.status == binding.SP_ECAPACITY
    for what in ("app_hi", "app_neg", "deadline", "deadline_nan", "weight"):
        a2, D2, w2 = app.clone(), D.clone(), wt.clone()
        if what == "app_hi":
            a2[17] = 2
        elif what == "app_neg":
            a2[3] = -1
        elif what == "deadline":
            D2[5] = 0.0
        elif what == "deadline_nan":
            D2[5] = float("nan")
        else:
            w2[99] = -0.5
        ctx.sp_score(x, a2, D2, w2)
        with pytest.raises(binding.SneakPeekError) as e:
            ctx.sp_schedule(0)
        assert e.value.status == binding.SP_EINVAL, what
        with pytest.raises(binding.SneakPeekError) as e:
            ctx.sp_greedy_round()
        assert e.value.status == binding.SP_EINVAL, what
    # the context recovers with a good window
    ctx.sp_score(x, app, D, wt)
    rc, summ, _ = ctx.sp_schedule(0)
    assert rc == binding.SP_DONE and summ["n_scheduled"] + summ["n_dropped"] == 100
    ctx.close()


def random_case(seed):
    """A small workload, a policy and the optional profile extras, all drawn from the seed."""
    rng = np.random.Generator(np.random.PCG64(7000 + seed))
    A = int(rng.integers(1, 6))
    classes = tuple(int(c) for c in np.where(rng.random(A) < 0.15, rng.integers(100, 300, A), rng.integers(2, 70, A)))
    models = tuple(int(m) for m in rng.integers(1, 17, A))
    head = ["logistic", "mlp_f32", "mlp_bf16", "logistic_bf16"][int(rng.integers(0, 4))]
    bf16 = head.endswith("bf16")
    wide = rng.random() < 0.12                      # beyond the widths the matrix-core kernels take
    d = int(rng.integers(1, 6)) * 8 if bf16 else int(rng.integers(1, 41))
    hidden = 0 if head.startswith("logistic") else int(rng.integers(3, 41))
    if wide:
        d = int(rng.integers(33, 41)) * 8
        hidden = 0 if hidden == 0 else int(rng.integers(257, 300))
    lo = float(rng.uniform(2.0, 20.0))
    frac = rng.dirichlet(np.full(A, 2.0))
    frac = tuple(float(f) for f in frac / frac.sum())
    n = int(rng.integers(1, 1500)) if rng.random() < 0.6 else int(rng.integers(1500, 6000))
    w = wl.tiny(seed=7100 + seed, n=n, classes=classes, models=models,
                max_batch=int(rng.integers(1, 25)), feat_dim=d, hidden_dim=hidden,
                feat_dtype=wl.BF16 if bf16 else wl.F32, penalty=int(rng.integers(0, 3)),
                deadline=(lo, lo * float(rng.uniform(1.5, 12.0))), fractions=frac)
    if rng.random() < 0.5:
        wl.attach_priors(w.profile, seed=7200 + seed)
    if rng.random() < 0.5:
        wl.attach_swap_costs(w.profile, seed=7300 + seed, lo=0.2, hi=6.0, skip_every=int(rng.integers(0, 4)))
    names = ["sneakpeek", "alg1", "lo_priority", "lo_edf", "maxacc_edf", "capped", "unit", "split", "split_alg1"]
    name = names[int(rng.integers(0, len(names)))]
    if name == "capped":
        policy = wl.Policy(batch_cap=int(rng.integers(1, 9)))
    elif name == "unit":
        policy = wl.Policy(weight=wl.WEIGHT_UNIT, order=wl.ORDER_EDF if rng.random() < 0.5 else wl.ORDER_PRIORITY)
    elif name.startswith("split"):
        policy = copy.copy(wl.named_policy("alg1" if name == "split_alg1" else "sneakpeek"))
        policy.split_groups = 1
    else:
        policy = wl.named_policy(name)
    return w, policy, bf16, name


@pytest.mark.parametrize("seed", range(64))
def test_random_shapes_policies_and_profile_extras(gpu, seed):
    """Random small workloads (ragged class / variant counts, every head kind and penalty, priors, swap-in
    costs, every policy) through the whole path, against the oracle."""
    w, policy, bf16, name = random_case(seed)
    p = w.profile
    print(f"seed {seed}: n={w.requests.n} classes={tuple(int(c) for c in p.n_classes)} models={tuple(int(m) for m in p.n_models)} "
          f"B={p.max_batch} d={p.feat_dim} H={p.hidden_dim} bf16={bf16} policy={name}", flush=True)
    full_parity(gpu, w, max_rounds=60, policy=policy, ea_tol=2e-3 if bf16 else None, want_cube=not bf16)


@pytest.mark.parametrize("d", [64, 65, 100, 128, 129, 201, 252, 256])
def test_logistic_widths_of_the_matrix_core_kernel(gpu, d):
    """Every padded feature width of the matrix-core logistic kernel (64, 128, 256), at and next to the
    boundaries, with and without rows that are multiples of 16 bytes; several class tiles, a ragged last
    class tile, several request tiles with a ragged tail."""
    w = wl.tiny(seed=7400 + d, n=1100, classes=(70, 33, 5, 129), models=(3, 16, 1, 7), max_batch=9, feat_dim=d,
                deadline=(5.0, 80.0), fractions=(0.45, 0.25, 0.05, 0.25))
    wl.attach_priors(w.profile, seed=7500 + d, kinds=(None, "weak"))
    full_parity(gpu, w, max_rounds=20, want_cube=True)


@pytest.mark.parametrize("d,H", [(8, 3), (72, 33), (136, 128), (192, 64), (264, 200), (448, 96), (512, 256), (40, 255)])
def test_bf16_mlp_widths_of_the_matrix_core_kernel(gpu, d, H):
    """Input widths across the 64-channel slices of layer 1 (a ragged last slice included; slice counts of
    every remainder modulo three, the depth of the kernel's feature ring) and hidden widths up to the
    kernel's 256."""
    w = wl.tiny(seed=7600 + d, n=900, classes=(70, 33, 5), models=(3, 16, 1), max_batch=9, feat_dim=d, hidden_dim=H,
                feat_dtype=wl.BF16, deadline=(5.0, 80.0), fractions=(0.5, 0.3, 0.2))
    full_parity(gpu, w, max_rounds=20, ea_tol=2e-3)


def test_matrix_core_rate_diagnostic(gpu):
    torch, binding = gpu
    tf_c, ghz_c = binding.sp_debug_mfma_rate(False, iters=2048)
    tf_r, ghz_r = binding.sp_debug_mfma_rate(True, iters=2048)
    # one instruction per 32 cycles and SIMD is the most the hardware does (2048 wavefronts on 1024 SIMDs);
    # how the workgroups spread over the CUs and what clock the device picks are not this library's to fix
    for tf, ghz in ((tf_c, ghz_c), (tf_r, ghz_r)):
        assert 100.0 < tf < 2600.0 and 0.5 < ghz < 3.0
        ceiling = 1024 * 32768 / 32 * ghz * 1e9 / 1e12
        assert 0.3 * ceiling < tf < 1.15 * ceiling
    with pytest.raises(binding.SneakPeekError) as e:
        binding.sp_debug_mfma_rate(True, iters=0)
    assert e.value.status == binding.SP_EINVAL
    with pytest.raises(binding.SneakPeekError) as e:
        binding.sp_debug_mfma_rate(True, iters=64, idle=3)
    assert e.value.status == binding.SP_EINVAL
    # with idle gaps (one wavefront per SIMD) the matrix cores cannot be busier than without
    for idle in (1, 8):
        tf, ghz = binding.sp_debug_mfma_rate(True, iters=2048, idle=idle)
        ceiling = 1024 * 32768 / 32 * ghz * 1e9 / 1e12
        assert 0.05 * ceiling < tf < 1.15 * ceiling
        if idle == 8:
            assert tf < 0.6 * ceiling            # 256 busy cycles, then some 512 idle ones


def test_copy_rate_diagnostic_and_stage_timing(gpu):
    torch, binding = gpu
    gbs = binding.sp_debug_copy_rate(1 << 26)
    assert 100.0 < gbs < 16000.0                 # read + written; the data sheet says 8,000 GB/s
    lib = binding.load_library()
    import ctypes as C
    out = C.c_double(0.0)
    assert lib.sp_debug_copy_rate(0, 8, None, C.byref(out)) == binding.SP_EINVAL
    assert lib.sp_debug_copy_rate(0, 1 << 20, None, None) == binding.SP_EINVAL
    # the timing record: stage times are consistent, the evaluation count is the triangle's
    w = wl.tiny(seed=7700, n=600, classes=(4, 3), models=(2, 3), max_batch=7, deadline=(50.0, 90.0))
    ctx = binding.Context(w.profile, 600)
    ctx.sp_set_timing(1)
    x, app, D, wt = binding.to_device(w.requests)
    model = torch.zeros(600, dtype=torch.int32, device="cuda:0")
    for one_launch in (True, False):
        ctx.sp_score(x, app, D, wt)
        if one_launch:
            rc, summ, _ = ctx.sp_schedule(3, model_out=model)
        else:
            for _ in range(3):
                ctx.sp_greedy_round()
            rc, summ, _ = ctx.sp_schedule(0 if False else 1, model_out=model)    # brings the state to the host
        tm = ctx.sp_get_timing()
        assert 0.0 < tm["finish_order_ms"] <= tm["order_ms"] and tm["copy_outputs_ms"] > 0.0
        # loose deadlines: every round sees full windows of 7 requests in both applications
        rounds = summ["n_rounds"]
        assert tm["utility_evaluations"] == rounds * (2 + 3) * 7 * 8 // 2
    # level 3: the two events around the scoring kernel only; the other fields stay 0
    ctx.sp_set_timing(3)
    ctx.sp_score(x, app, D, wt)
    ctx.sp_schedule(3, model_out=model)
    tm = ctx.sp_get_timing()
    assert tm["score_kernel_ms"] > 0.0
    assert tm["group_ms"] == 0.0 and tm["order_ms"] == 0.0 and tm["rounds_ms"] == 0.0 and tm["copy_outputs_ms"] == 0.0
    ctx.close()


def test_a_caller_stream_is_honoured(gpu):
    """Everything a window launches goes to the stream the caller names: the same window on a stream of the
    caller's own (default priority), behind other work queued on that stream, gives bit-identical results."""
    torch, binding = gpu
    w = wl.tiny(seed=7700, n=3000, classes=(40, 7, 90), models=(5, 16, 3), max_batch=12, feat_dim=48, deadline=(4.0, 90.0))
    ref = run_window(gpu, w, 0, want_cube=True)
    side = torch.cuda.Stream()
    noise = torch.randn(2048, 2048, device="cuda:0")
    with torch.cuda.stream(side):
        for _ in range(3):
            noise = noise @ noise * 1e-3               # unrelated work ahead of the window on the same stream
        got = run_window(gpu, w, 0, want_cube=True)
    side.synchronize()
    torch.cuda.synchronize()
    assert got["log"] == ref["log"] and got["summary"] == ref["summary"]
    for k in ("ea", "key", "order", "seg", "cube", "model", "round_of", "order_of", "util"):
        assert np.array_equal(got[k], ref[k], equal_nan=True), k
    ref["close"]()
    got["close"]()


def test_two_contexts_interleaved_are_independent(gpu):
    """Separate contexts share nothing: windows of two contexts scheduled in alternating chunks end exactly
    as when each runs alone."""
    torch, binding = gpu
    wa = wl.tiny(seed=7800, n=2500, classes=(30, 8), models=(4, 9), max_batch=10, feat_dim=40, deadline=(4.0, 120.0))
    wb = wl.tiny(seed=7801, n=1800, classes=(5, 60, 12), models=(16, 2, 7), max_batch=6, feat_dim=24, hidden_dim=12,
                 feat_dtype=wl.BF16, deadline=(3.0, 80.0))
    alone = [run_window(gpu, w, 0) for w in (wa, wb)]
    ctxs = [binding.Context(w.profile, w.requests.n) for w in (wa, wb)]
    devs = [binding.to_device(w.requests) for w in (wa, wb)]
    outs = []
    for ctx, (x, app, D, wt), w in zip(ctxs, devs, (wa, wb)):
        ctx.sp_score(x, app, D, wt)
        n = w.requests.n
        outs.append([torch.full((n,), 99, dtype=torch.int32, device="cuda:0") for _ in range(3)] +
                    [torch.full((n,), -7.0, device="cuda:0")])
    done = [False, False]
    logs = [[], []]
    summ = [None, None]
    while not all(done):
        for i, ctx in enumerate(ctxs):
            if done[i]:
                continue
            rc, sm, _ = ctx.sp_schedule(3, *outs[i], log_capacity=0)
            summ[i] = sm
            done[i] = rc == binding.SP_DONE
    for i in range(2):
        assert summ[i] == alone[i]["summary"]
        for t, k in zip(outs[i], ("model", "round_of", "order_of", "util")):
            assert np.array_equal(t.cpu().numpy(), alone[i][k]), (i, k)
        ctxs[i].close()
        alone[i]["close"]()


@pytest.mark.parametrize("name", ["sneakpeek", "alg1"])
def test_many_rounds_across_several_launches(gpu, name):
    """Several hundred rounds in one sp_schedule call: the one-launch kernel is launched again every 64
    rounds and has to pick up clock, resident variant (swap-in costs), head pointers and generation
    numbers where the previous launch left them."""
    w = wl.tiny(seed=7900, n=700, classes=(6, 20, 3), models=(3, 5, 2), max_batch=3, feat_dim=16, penalty=wl.PEN_LINEAR,
                deadline=(200.0, 2500.0), alpha=(1.0, 4.0), beta=(0.2, 1.0), fractions=(0.5, 0.3, 0.2))
    wl.attach_swap_costs(w.profile, seed=7901, lo=0.5, hi=5.0)
    got, stats = full_parity(gpu, w, max_rounds=0, policy=wl.named_policy(name), want_cube=True)
    assert stats["rounds"] > 150 and got["summary"]["done"] == 1
    assert got["summary"]["n_scheduled"] + got["summary"]["n_dropped"] == 700 and got["summary"]["total_violation_ms"] > 0


def test_round_generations_start_over_cleanly(gpu):
    """The exchange words of the one-launch rounds kernel carry generation numbers that start over after
    2^23 - 1 rounds in the life of a context: a window placed across that point is scheduled exactly as
    one that is not."""
    torch, binding = gpu
    w = wl.tiny(seed=7900, n=700, classes=(6, 20, 3), models=(3, 5, 2), max_batch=3, feat_dim=16, penalty=wl.PEN_LINEAR,
                deadline=(200.0, 2500.0), alpha=(1.0, 4.0), beta=(0.2, 1.0), fractions=(0.5, 0.3, 0.2))
    ref = run_window(gpu, w, 0)
    assert ref["summary"]["n_rounds"] > 150
    ctx = binding.Context(w.profile, 700)
    if not ctx.rounds_in_one_launch:
        pytest.skip("this device does not hold the one-launch rounds kernel")
    ctx.sp_debug_set_generation((1 << 23) - 1 - 100)         # the second launch of the window reaches the limit
    got = run_window(gpu, w, 0, ctx=ctx)
    assert got["log"] == ref["log"] and got["summary"] == ref["summary"]
    for k in ("model", "round_of", "order_of", "util"):
        assert np.array_equal(got[k], ref[k]), k
    got2 = run_window(gpu, w, 0, ctx=ctx)                     # and the context goes on normally afterwards
    assert got2["log"] == ref["log"] and got2["summary"] == ref["summary"]
    with pytest.raises(binding.SneakPeekError):
        ctx.sp_debug_set_generation(1 << 23)
    ctx.close()
    ref["close"]()


def test_a_wait_that_runs_out_fails_the_call_and_the_context_carries_on_with_two_kernels(gpu):
    """The bounded waits of the one-launch rounds kernel, forced to run out from the host (a poll limit of
    one; every kernel still ends normally): sp_schedule reports SP_EDEVICE, the window has to be scored
    again, and from then on the context schedules with two kernels per round, with the same decisions."""
    torch, binding = gpu
    w = wl.tiny(seed=7950, n=2000, classes=(9, 30), models=(4, 7), max_batch=8, feat_dim=20, deadline=(4.0, 90.0))
    ref = run_window(gpu, w, 0)
    ctx = binding.Context(w.profile, 2000)
    if not ctx.rounds_in_one_launch:
        pytest.skip("this device does not hold the one-launch rounds kernel")
    x, app, D, wt = binding.to_device(w.requests)
    ctx.sp_debug_set_spin_limit(1)
    ctx.sp_score(x, app, D, wt)
    with pytest.raises(binding.SneakPeekError) as e:
        ctx.sp_schedule(0, log_capacity=16)
    assert e.value.status == binding.SP_EDEVICE
    assert not ctx.lib.sp_rounds_in_one_launch(ctx.h)
    with pytest.raises(binding.SneakPeekError) as e:
        ctx.sp_schedule(0, log_capacity=16)                   # the window's state is not to be trusted any more
    assert e.value.status == binding.SP_ESTATE
    ctx.sp_debug_set_spin_limit(0)
    got = run_window(gpu, w, 0, ctx=ctx)                      # scored again, two kernels per round
    assert got["log"] == ref["log"] and got["summary"] == ref["summary"]
    for k in ("model", "round_of", "order_of", "util"):
        assert np.array_equal(got[k], ref[k]), k
    ctx.close()
    ref["close"]()


def test_a_look_back_that_runs_out_fails_the_window_and_the_context_carries_on(gpu):
    """The bounded look-back of the radix passes, forced to give up from the host (every kernel still ends
    normally): the rounds report SP_EDEVICE, the window has to be scored again, and then all is as before."""
    torch, binding = gpu
    # one application with three sort tiles, one with a single tile (which never looks back)
    w = wl.tiny(seed=7955, n=12000, classes=(9, 5), models=(3, 2), max_batch=8, feat_dim=12, deadline=(4.0, 90.0),
                fractions=(0.85, 0.15))
    ref = run_window(gpu, w, 0)
    ctx = binding.Context(w.profile, 12000)
    x, app, D, wt = binding.to_device(w.requests)
    ctx.sp_debug_set_sort_spin_limit(-1)
    ctx.sp_score(x, app, D, wt)
    for call in (ctx.sp_greedy_round, lambda: ctx.sp_schedule(0, log_capacity=16)):
        with pytest.raises(binding.SneakPeekError) as e:
            call()
        assert e.value.status in (binding.SP_EDEVICE, binding.SP_ESTATE)
    assert b"look-back" in ctx.lib.sp_last_hip_error(ctx.h)
    ctx.sp_debug_set_sort_spin_limit(0)
    got = run_window(gpu, w, 0, ctx=ctx)
    assert got["log"] == ref["log"] and got["summary"] == ref["summary"]
    for k in ("model", "round_of", "order_of", "util", "order"):
        assert np.array_equal(got[k], ref[k]), k
    ctx.close()
    ref["close"]()


@pytest.mark.parametrize("path", ["one launch", "two kernels"])
def test_timing_aid_changes_nothing_and_reports_sane_times(gpu, path):
    """sp_set_timing: the same schedule with stage and per-round timing on, on both rounds paths; the
    times are positive, one per round, and add up to no more than the whole."""
    torch, binding = gpu
    if path == "one launch":
        w = wl.tiny(seed=7960, n=2500, classes=(9, 30), models=(4, 7), max_batch=8, feat_dim=20, deadline=(4.0, 90.0))
    else:
        A = 90                                               # too many (application, variant) pairs to stay resident
        w = wl.tiny(seed=7961, n=4000, classes=tuple(2 + (a % 5) for a in range(A)), models=tuple(9 + (a % 4) for a in range(A)),
                    max_batch=7, feat_dim=12, deadline=(5.0, 90.0))
    ref = run_window(gpu, w, 0)
    ctx = binding.Context(w.profile, w.requests.n)
    if (path == "one launch") != ctx.rounds_in_one_launch:
        pytest.skip("this device runs the rounds of this profile the other way")
    with pytest.raises(binding.SneakPeekError) as e:
        ctx.sp_get_timing()
    assert e.value.status == binding.SP_ESTATE
    ctx.sp_set_timing(2)
    got = run_window(gpu, w, 0, ctx=ctx)
    assert got["log"] == ref["log"] and got["summary"] == ref["summary"]
    tm = ctx.sp_get_timing()
    per_round = ctx.sp_get_round_times()
    n_rounds = ref["summary"]["n_rounds"]
    assert tm["n_rounds_timed"] == len(per_round) == n_rounds
    assert all(0.0 < t < 5.0 for t in per_round)             # milliseconds
    assert 0.0 < tm["score_kernel_ms"] < 50.0 and 0.0 < tm["group_ms"] < 50.0 and 0.0 < tm["order_ms"] < 50.0
    assert sum(per_round) <= tm["rounds_ms"] * 1.05 + 0.05
    ctx.sp_set_timing(0)
    ctx.close()
    ref["close"]()


def test_optional_outputs_short_log_and_calls_after_the_end(gpu):
    """sp_schedule with only some outputs, a log shorter than the schedule, and further calls once nothing
    is live: the same schedule, the log's first entries, SP_DONE with the same summary."""
    torch, binding = gpu
    w = wl.tiny(seed=7970, n=1500, classes=(9, 30), models=(4, 7), max_batch=8, feat_dim=20, deadline=(4.0, 90.0))
    ref = run_window(gpu, w, 0)
    assert ref["summary"]["n_rounds"] > 8
    ctx = binding.Context(w.profile, 1500)
    x, app, D, wt = binding.to_device(w.requests)
    ctx.sp_score(x, app, D, wt)                              # no EA / key outputs asked for
    util = torch.full((1500,), -7.0, device="cuda:0")
    rc, summ, log = ctx.sp_schedule(0, util_out=util, log_capacity=5)
    assert rc == binding.SP_DONE and summ == ref["summary"]
    assert log == ref["log"][:5]
    assert np.array_equal(util.cpu().numpy(), ref["util"])
    model = torch.full((1500,), 99, dtype=torch.int32, device="cuda:0")
    rc, summ2, log2 = ctx.sp_schedule(0, model_out=model, log_capacity=1500)     # nothing left to do
    assert rc == binding.SP_DONE and summ2 == ref["summary"] and log2 == ref["log"]
    assert np.array_equal(model.cpu().numpy(), ref["model"])
    rc, dec = ctx.sp_greedy_round()
    assert rc == binding.SP_DONE
    ctx.close()
    ref["close"]()
