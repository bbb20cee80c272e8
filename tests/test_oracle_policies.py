"""Pins for the oracle's policy knobs: each approach of Sec. 6.1 is written out here as the plain
request-at-a-time (or group-at-a-time) loop the paper describes, independently of the oracle's round
machinery, and the oracle run with the matching knobs must take the same decisions."""
import math

import numpy as np
import pytest

from oracle import sneakpeek_oracle as orc
from paper_2505_06641_amd import workloads as wl

STEP, LINEAR, SIGMOID = wl.PEN_STEP, wl.PEN_LINEAR, wl.PEN_SIGMOID


def gamma(kind, d, e):
    """Scalar penalty of Sec. 6.1 (rational sigmoid, capped at 1), written independently of the oracle."""
    if e <= d:
        return 0.0
    if kind == STEP:
        return 1.0
    x = (e - d) / d
    if x >= 1.0:
        return 1.0
    return x if kind == LINEAR else x ** 3 / (x ** 3 + (1.0 - x) ** 3)


def scored(w):
    ea, key = orc.score_requests(w.profile, w.requests)
    return ea, key


def request_at_a_time(w, ea, key, edf, max_accuracy):
    """Sec. 6.1: an ordering policy (EDF or the priority of eq. 12) and a per-request model choice:
    locally optimal (eq. 13: the variant with the best utility at the current time) or max accuracy (the
    most accurate variant that still meets the deadline).  Requests whose penalty is already 1 on the
    fastest variant are skipped, as everywhere in this library."""
    p, rq = w.profile, w.requests
    n = rq.app.shape[0]
    D = rq.deadline_rel_ms.astype(np.float64)
    pending = set(range(n))
    t, log = 0.0, []
    while True:
        live = []
        for i in pending:
            a = int(rq.app[i])
            lmin = min(float(p.lat_ms[a][m, 0]) for m in range(int(p.n_models[a])))
            if gamma(int(p.penalty[a]), D[i], t + lmin) < 1.0:
                live.append(i)
        if not live:
            break
        i = min(live, key=(lambda j: (D[j], j)) if edf else (lambda j: (-key[j], j)))
        a = int(rq.app[i])
        best_m, best_v = 0, -1.0
        for m in range(int(p.n_models[a])):
            e = t + float(p.lat_ms[a][m, 0])
            if max_accuracy:
                v = ea[i, m] if e <= D[i] else 0.0
            else:
                v = ea[i, m] * (1.0 - gamma(int(p.penalty[a]), D[i], e))
            if v > best_v:
                best_m, best_v = m, v
        t = t + float(p.lat_ms[a][best_m, 0])
        u = ea[i, best_m] * (1.0 - gamma(int(p.penalty[a]), D[i], t))
        log.append((i, best_m, t, u))
        pending.discard(i)
    return log


@pytest.mark.parametrize("name,edf,maxacc", [("lo_priority", False, False), ("lo_edf", True, False),
                                             ("maxacc_edf", True, True)])
@pytest.mark.parametrize("seed,kind", [(0, SIGMOID), (1, STEP), (2, LINEAR)])
def test_request_level_baselines(name, edf, maxacc, seed, kind):
    w = wl.tiny(seed=400 + seed, n=30, classes=(3, 4, 2), models=(3, 2, 4), max_batch=6, penalty=kind,
                deadline=(3.0, 45.0))
    ea, key = scored(w)
    want = request_at_a_time(w, ea, key, edf, maxacc)
    win = orc.Window(w.profile, w.requests, ea=ea, key=key, policy=wl.named_policy(name))
    win.run()
    assert len(win.log) == len(want) > 5
    for rec, (i, m, t, u) in zip(win.log, want):
        assert rec["batch"] == 1 and int(rec["ids"][0]) == i and rec["model"] == m
        assert rec["t_end"] == pytest.approx(t, rel=1e-14)
        assert win.util[i] == pytest.approx(u, rel=1e-9, abs=1e-13)   # 1 - gamma cancels near gamma = 1


def test_max_accuracy_differs_from_locally_optimal_when_a_late_variant_is_still_worth_more():
    # one request, deadline 10: the accurate variant finishes at 11 (linear penalty 0.1 -> utility 0.81),
    # the weak one on time (0.5).  Locally optimal takes the accurate one, max accuracy the one on time.
    w = wl.tiny(seed=410, n=1, classes=(2,), models=(2,), max_batch=1, penalty=LINEAR, deadline=(10.0, 10.0))
    p = w.profile
    p.acc[0][0, :] = 0.9
    p.acc[0][1, :] = 0.5
    p.lat_ms[0][0, :] = 11.0
    p.lat_ms[0][1, :] = 2.0
    w.requests.deadline_rel_ms[:] = 10.0
    lo = orc.Window(p, w.requests, policy=wl.named_policy("lo_edf"))
    ma = orc.Window(p, w.requests, policy=wl.named_policy("maxacc_edf"))
    r1, r2 = lo.step(), ma.step()
    assert r1["model"] == 0 and lo.util[0] == pytest.approx(0.9 * 0.9, rel=1e-6)
    assert r2["model"] == 1 and ma.util[0] == pytest.approx(0.5, rel=1e-6)


def algorithm_1(w, ea, key):
    """Alg. 1 as printed, for queues where no group exceeds the batch cap: groups ordered by mean
    request priority (eq. 14), one variant per group by the group's average utility (eq. 13 at the
    group level), requests inside a group in priority order, one running order counter."""
    p, rq = w.profile, w.requests
    D = rq.deadline_rel_ms.astype(np.float64)
    groups = {}
    for i in range(rq.app.shape[0]):
        groups.setdefault(int(rq.app[i]), []).append(i)
    ordered = sorted(groups, key=lambda a: (-math.fsum(key[i] for i in groups[a]) / len(groups[a]), a))
    t, order, out = 0.0, 1, []
    for a in ordered:
        g = sorted(groups[a], key=lambda i: (-key[i], i))
        best_m, best_v = 0, -1.0
        for m in range(int(p.n_models[a])):
            e = t + float(p.lat_ms[a][m, len(g) - 1])
            v = math.fsum(ea[i, m] * (1.0 - gamma(int(p.penalty[a]), D[i], e)) for i in g) / len(g)
            if v > best_v:
                best_m, best_v = m, v
        t = t + float(p.lat_ms[a][best_m, len(g) - 1])
        for i in g:
            out.append((i, a, best_m, order))
            order += 1
    return out, t


@pytest.mark.parametrize("seed,kind", [(0, SIGMOID), (1, LINEAR), (2, STEP), (3, SIGMOID)])
def test_group_level_scheduling_as_printed(seed, kind):
    # deadlines long enough that nobody's penalty reaches 1 while earlier groups run (Alg. 1 has no
    # notion of dropping requests), short enough that the variants differ in utility
    w = wl.tiny(seed=420 + seed, n=22, classes=(3, 4, 2), models=(3, 2, 4), max_batch=16, penalty=kind,
                deadline=(55.0, 120.0) if kind == STEP else (30.0, 90.0), alpha=(2.0, 9.0), beta=(0.5, 3.0))
    ea, key = scored(w)
    want, t_end = algorithm_1(w, ea, key)
    win = orc.Window(w.profile, w.requests, ea=ea, key=key, policy=wl.named_policy("alg1"))
    win.run()
    assert win.summary()["n_dropped"] == 0
    assert len(win.log) == 3 and win.t == pytest.approx(t_end, rel=1e-14)
    for i, a, m, order in want:
        assert win.model[i] == m and win.order_of[i] == order and win.app[i] == a


def test_whole_window_rule_and_unit_weights_on_a_capped_queue():
    # with more requests than the cap, "the group runs whole" means the whole candidate window
    w = wl.tiny(seed=430, n=40, classes=(3, 2), models=(2, 3), max_batch=8, deadline=(30.0, 200.0))
    ea, key = scored(w)
    win = orc.Window(w.profile, w.requests, ea=ea, key=key, policy=wl.named_policy("alg1"))
    while True:
        sizes = [win.candidate_window(a).shape[0] for a in range(2)]
        prios = [win.group_priority(a) for a in range(2)]
        rec = win.step()
        if rec is None:
            break
        a = rec["app"]
        assert rec["batch"] == sizes[a]
        assert all(prios[a] >= v for v in prios if v is not None)
        q = rec["ids"]
        e = rec["t_end"]
        per_model = [math.fsum(ea[i, m] * (1.0 - gamma(int(w.profile.penalty[a]), float(win.D[i]), e_m))
                               for i in q)
                     for m, e_m in enumerate(rec["t_start"] + w.profile.lat_ms[a][:, len(q) - 1].astype(np.float64))]
        assert rec["model"] == int(np.argmax(per_model))
        assert rec["score"] == pytest.approx(per_model[rec["model"]], rel=1e-12)
    assert win.summary()["n_scheduled"] + win.summary()["n_dropped"] == 40


def test_batch_cap_and_default_policy_equivalences():
    w = wl.tiny(seed=440, n=50, classes=(3, 4), models=(2, 3), max_batch=6, deadline=(4.0, 70.0))
    ea, key = scored(w)
    ref = orc.Window(w.profile, w.requests, ea=ea, key=key); ref.run()
    same = orc.Window(w.profile, w.requests, ea=ea, key=key, policy=wl.Policy()); same.run()
    assert [(r["app"], r["model"], r["batch"]) for r in ref.log] == [(r["app"], r["model"], r["batch"]) for r in same.log]
    capped = orc.Window(w.profile, w.requests, ea=ea, key=key, policy=wl.Policy(batch_cap=2)); capped.run()
    assert max(r["batch"] for r in capped.log) == 2
    # a cap above the profile's batch limit changes nothing
    loose = orc.Window(w.profile, w.requests, ea=ea, key=key, policy=wl.Policy(batch_cap=99)); loose.run()
    assert [(r["app"], r["model"], r["batch"]) for r in ref.log] == [(r["app"], r["model"], r["batch"]) for r in loose.log]


def test_edf_order_inside_an_application_and_unit_weights():
    w = wl.tiny(seed=450, n=24, classes=(3,), models=(2,), max_batch=4, deadline=(20.0, 200.0))
    ea, key = scored(w)
    win = orc.Window(w.profile, w.requests, ea=ea, key=key, policy=wl.Policy(order=wl.ORDER_EDF, weight=wl.WEIGHT_UNIT))
    D = w.requests.deadline_rel_ms
    assert win.order[0].tolist() == sorted(range(24), key=lambda i: (D[i], i))
    cube = win.score_cube()
    q = win.candidate_window(0)
    for m in range(2):
        for b in range(1, 5):
            e = float(w.profile.lat_ms[0][m, b - 1])
            v = math.fsum(ea[i, m] * (1.0 - gamma(int(w.profile.penalty[0]), float(D[i]), e)) for i in q[:b])
            assert cube[0, m, b - 1] == pytest.approx(v, rel=1e-12)
    assert np.allclose(cube, win.score_cube_fast(), rtol=1e-13, equal_nan=True)
