"""Pins for the oracle's greedy rounds: brute force on tiny inputs, the
paper's counting formula, degenerate instances and conservation laws."""
import itertools
import math

import numpy as np
import pytest

from oracle import sneakpeek_oracle as orc
from paper_2505_06641_amd import workloads as wl

STEP, LINEAR, SIGMOID = wl.PEN_STEP, wl.PEN_LINEAR, wl.PEN_SIGMOID


def gamma(kind, d, e):
    """Scalar penalty written from Sec. 6.1 independently of the oracle
    (rational form of the sigmoid, cap at 1)."""
    if e <= d:
        return 0.0
    if kind == STEP:
        return 1.0
    x = (e - d) / d
    if x >= 1.0:
        return 1.0
    if kind == LINEAR:
        return x
    return x ** 3 / (x ** 3 + (1.0 - x) ** 3)


def live_ids(win, a):
    p = win.p
    lmin = min(float(p.lat_ms[a][m, 0]) for m in range(int(p.n_models[a])))
    out = []
    for i in range(win.n):
        if win.app[i] == a and win.alive[i] and gamma(int(p.penalty[a]), win.D[i], win.t + lmin) < 1.0:
            out.append(i)
    return out


def direct_value(win, a, m, S):
    e = win.t + float(win.p.lat_ms[a][m, len(S) - 1])
    return math.fsum(win.key[i] * win.ea[i, m] * (1.0 - gamma(int(win.p.penalty[a]), win.D[i], e)) for i in S)


# ---- BF1: one round against subset enumeration -------------------------------
@pytest.mark.parametrize("seed,kind", [(s, k) for s in range(6) for k in (STEP, LINEAR, SIGMOID)])
def test_round_against_subset_enumeration(seed, kind):
    w = wl.tiny(seed=100 + seed, n=8, classes=(3, 2), models=(3, 2), max_batch=4, penalty=kind,
                deadline=(3.0, 25.0))
    win = orc.Window(w.profile, w.requests)
    for _ in range(3):                      # check at t = 0 and after one and two commits
        cube = win.score_cube()
        assert np.allclose(cube, win.score_cube_fast(), rtol=1e-13, atol=0, equal_nan=True)
        best_prefix = None
        for a in range(2):
            live = live_ids(win, a)
            ranked = sorted(live, key=lambda i: (-win.key[i], i))
            assert win.live_queue(a).tolist() == ranked
            B = int(w.profile.max_batch)
            for m in range(int(w.profile.n_models[a])):
                for b in range(1, B + 1):
                    for S in itertools.combinations(ranked, b):
                        v = direct_value(win, a, m, S)
                        if list(S) == ranked[:b]:       # the priority prefix of size b
                            assert cube[a, m, b - 1] == pytest.approx(v, rel=1e-12, abs=1e-300)
                            if best_prefix is None or v > best_prefix[0]:
                                best_prefix = (v, a, m, b)
                for b in range(len(ranked) + 1, B + 1):
                    assert cube[a, m, b - 1] == -np.inf
            for m in range(int(w.profile.n_models[a]), cube.shape[1]):
                assert np.all(cube[a, m] == -np.inf)
        d = win.decide(cube)
        if best_prefix is None:
            assert d is None
            break
        assert (d["app"], d["model"], d["batch"]) == best_prefix[1:]
        assert d["score"] == pytest.approx(best_prefix[0], rel=1e-12)
        win.commit(d["app"], d["model"], d["ids"])


# ---- BF2: whole schedule against every sequence of batches -------------------
def best_sequence(win_template, remaining, t, memo):
    """max over all sequences of batches of sum w*u, by exhaustive recursion."""
    p = win_template.p
    key = (remaining, round(t, 9))
    if key in memo:
        return memo[key]
    best = 0.0
    rem = list(remaining)
    for a in range(int(p.n_apps)):
        mine = [i for i in rem if win_template.app[i] == a]
        for b in range(1, min(len(mine), int(p.max_batch)) + 1):
            for S in itertools.combinations(mine, b):
                for m in range(int(p.n_models[a])):
                    e = t + float(p.lat_ms[a][m, b - 1])
                    gain = math.fsum(win_template.w[i] * win_template.ea[i, m] *
                                     (1.0 - gamma(int(p.penalty[a]), win_template.D[i], e)) for i in S)
                    rest = best_sequence(win_template, tuple(i for i in rem if i not in S), e, memo)
                    best = max(best, gain + rest)
    memo[key] = best
    return best


@pytest.mark.parametrize("seed,kind", [(0, SIGMOID), (1, STEP), (2, LINEAR), (3, SIGMOID)])
def test_greedy_never_beats_exhaustive_optimum(seed, kind):
    w = wl.tiny(seed=200 + seed, n=5, classes=(3, 2), models=(2, 2), max_batch=3, penalty=kind,
                deadline=(4.0, 20.0), fractions=(0.6, 0.4))
    win = orc.Window(w.profile, w.requests)
    opt = best_sequence(win, tuple(range(win.n)), 0.0, {})
    got = orc.Window(w.profile, w.requests).run()
    assert got["total_weighted_utility"] <= opt * (1 + 1e-12) + 1e-15
    assert got["total_weighted_utility"] > 0


def test_single_batch_is_optimal_when_nothing_can_be_late():
    w = wl.tiny(seed=300, n=5, classes=(4,), models=(1,), max_batch=8, deadline=(1e3, 2e3))
    win = orc.Window(w.profile, w.requests)
    opt = best_sequence(win, tuple(range(win.n)), 0.0, {})
    res = win.run()
    assert res["n_rounds"] == 1 and res["n_scheduled"] == 5 and res["n_dropped"] == 0
    assert res["total_weighted_utility"] == pytest.approx(opt, rel=1e-13)
    assert res["total_weighted_utility"] == pytest.approx(float((win.w * win.ea[:, 0]).sum()), rel=1e-13)
    assert res["total_violation_ms"] == 0.0


# ---- BF3: the paper's un-batched problem (B = 1, eq. (1) clock) ---------------
@pytest.mark.parametrize("n,M,seed", [(3, 2, 0), (4, 2, 1), (3, 3, 2)])
def test_unbatched_problem_enumeration_count_and_bound(n, M, seed):
    w = wl.tiny(seed=400 + seed, n=n, classes=(3,), models=(M,), max_batch=1, deadline=(4.0, 18.0))
    w.requests.weight[:] = 1.0
    win = orc.Window(w.profile, w.requests)
    kind = int(w.profile.penalty[0])
    visited, best = 0, -1.0
    for perm in itertools.permutations(range(n)):
        for models in itertools.product(range(M), repeat=n):
            visited += 1
            t, total = 0.0, 0.0
            for pos, i in enumerate(perm):
                m = models[i]
                e = t + float(w.profile.lat_ms[0][m, 0])          # eq. (1): everything ordered ahead
                total += win.ea[i, m] * (1.0 - gamma(kind, win.D[i], e))
                t = e
            best = max(best, total / n)
    assert visited == math.factorial(n) * M ** n               # Sec. 3.1: n! |M|^n candidate solutions
    res = win.run()
    assert res["mean_utility"] <= best * (1 + 1e-12)
    assert all(r["batch"] == 1 for r in win.log)


def test_batch_of_one_round_is_locally_optimal_selection_on_top_priority_request():
    w = wl.tiny(seed=500, n=12, classes=(3, 4, 2), models=(3, 2, 2), max_batch=1, deadline=(3.0, 30.0))
    win = orc.Window(w.profile, w.requests)
    while True:
        heads = {}
        for a in range(3):
            live = sorted(live_ids(win, a), key=lambda i: (-win.key[i], i))
            if live:
                i = live[0]
                us = [win.key[i] * win.ea[i, m] *
                      (1.0 - gamma(int(w.profile.penalty[a]), win.D[i], win.t + float(w.profile.lat_ms[a][m, 0])))
                      for m in range(int(w.profile.n_models[a]))]
                heads[a] = (max(us), int(np.argmax(us)), i)
        d = win.decide()
        if not heads:
            assert d is None
            break
        a_best = max(heads, key=lambda a: (heads[a][0], -a))
        assert (d["app"], d["model"], d["ids"].tolist()) == (a_best, heads[a_best][1], [heads[a_best][2]])
        win.commit(d["app"], d["model"], d["ids"])


def test_loose_deadlines_pick_the_most_accurate_variant():
    w = wl.tiny(seed=600, n=6, classes=(5,), models=(4,), max_batch=1, deadline=(1e3, 2e3))
    win = orc.Window(w.profile, w.requests)
    d = win.decide()
    top = int(d["ids"][0])
    assert top == int(np.argmax(win.key))
    assert d["model"] == int(np.argmax(win.ea[top]))


# ---- degenerate instances -----------------------------------------------------
def test_hardness_instance_counts_on_time_requests():
    # appendix: one variant per application, accuracy 1, step penalty
    w = wl.tiny(seed=700, n=30, classes=(3, 2), models=(1, 1), max_batch=3, penalty=STEP, deadline=(2.0, 14.0))
    for a in range(2):
        w.profile.acc[a][:] = 1.0
    w.requests.weight[:] = 1.0
    win = orc.Window(w.profile, w.requests)
    res = win.run()
    done = win.model >= 0
    on_time = int(np.sum(win.finish[done] <= win.D[done]))
    assert res["total_weighted_utility"] == pytest.approx(on_time, abs=1e-12)
    assert res["n_dropped"] > 0 and on_time > 0
    assert np.all((win.util == 0.0) | (np.abs(win.util - 1.0) < 1e-14))


def test_short_circuit_variant_wins_exactly_when_real_variants_miss():
    # Sec. 5.3.1: the SneakPeek model as a variant with zero latency and its profiled accuracy
    w = wl.tiny(seed=800, n=4, classes=(3,), models=(2,), max_batch=2, penalty=STEP, deadline=(10.0, 10.0))
    w.requests.deadline_rel_ms[:] = 10.0
    w.profile.acc[0][0, :] = 0.9          # the real variant
    w.profile.acc[0][1, :] = 0.4          # short circuit: constant (profiled) accuracy
    w.profile.lat_ms[0][1, :] = 0.0
    w.profile.lat_ms[0][0, :] = [50.0, 60.0]
    d = orc.Window(w.profile, w.requests).decide()
    assert d["model"] == 1 and d["batch"] == 2 and d["t_end"] == 0.0
    w.profile.lat_ms[0][0, :] = [5.0, 6.0]
    d = orc.Window(w.profile, w.requests).decide()
    assert d["model"] == 0 and d["batch"] == 2


def test_exact_ties_go_to_smallest_app_model_batch():
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
    win = orc.Window(p, r)
    cube = win.score_cube()
    assert cube[0, 0, 1] == cube[0, 1, 1] == cube[1, 0, 1] == cube[1, 1, 1]
    d = win.decide(cube)
    assert (d["app"], d["model"], d["batch"]) == (0, 0, 2)


def test_empty_queue_and_all_dead_queue():
    w = wl.tiny(seed=1000, n=0, classes=(3,), models=(2,))
    win = orc.Window(w.profile, w.requests)
    assert win.decide() is None
    assert win.run() == {"total_weighted_utility": 0.0, "mean_utility": 0.0, "total_violation_ms": 0.0,
                         "n_rounds": 0, "n_scheduled": 0, "n_dropped": 0}
    w = wl.tiny(seed=1001, n=5, classes=(3,), models=(2,), penalty=STEP, deadline=(0.01, 0.02))
    win = orc.Window(w.profile, w.requests)
    assert win.decide() is None
    assert win.run()["n_dropped"] == 5


# ---- conservation over a longer run ------------------------------------------
@pytest.mark.parametrize("kind", [STEP, LINEAR, SIGMOID])
def test_schedule_conservation_laws(kind):
    w = wl.tiny(seed=1100 + kind, n=300, classes=(4, 3, 2), models=(3, 2, 4), max_batch=8, penalty=kind,
                deadline=(5.0, 60.0), fractions=(0.5, 0.3, 0.2))
    win = orc.Window(w.profile, w.requests)
    res = win.run()
    assert res["n_scheduled"] + res["n_dropped"] == 300
    seen = np.concatenate([r["ids"] for r in win.log])
    assert len(np.unique(seen)) == len(seen) == res["n_scheduled"]
    assert sorted(win.order_of[win.model >= 0].tolist()) == list(range(1, res["n_scheduled"] + 1))
    assert np.all(win.order_of[win.model < 0] == 0) and np.all(win.util[win.model < 0] == 0)
    clock = 0.0
    for k, r in enumerate(win.log):
        assert 1 <= r["batch"] <= 8 and r["round"] == k
        assert r["t_start"] == clock
        clock = clock + float(w.profile.lat_ms[r["app"]][r["model"], r["batch"] - 1])
        assert r["t_end"] == clock
        ids = r["ids"]
        assert np.all(np.diff(win.order_of[ids]) == 1)
        assert np.all(np.diff(win.key[ids]) <= 0)           # served in priority order
    assert win.t == clock
    # whoever was left behind can no longer earn anything
    for a in range(3):
        assert live_ids(win, a) == []
    assert np.all(win.util >= 0) and np.all(win.util <= win.ea.max(axis=1) + 1e-15)
    viol = sum(max(0.0, win.finish[i] - win.D[i]) for i in range(300) if win.model[i] >= 0)
    assert res["total_violation_ms"] == pytest.approx(viol, rel=1e-12)
    assert res["mean_utility"] == pytest.approx(win.util.sum() / 300, rel=1e-14)


def test_max_rounds_stops_early_and_resumes():
    w = wl.tiny(seed=1200, n=60, classes=(3, 2), models=(2, 2), max_batch=4, deadline=(20.0, 200.0))
    full = orc.Window(w.profile, w.requests)
    full.run()
    part = orc.Window(w.profile, w.requests)
    part.run(max_rounds=3)
    assert part.round == 3
    part.run()
    assert [(r["app"], r["model"], r["batch"]) for r in part.log] == \
           [(r["app"], r["model"], r["batch"]) for r in full.log]


# ---- swap-in cost of a variant (Sec. 3.1 "context switch time", Sec. 5.2 model locality) -----------
def test_swap_cost_is_paid_once_per_run_of_batches_on_the_same_variant():
    # one application, one variant, deadlines that nothing can miss: the greedy serves the queue in
    # full batches back to back, so the clock ends at swap + sum of batch latencies
    w = wl.tiny(seed=300, n=10, classes=(3,), models=(1,), max_batch=4, deadline=(1e3, 2e3))
    w.profile.swap_ms = [np.array([7.5], dtype=np.float32)]
    win = orc.Window(w.profile, w.requests)
    win.run()
    L = w.profile.lat_ms[0][0].astype(np.float64)
    assert [r["batch"] for r in win.log] == [4, 4, 2]
    assert win.t == pytest.approx(7.5 + L[3] + L[3] + L[1], rel=1e-15)
    assert win.log[0]["t_end"] == pytest.approx(7.5 + L[3], rel=1e-15)
    assert win.log[1]["t_end"] - win.log[1]["t_start"] == pytest.approx(L[3], rel=1e-12)


@pytest.mark.parametrize("seed,kind", [(s, k) for s in range(4) for k in (STEP, LINEAR, SIGMOID)])
def test_round_with_swap_costs_against_direct_enumeration(seed, kind):
    w = wl.tiny(seed=310 + seed, n=9, classes=(3, 2), models=(3, 2), max_batch=3, penalty=kind, deadline=(4.0, 30.0))
    wl.attach_swap_costs(w.profile, seed=320 + seed, lo=0.5, hi=6.0)
    win = orc.Window(w.profile, w.requests)
    resident = None
    for _ in range(4):
        best = None
        for a in range(2):
            ranked = sorted(live_ids(win, a), key=lambda i: (-win.key[i], i))
            for m in range(int(w.profile.n_models[a])):
                start = win.t + (0.0 if resident == (a, m) else float(w.profile.swap_ms[a][m]))
                for b in range(1, min(3, len(ranked)) + 1):
                    e = start + float(w.profile.lat_ms[a][m, b - 1])
                    v = math.fsum(win.key[i] * win.ea[i, m] * (1.0 - gamma(kind, win.D[i], e)) for i in ranked[:b])
                    if best is None or v > best[0]:
                        best = (v, a, m, b, e)
        d = win.decide()
        if best is None:
            assert d is None
            break
        assert (d["app"], d["model"], d["batch"]) == best[1:4]
        assert d["score"] == pytest.approx(best[0], rel=1e-12)
        assert d["t_end"] == pytest.approx(best[4], rel=1e-15)
        win.commit(d["app"], d["model"], d["ids"])
        resident = (d["app"], d["model"])
        assert win.t == pytest.approx(best[4], rel=1e-15)


def test_zero_or_missing_swap_costs_change_nothing():
    w = wl.tiny(seed=330, n=40, classes=(3, 4), models=(2, 3), max_batch=5, deadline=(4.0, 60.0))
    ref = orc.Window(w.profile, w.requests); ref.run()
    w.profile.swap_ms = [np.zeros(2, dtype=np.float32), None]
    got = orc.Window(w.profile, w.requests); got.run()
    assert [(r["app"], r["model"], r["batch"], r["t_end"]) for r in got.log] == \
           [(r["app"], r["model"], r["batch"], r["t_end"]) for r in ref.log]


def test_swap_cost_makes_the_greedy_stay_on_the_resident_variant():
    # two equally accurate variants, the second a shade faster but costly to bring in; every request is
    # already late when it completes (linear penalty), so faster is strictly better: without swap cost
    # the greedy takes the faster variant, with it the cheap-to-load one, and then stays on it
    w = wl.tiny(seed=340, n=8, classes=(2,), models=(2,), max_batch=2, penalty=LINEAR, deadline=(20.0, 21.0))
    p = w.profile
    p.acc[0][:] = 0.9
    p.lat_ms[0][0] = np.array([23.0, 24.0], dtype=np.float32)
    p.lat_ms[0][1] = np.array([22.0, 23.0], dtype=np.float32)
    plain = orc.Window(p, w.requests)
    assert plain.step()["model"] == 1
    p.swap_ms = [np.array([0.5, 6.0], dtype=np.float32)]
    sw = orc.Window(p, w.requests)
    first = sw.step()
    assert first["model"] == 0 and first["t_end"] == pytest.approx(0.5 + float(p.lat_ms[0][0][first["batch"] - 1]))
    second = sw.step()
    if second is not None:
        assert second["model"] == 0
        assert second["t_end"] - second["t_start"] == pytest.approx(float(p.lat_ms[0][0][second["batch"] - 1]), rel=1e-12)
