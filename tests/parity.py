"""Comparison protocol between the HIP library's outputs and the CPU oracle.

Values (EA, keys, scores, utilities) are compared element by element with a
relative tolerance whose denominator is max(|reference|, 1e-6).

Decisions are compared by replaying the library's round log inside the oracle:
at every round the oracle decides from the *replayed* state.  The library's
decision is an exact match if (application, variant, batch size, member list)
are identical.  Otherwise it is accepted as a tolerance tie only if
  (i)   the oracle's score of the library's batch is within `tol` (relative)
        of the oracle's best score,
  (ii)  every member is live in the oracle's state, and no live non-member of
        that application has an oracle key more than `tol` (relative) above a
        member's key (the batch is a top-b prefix up to near-equal keys);
anything else is a failure.  The replay then continues from the library's
choice, so one tie does not invalidate the following rounds.
"""
from __future__ import annotations

import numpy as np

from oracle import sneakpeek_oracle as orc


def rel_err(got, ref, floor=1e-6):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    return np.abs(got - ref) / np.maximum(np.abs(ref), floor)


def assert_close(name, got, ref, tol, floor=1e-6):
    e = rel_err(got, ref, floor)
    bad = ~(e <= tol)
    if np.any(bad):
        i = int(np.argmax(np.where(np.isnan(e), np.inf, e)))
        raise AssertionError(f"{name}: {int(bad.sum())} of {e.size} beyond {tol:g}; worst at flat index {i}: "
                             f"got {np.ravel(got)[i]!r} ref {np.ravel(ref)[i]!r} rel {np.ravel(e)[i]:.3g}")
    return float(e.max()) if e.size else 0.0


def check_order(order_gpu, seg_gpu, app, key_ref, n_apps, tol):
    """The library's service order against the oracle's: same segments, same
    request sets, and any position that differs holds a key within tol of the
    oracle's key at that position (swap between near-equal keys)."""
    ref = orc.service_order(app, key_ref, n_apps)
    swaps = 0
    for a in range(n_apps):
        got = np.asarray(order_gpu[seg_gpu[a]:seg_gpu[a + 1]])
        want = ref[a]
        assert got.shape == want.shape, f"app {a}: segment length {got.shape} vs {want.shape}"
        diff = np.nonzero(got != want)[0]
        if diff.size:
            assert np.array_equal(np.sort(got), np.sort(want)), f"app {a}: different request sets"
            e = rel_err(key_ref[got[diff]], key_ref[want[diff]], floor=1e-30)
            assert np.all(e <= tol), f"app {a}: order differs beyond key tolerance (max rel {e.max():.3g})"
            swaps += int(diff.size)
    return swaps


def members_by_round(round_of, order_of, n_rounds):
    """Per round, the request ids in execution order, from the per-request outputs."""
    round_of = np.asarray(round_of)
    order_of = np.asarray(order_of)
    served = np.nonzero(round_of >= 0)[0]
    srt = served[np.argsort(order_of[served], kind="stable")]
    out = [[] for _ in range(n_rounds)]
    for i in srt:
        out[int(round_of[i])].append(int(i))
    return [np.asarray(m, dtype=np.int64) for m in out]


def replay(profile, requests, ea_ref, key_ref, log, members, done, tol, policy=None, sub=None):
    """Replay the library's rounds in the oracle.  Returns (window, stats)."""
    win = orc.Window(profile, requests, ea=ea_ref, key=key_ref, policy=policy, sub=sub)
    stats = {"rounds": len(log), "exact": 0, "ties": 0, "max_score_rel": 0.0}
    for r, rec in enumerate(log):
        a, m, b = int(rec["app"]), int(rec["model"]), int(rec["batch"])
        ids = members[r]
        assert rec["round"] == r and len(ids) == b, f"round {r}: log says batch {b}, outputs hold {len(ids)}"
        cube = win.score_cube_fast()
        d = win.decide(cube)
        assert d is not None, f"round {r}: library committed a batch but nothing is live in the oracle"
        assert abs(rec["t_start_ms"] - win.t) <= 1e-9 * max(1.0, abs(win.t)), f"round {r}: clock {rec['t_start_ms']} vs {win.t}"
        exact = (d["app"], d["model"], d["batch"]) == (a, m, b) and np.array_equal(d["ids"], ids)
        grp = int(win.gid[ids[0]])           # the group the library's batch belongs to
        kind = win.scoring_penalty(a)
        t_end = win.start_time(a, m) + win.lat[a][m, b - 1]
        mine = float((win.wsum[ids] * orc.utility(win.ea[ids, m], kind, win.D[ids], t_end)).sum())
        if exact:
            stats["exact"] += 1
        else:
            live = win.live_queue(grp)
            assert np.all(np.isin(ids, live)), f"round {r}: a chosen request is not live in the oracle"
            best_here = d["score"]
            if win.group_first and d["group"] != grp:
                # a different group went first: its priority must tie the oracle's choice within tolerance
                pa, pb = win.group_priority(grp), win.group_priority(d["group"])
                assert pa is not None and pa >= pb - tol * abs(pb), f"round {r}: group {grp} ({pa!r}) is not the top group ({pb!r})"
                best_here = float(np.max(cube[grp]))
            assert mine >= best_here * (1.0 - tol) - 1e-300, \
                f"round {r}: library chose ({a},{m},{b}) worth {mine!r}, oracle best {d['score']!r} at " \
                f"({d['app']},{d['model']},{d['batch']})"
            others = live[~np.isin(live, ids)]
            if others.size:
                lowest = float(win.omega[ids].min())
                assert win.omega[others].max() <= lowest + tol * abs(lowest), \
                    f"round {r}: batch is not a top-{b} prefix within key tolerance"
            stats["ties"] += 1
        e = float(rel_err(rec["score"], mine))
        stats["max_score_rel"] = max(stats["max_score_rel"], e)
        assert e <= tol, f"round {r}: score {rec['score']!r} vs oracle {mine!r}"
        out = win.commit(a, m, ids)
        assert abs(rec["t_end_ms"] - out["t_end"]) <= 1e-9 * max(1.0, abs(out["t_end"]))
        assert float(rel_err(rec["batch_utility"], out["batch_utility"])) <= max(tol, 2e-6), \
            f"round {r}: batch utility {rec['batch_utility']!r} vs {out['batch_utility']!r}"
    if done:
        assert win.decide() is None, "library reports an exhausted queue but the oracle still has live requests"
    return win, stats


def check_outputs(win, model, round_of, order_of, util, summary, tol):
    """Per-request outputs and totals against the replayed oracle window."""
    assert np.array_equal(np.asarray(model), win.model), "assigned variants differ"
    assert np.array_equal(np.asarray(round_of), win.round_of), "round ids differ"
    assert np.array_equal(np.asarray(order_of), win.order_of), "execution order differs"
    worst = assert_close("utility", util, win.util, tol)
    ref = win.summary()
    assert summary["n_rounds"] == ref["n_rounds"] and summary["n_scheduled"] == ref["n_scheduled"]
    assert summary["n_dropped"] == ref["n_dropped"]
    for k in ("total_weighted_utility", "mean_utility", "total_violation_ms"):
        assert float(rel_err(summary[k], ref[k])) <= tol, f"{k}: {summary[k]!r} vs {ref[k]!r}"
    return worst
