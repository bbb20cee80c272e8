"""Parity at the full size of the largest configuration, in the launch
configuration bench.py times: every EA and key against the oracle, the whole
service order, and the decisions of all rounds by replay."""
import numpy as np
import pytest

from oracle import sneakpeek_oracle as orc
from paper_2505_06641_amd import workloads as wl
from tests import parity
from tests.test_gpu_parity import gpu, run_window  # noqa: F401  (fixture + helper)

pytestmark = pytest.mark.gpu


def test_cfg5_full_size_scoring_order_and_rounds(gpu):
    torch, binding = gpu
    w = wl.make("cfg5")
    p, rq = w.profile, w.requests
    print("cfg5: oracle scoring of", rq.n, "requests", flush=True)
    ea_ref, key_ref = orc.score_requests(p, rq)
    print("cfg5: library", flush=True)
    got = run_window(gpu, w, max_rounds=w.rounds)
    stats = {}
    stats["ea_rel"] = parity.assert_close("EA", got["ea"], ea_ref, 1e-5)
    stats["key_rel"] = parity.assert_close("key", got["key"], key_ref, 1e-5, floor=1e-30)
    # invariants that hold at any size: convexity of EA, normalised outputs
    for a in range(p.n_apps):
        sel = rq.app == a
        acc = p.acc[a].astype(np.float64)
        assert np.all(got["ea"][sel] >= acc.min(axis=1) - 1e-6) and np.all(got["ea"][sel] <= acc.max(axis=1) + 1e-6)
    stats["order_swaps"] = parity.check_order(got["order"], got["seg"], rq.app, key_ref, p.n_apps, 1e-5)
    members = parity.members_by_round(got["round_of"], got["order_of"], len(got["log"]))
    print("cfg5: replay of", len(got["log"]), "rounds", flush=True)
    win, rstats = parity.replay(p, rq, ea_ref, key_ref, got["log"], members, got["summary"]["done"] == 1, 1e-5)
    stats.update(rstats)
    stats["util_rel"] = parity.check_outputs(win, got["model"], got["round_of"], got["order_of"], got["util"],
                                             got["summary"], 1e-5)
    got["close"]()
    print("cfg5", stats, got["summary"])
    assert stats["exact"] + stats["ties"] == got["summary"]["n_rounds"] > 0
    assert stats["ties"] <= 4
