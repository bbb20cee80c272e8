"""Pins for data-aware group splitting (Sec. 5.3.2): the labelling rule on the paper's examples, and the
equivalence "a split group behaves exactly like an application of its own"."""
import copy

import numpy as np
import pytest

from oracle import sneakpeek_oracle as orc
from paper_2505_06641_amd import workloads as wl


def test_labelling_rule_on_the_papers_examples():
    # Fig. "group splitting": two binary tasks.  Same predicted class -> one subgroup; different
    # predicted classes -> two subgroups; inconclusive multi-class probabilities -> not split.
    same = orc.split_labels([[0.9, 0.1], [0.8, 0.2]])
    assert same.tolist() == [1, 1]
    diff = orc.split_labels([[0.9, 0.1], [0.3, 0.7]])
    assert diff.tolist() == [1, 2]
    flat = orc.split_labels([[0.4, 0.3, 0.3], [0.5, 0.5], [0.5000001, 0.4999999]])
    assert flat.tolist() == [0, 0, 1]           # "theta_i > 0.5": exactly one half does not qualify


def relabelled_as_applications(w, sub):
    """The same requests with every non-empty (application, subgroup) pair registered as an application
    of its own (same head, tables and penalty as its parent), in ascending (application, subgroup) order."""
    p, rq = w.profile, w.requests
    pairs = sorted(set(zip(rq.app.tolist(), sub.tolist())))
    index = {pr: i for i, pr in enumerate(pairs)}
    q = copy.copy(p)
    q.n_apps = len(pairs)
    for name in ("n_classes", "n_models", "penalty"):
        setattr(q, name, np.array([getattr(p, name)[a] for a, _ in pairs], dtype=np.int32))
    for name in ("W1", "b1", "W2", "b2", "acc", "theta_test", "lat_ms"):
        setattr(q, name, [getattr(p, name)[a] for a, _ in pairs])
    r2 = copy.copy(rq)
    r2.app = np.array([index[(int(a), int(s))] for a, s in zip(rq.app, sub)], dtype=np.int32)
    return q, r2, [a for a, _ in pairs]


@pytest.mark.parametrize("seed,policy", [(0, "sneakpeek"), (1, "alg1"), (2, "sneakpeek"), (3, "lo_priority")])
def test_a_split_group_behaves_like_an_application_of_its_own(seed, policy):
    w = wl.tiny(seed=500 + seed, n=60, classes=(2, 3, 2), models=(2, 3, 2), max_batch=5, deadline=(5.0, 80.0),
                feat_dim=6)
    for a in range(3):
        w.profile.W1[a] *= 3.0                  # fairly confident heads: many requests get a subgroup
    ea, key, thetas = orc.score_requests(w.profile, w.requests, return_theta=True)
    sub = orc.split_labels(thetas)
    assert len(set(zip(w.requests.app.tolist(), sub.tolist()))) > 3 and (sub > 0).any()
    pol = wl.named_policy(policy)
    pol.split_groups = 1
    split = orc.Window(w.profile, w.requests, ea=ea, key=key, policy=pol, sub=sub)
    split.run()
    q, r2, parent = relabelled_as_applications(w, sub)
    pol2 = wl.named_policy(policy)
    flat = orc.Window(q, r2, ea=ea, key=key, policy=pol2)
    flat.run()
    assert len(split.log) == len(flat.log) > 3
    for x, y in zip(split.log, flat.log):
        assert x["app"] == parent[y["app"]] and x["model"] == y["model"] and x["batch"] == y["batch"]
        assert np.array_equal(x["ids"], y["ids"]) and x["t_end"] == y["t_end"]
    assert np.array_equal(split.model, flat.model) and np.array_equal(split.util, flat.util)
    # a batch never mixes subgroups
    for x in split.log:
        assert len(set(sub[x["ids"]].tolist())) == 1


def test_no_confident_request_means_no_split():
    w = wl.tiny(seed=510, n=40, classes=(6, 5), models=(2, 3), max_batch=4, deadline=(5.0, 80.0))
    for a in range(2):
        w.profile.W1[a] *= 0.01                 # flat posteriors: nobody above one half
    ea, key, thetas = orc.score_requests(w.profile, w.requests, return_theta=True)
    sub = orc.split_labels(thetas)
    assert not sub.any()
    pol = wl.Policy(split_groups=1)
    a_ = orc.Window(w.profile, w.requests, ea=ea, key=key, policy=pol, sub=sub); a_.run()
    b_ = orc.Window(w.profile, w.requests, ea=ea, key=key); b_.run()
    assert [(r["app"], r["model"], r["batch"], r["t_end"]) for r in a_.log] == \
           [(r["app"], r["model"], r["batch"], r["t_end"]) for r in b_.log]
