"""The seeded generator: shapes, determinism, value ranges of the five configs
(the two largest are checked at a reduced queue length here; their full size
is only drawn by the GPU tests and the benchmark)."""
import numpy as np
import pytest

from paper_2505_06641_amd import workloads as wl


@pytest.mark.parametrize("name,n", [("cfg1", None), ("cfg2", None), ("cfg3", None), ("cfg4", 2048), ("cfg5", 4096)])
def test_shapes_and_ranges(name, n):
    w = wl.make(name, n_requests=n)
    r = wl.RECIPES[name]
    p, q = w.profile, w.requests
    N = r.n_requests if n is None else n
    assert q.n == N and q.x.shape == (N, r.feat_dim)
    assert q.x.dtype == (np.uint16 if r.feat_dtype == wl.BF16 else np.float32)
    assert sum(w.notes["counts"]) == N
    assert np.bincount(q.app, minlength=p.n_apps).tolist() == w.notes["counts"]
    assert np.all(q.deadline_rel_ms >= np.float32(r.deadline[0])) and np.all(q.deadline_rel_ms <= np.float32(r.deadline[1]))
    assert np.all(q.weight >= 0) and np.all(q.weight <= 1)
    for a in range(p.n_apps):
        C, M = r.classes[a], r.models[a]
        assert p.acc[a].shape == (M, C) and p.acc[a].min() >= 0 and p.acc[a].max() <= 1
        assert p.lat_ms[a].shape == (M, r.max_batch)
        assert np.all(np.diff(p.lat_ms[a], axis=1) > 0) and p.lat_ms[a].min() > 0
        assert p.W1[a].shape == ((r.feat_dim, r.hidden_dim) if r.hidden_dim else (r.feat_dim, C))
        if r.hidden_dim:
            assert p.W2[a].shape == (r.hidden_dim, C)
        assert np.all(q.label[q.app == a] < C)


def test_split_counts_match_the_stated_shares():
    assert wl.split_counts(4096, (0.5, 0.3, 0.2)).tolist() == [2049, 1228, 819]
    assert wl.split_counts(16384, (0.5, 0.3, 0.2)).tolist() == [8193, 4915, 3276]
    assert wl.split_counts(65536, [1 / 8] * 8).tolist() == [8192] * 8


def test_same_seed_same_bytes_and_other_seed_differs():
    a, b, c = wl.make("cfg2"), wl.make("cfg2"), wl.make("cfg2", seed=99)
    assert np.array_equal(a.requests.x, b.requests.x) and np.array_equal(a.profile.acc[1], b.profile.acc[1])
    assert not np.array_equal(a.requests.x, c.requests.x)


def test_cfg1_fixed_latency_table():
    p = wl.make("cfg1").profile
    assert p.lat_ms[0][:, 0] == pytest.approx([2.3, 5.8, 14.0], rel=1e-6)
    assert p.lat_ms[0][:, 15] == pytest.approx([2 + 0.3 * 16, 5 + 0.8 * 16, 12 + 2.0 * 16], rel=1e-6)


def test_label_shift_moves_class_means():
    w = wl.make("cfg5", n_requests=8192)
    assert len(np.unique(w.requests.label)) > 1
    x = w.requests.x
    assert abs(float(x.mean())) < 0.05 and 0.9 < float(x.std()) < 1.1
