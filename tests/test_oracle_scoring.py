"""Pins for the oracle's scoring half (posterior, expected accuracy, priority).

Each test checks the oracle against something other than itself: a closed
form, a value the paper prints, a pure-Python re-derivation with `math` and
`fractions`, or another library's conversion.
"""
import math
from fractions import Fraction

import numpy as np
import pytest

from oracle import sneakpeek_oracle as orc
from paper_2505_06641_amd import workloads as wl


def py_softmax(z):
    m = max(z)
    e = [math.exp(v - m) for v in z]
    s = math.fsum(e)
    return [v / s for v in e]


def py_head(x, W1, b1, W2, b2):
    d = len(x)
    z = [math.fsum(x[k] * W1[k][j] for k in range(d)) + b1[j] for j in range(len(b1))]
    if W2 is None:
        return z
    h = [max(0.0, v) for v in z]
    return [math.fsum(h[k] * W2[k][c] for k in range(len(h))) + b2[c] for c in range(len(b2))]


def test_hand_example_theta_and_ea():
    # logits (0, ln 3) -> theta = (1/4, 3/4); recall rows differ per variant and M != C
    z = np.array([[0.0, math.log(3.0)]])
    th = orc.posterior(z)
    assert th[0] == pytest.approx([0.25, 0.75], abs=1e-15)
    recall = np.array([[0.9, 0.5], [0.2, 0.6], [1.0, 0.0]], dtype=np.float32)
    ea = orc.expected_accuracy(th, recall)
    want = [0.25 * float(np.float32(0.9)) + 0.75 * 0.5,
            0.25 * float(np.float32(0.2)) + 0.75 * float(np.float32(0.6)), 0.25]
    assert ea.shape == (1, 3)
    assert ea[0] == pytest.approx(want, abs=1e-15)


@pytest.mark.parametrize("hidden", [0, 5])
def test_head_matches_pure_python_loops(hidden):
    rng = np.random.default_rng(7)
    n, d, C = 6, 4, 3
    x = rng.standard_normal((n, d)).astype(np.float32)
    if hidden:
        W1 = rng.standard_normal((d, hidden)).astype(np.float32)
        b1 = rng.standard_normal(hidden).astype(np.float32)
        W2 = rng.standard_normal((hidden, C)).astype(np.float32)
        b2 = rng.standard_normal(C).astype(np.float32)
    else:
        W1 = rng.standard_normal((d, C)).astype(np.float32)
        b1 = rng.standard_normal(C).astype(np.float32)
        W2 = b2 = None
    recall = rng.uniform(0, 1, size=(2, C)).astype(np.float32)
    z = orc.head_logits(x, W1, b1, W2, b2)
    th = orc.posterior(z)
    ea = orc.expected_accuracy(th, recall)
    for i in range(n):
        zi = py_head(x[i].tolist(), W1.tolist(), b1.tolist(),
                     None if W2 is None else W2.tolist(), None if b2 is None else b2.tolist())
        ti = py_softmax(zi)
        assert z[i] == pytest.approx(zi, rel=1e-13, abs=1e-13)
        assert th[i] == pytest.approx(ti, rel=1e-13)
        for m in range(2):
            want = math.fsum(ti[c] * float(recall[m, c]) for c in range(C))
            assert ea[i, m] == pytest.approx(want, rel=1e-13)


def test_relu_is_applied_between_layers():
    # x W1 = (-1, 2): without the ReLU the logits would be (-1+2, ...) instead of (2, ...)
    x = np.array([[1.0]], dtype=np.float32)
    W1 = np.array([[-1.0, 2.0]], dtype=np.float32)
    W2 = np.array([[1.0, 0.0], [1.0, 1.0]], dtype=np.float32)
    z = orc.head_logits(x, W1, np.zeros(2, np.float32), W2, np.zeros(2, np.float32))
    assert z[0].tolist() == [2.0, 2.0]


def test_bf16_widening_matches_torch():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(3)
    a = rng.standard_normal(1000).astype(np.float32) * 37.0
    bits = wl.f32_to_bf16_bits(a)
    t = torch.from_numpy(a).to(torch.bfloat16)
    assert np.array_equal(bits.view(np.int16), t.view(torch.int16).numpy())
    assert np.array_equal(orc.widen(bits), t.to(torch.float64).numpy())
    assert np.array_equal(wl.bf16_bits_to_f32(bits), t.to(torch.float32).numpy())


def test_confusion_matrix_forms_agree_and_fallback_to_profiled_accuracy():
    # eq. (7) == eq. (9) with theta = class frequencies of the test set
    rng = np.random.default_rng(11)
    for C in (2, 3, 7):
        Z = rng.integers(1, 50, size=(C, C))
        tr_form = Fraction(int(np.trace(Z)), int(Z.sum()))
        assert orc.accuracy_from_confusion(Z) == pytest.approx(float(tr_form), rel=1e-15)
        theta = orc.class_frequency_from_confusion(Z)
        recall = orc.recall_from_confusion(Z)
        assert theta.sum() == pytest.approx(1.0, rel=1e-15)
        ea = orc.expected_accuracy(theta[None, :], recall[None, :])
        assert ea[0, 0] == pytest.approx(float(tr_form), rel=1e-14)


def test_zero_weights_give_uniform_theta_and_mean_recall():
    w = wl.tiny(seed=5, n=9, classes=(4, 3), models=(3, 2), feat_dim=6)
    for a in range(2):
        w.profile.W1[a][:] = 0
    ea, _ = orc.score_requests(w.profile, w.requests)
    for i in range(w.requests.n):
        a = int(w.requests.app[i])
        M = int(w.profile.n_models[a])
        assert ea[i, :M] == pytest.approx(w.profile.acc[a].astype(np.float64).mean(axis=1), rel=1e-14)
        assert np.all(ea[i, M:] == 0)


def test_one_hot_theta_gives_per_class_recall():
    # "true model accuracy": theta = 1 on one label (Sec. 6.3, accuracy-estimation experiment)
    C, M = 5, 3
    recall = np.random.default_rng(2).uniform(0, 1, (M, C)).astype(np.float32)
    for c in range(C):
        z = np.full((1, C), -800.0)
        z[0, c] = 800.0
        ea = orc.expected_accuracy(orc.posterior(z), recall)
        assert ea[0] == pytest.approx(recall[:, c].astype(np.float64), abs=0)


@pytest.mark.parametrize("hidden", [0, 8])
def test_convexity_and_normalisation(hidden):
    w = wl.tiny(seed=21, n=40, classes=(5, 2, 7), models=(3, 1, 4), feat_dim=8, hidden_dim=hidden)
    ea, key, th = orc.score_requests(w.profile, w.requests, return_theta=True)
    for i in range(w.requests.n):
        a = int(w.requests.app[i])
        M = int(w.profile.n_models[a])
        acc = w.profile.acc[a].astype(np.float64)
        assert th[i].shape == (int(w.profile.n_classes[a]),)
        assert th[i].sum() == pytest.approx(1.0, rel=1e-14)
        assert np.all(th[i] >= 0)
        assert np.all(ea[i, :M] >= acc.min(axis=1) - 1e-15)
        assert np.all(ea[i, :M] <= acc.max(axis=1) + 1e-15)
        assert 0.0 <= ea[i, :M].min() and ea[i, :M].max() <= 1.0
        assert key[i] > 0


def test_score_requests_uses_each_requests_own_application():
    w = wl.tiny(seed=4, n=12, classes=(3, 4), models=(2, 3), feat_dim=5)
    ea, _ = orc.score_requests(w.profile, w.requests)
    for i in range(w.requests.n):
        a = int(w.requests.app[i])
        zi = py_head(w.requests.x[i].astype(np.float64).tolist(), w.profile.W1[a].astype(np.float64).tolist(),
                     w.profile.b1[a].astype(np.float64).tolist(), None, None)
        ti = py_softmax(zi)
        for m in range(int(w.profile.n_models[a])):
            want = math.fsum(ti[c] * float(w.profile.acc[a][m, c]) for c in range(len(ti)))
            assert ea[i, m] == pytest.approx(want, rel=1e-13)


# ---- priority (eq. 12) ------------------------------------------------------
def test_population_variance_of_the_papers_variant_set(golden):
    accs = golden["heterogeneity_accuracies"]          # 79.2%, 80%, 80.8%
    delta = Fraction(8, 1000)
    want = float(2 * delta * delta / 3)                # {mu-d, mu, mu+d}: population variance 2 d^2 / 3
    assert want == pytest.approx(4.2667e-5, rel=1e-4)
    assert orc.population_variance(accs) == pytest.approx(want, rel=1e-12)
    # sample variance (divide by M-1) would be 6.4e-5: must not match
    assert abs(orc.population_variance(accs) - 6.4e-5) > 1e-5


def test_single_variant_has_zero_variance_and_priority_is_exp_of_deadline():
    k = orc.request_priority(np.array([[0.7]]), np.array([1000.0], np.float32), 1.0, 1000.0)
    assert k[0] == pytest.approx(math.exp(-1.0), rel=1e-15)
    k = orc.request_priority(np.array([[0.7]]), np.array([250.0], np.float32), np.array([0.5], np.float32), 500.0)
    assert k[0] == pytest.approx(0.5 * math.exp(-0.5), rel=1e-15)


def test_priority_closed_form_and_monotonicity(golden):
    accs = np.array([golden["heterogeneity_accuracies"]])
    var = 2 * 0.008 ** 2 / 3
    k = orc.request_priority(accs, np.array([150.0], np.float32), 1.0, 1000.0)
    assert k[0] == pytest.approx((1 + var) * math.exp(-0.15), rel=1e-12)
    d = np.linspace(1, 500, 50).astype(np.float32)
    kd = orc.request_priority(np.repeat(accs, 50, axis=0), d, 1.0, 1000.0)
    assert np.all(np.diff(kd) < 0)                       # tighter deadline -> higher priority
    spread = np.array([[0.8 - s, 0.8, 0.8 + s] for s in np.linspace(0, 0.15, 20)])
    kv = orc.request_priority(spread, np.full(20, 100.0, np.float32), 1.0, 1000.0)
    assert np.all(np.diff(kv) > 0)                       # more variance -> higher priority


def test_dirichlet_posterior_mean_of_the_papers_example(golden):
    y = golden["knn_evidence_example"]
    a = golden["jeffreys_alpha"][0]
    got = orc.dirichlet_posterior_mean([a, a], y)
    assert got == pytest.approx([2.5 / 6.0, 3.5 / 6.0], rel=1e-15)


def test_smoothed_posterior_reproduces_the_papers_example_from_vote_shares(golden):
    # Sec. 4.2 "Evidence": five neighbours voting <2, 3> are the soft evidence 5 * (0.4, 0.6)
    y = np.asarray(golden["knn_evidence_example"], dtype=np.float64)
    a = golden["jeffreys_alpha"][0]
    got = orc.smoothed_posterior((y / y.sum())[None, :], [a, a], y.sum())
    assert got[0] == pytest.approx([2.5 / 6.0, 3.5 / 6.0], rel=1e-15)


def test_smoothed_posterior_limits_and_shrinkage_form():
    from fractions import Fraction
    rng = np.random.default_rng(21)
    C = 7
    theta = rng.dirichlet(np.full(C, 0.4), size=5)
    alpha = rng.uniform(0.1, 3.0, C)
    # no evidence -> the prior mean, whatever the head says
    got0 = orc.smoothed_posterior(theta, alpha, 0.0)
    assert np.allclose(got0, np.tile(alpha / alpha.sum(), (5, 1)), rtol=1e-15, atol=0)
    # overwhelming evidence -> the head's output; zero prior mass -> the head's output exactly
    assert np.allclose(orc.smoothed_posterior(theta, alpha, 1e14), theta, rtol=0, atol=1e-12)
    assert np.allclose(orc.smoothed_posterior(theta, np.zeros(C), 3.0), theta, rtol=1e-15, atol=0)
    # textbook shrinkage form of a Dirichlet-multinomial posterior mean: lambda * theta + (1 - lambda) * prior mean
    for k in (1.0, 5.0, 20.0):
        lam = k / (alpha.sum() + k)
        want = lam * theta + (1 - lam) * alpha / alpha.sum()
        got = orc.smoothed_posterior(theta, alpha, k)
        assert np.allclose(got, want, rtol=1e-13, atol=0)
        assert np.allclose(got.sum(axis=1), 1.0, rtol=1e-14)
    # exact rational arithmetic on a small case
    th = [Fraction(1, 4), Fraction(1, 2), Fraction(1, 4)]
    al = [Fraction(1, 2), Fraction(3, 2), Fraction(2)]
    k = Fraction(10)
    want = [(al[c] + k * th[c]) / (sum(al) + k) for c in range(3)]
    got = orc.smoothed_posterior(np.array([[float(v) for v in th]]), [float(v) for v in al], float(k))
    assert got[0] == pytest.approx([float(v) for v in want], rel=1e-15)


def test_scoring_with_priors_uses_the_smoothed_posterior_everywhere():
    w = wl.tiny(5, 40, classes=(3, 5, 2), models=(2, 3, 1))
    wl.attach_priors(w.profile, seed=6, kinds=("weak", None, "strong"))
    p, rq = w.profile, w.requests
    ea, key, thetas = orc.score_requests(p, rq, return_theta=True)
    w0 = wl.tiny(5, 40, classes=(3, 5, 2), models=(2, 3, 1))
    ea0, key0, thetas0 = orc.score_requests(w0.profile, w0.requests, return_theta=True)
    for i in range(rq.app.shape[0]):
        a = int(rq.app[i]); M = int(p.n_models[a])
        if p.prior_alpha[a] is None:
            assert np.array_equal(thetas[i], thetas0[i]) and np.array_equal(ea[i], ea0[i]) and key[i] == key0[i]
            continue
        al = p.prior_alpha[a].astype(np.float64); k = float(p.evidence_k[a])
        th = (al + k * thetas0[i]) / (al.sum() + k)
        assert np.allclose(thetas[i], th, rtol=1e-14)
        # eq. (9) on the smoothed posterior, and eq. (12) on those accuracies
        want = [math.fsum(float(th[c]) * float(p.acc[a][m, c]) for c in range(len(th))) for m in range(M)]
        assert ea[i, :M] == pytest.approx(want, rel=1e-13)
        mu = sum(want) / M
        var = sum((v - mu) ** 2 for v in want) / M
        assert key[i] == pytest.approx(float(rq.weight[i]) * (1 + var) * math.exp(-float(rq.deadline_rel_ms[i]) / p.prio_timescale_ms), rel=1e-13)
    # fallback of Sec. 4.1: with no evidence the estimate is the profiled accuracy under the prior's label mix
    for a in range(p.n_apps):
        p.evidence_k[a] = 0.0
    ea_k0, _ = orc.score_requests(p, rq)
    for i in range(rq.app.shape[0]):
        a = int(rq.app[i]); M = int(p.n_models[a])
        if p.prior_alpha[a] is None:
            continue
        mix = p.prior_alpha[a].astype(np.float64); mix = mix / mix.sum()
        assert ea_k0[i, :M] == pytest.approx(orc.expected_accuracy(mix[None, :], p.acc[a])[0], rel=1e-13)


def test_service_order_matches_python_sort_with_ties():
    rng = np.random.default_rng(9)
    n, A = 200, 3
    app = rng.integers(0, A, n).astype(np.int32)
    key = rng.integers(0, 8, n).astype(np.float64) / 8.0      # many duplicates
    got = orc.service_order(app, key, A)
    for a in range(A):
        want = sorted([i for i in range(n) if app[i] == a], key=lambda i: (-key[i], i))
        assert got[a].tolist() == want
