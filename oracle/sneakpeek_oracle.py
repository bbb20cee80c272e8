"""Plain CPU oracle for SneakPeek scoring and batch-aware greedy scheduling.

TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct checker
that the HIP library is compared against.  It is NumPy in float64, follows the
paper's definitions step by step, shares no code with the HIP path and is
never imported by it; only the tests, the smoke check and the benchmark's
CPU-baseline leg may call it.

What each function follows:

* head_logits / posterior  -- Def. 4.1.1, 4.1.2 (a SneakPeek model turns a
  request's data into class probabilities theta).  The parametric heads
  (logistic, one-hidden-layer ReLU MLP, softmax output) are the workload's.
* expected_accuracy        -- Sec. 4.1, eq. (9): Accuracy(m) = sum_c theta_c *
  recall_c(m), with theta treated as a per-request parameter.
* accuracy_from_confusion  -- Sec. 4.1, eq. (7): tr(Z) / sum(Z).
* request_priority         -- Sec. 5.1.1, eq. (12), population variance.
* penalty                  -- Sec. 6.1 (step / linear / sigmoid penalties).
* utility                  -- Sec. 3.1, eq. (2).
* service_order            -- Alg. 1 ("requests in g sorted by priority").
* Window.*                 -- Alg. 1 generalised to batch-capped greedy rounds;
  eq. (1) clock with the batch as the unit; eq. (13) arg max.
* split_labels             -- Sec. 5.3.2, data-aware subgroups of an application.
* dirichlet_posterior_mean -- Sec. 4.2, eq. (10)-(11).
* smoothed_posterior       -- Sec. 4.2, eq. (10)-(11) with the head's output as
  soft evidence (y = k * theta) under a per-application prior.

Readings of points the paper leaves open (all listed in the design notes):
the linear and sigmoid penalties are capped with min(1, .) (the printed
max(1, .) would make every miss worse than the step penalty and break the
monotone 0..1 range eq. (2) needs); deadlines are relative to the window's
start and must be positive; a deadline is missed only when completion is
strictly later; exp(-d) in eq. (12) takes the remaining time in units of a
timescale T_d (1000 ms by default); the per-request weight w multiplies both
the key and the reported utility (w = 1 recovers the paper); every member of a
batch completes at t + L[m,b]; a request is dead once its penalty would be 1
even alone on the fastest variant, and dead requests never come back; an
optional swap-in cost per variant is paid by every batch whose variant differs
from the previous batch's (liveness ignores it, so that it stays monotone).

Parity status: every function here is pinned by tests/test_oracle_*.py
against closed forms, the paper's worked numbers, or brute force, except the
paper's dataset-level results (utility gains on MMAct / Speech Commands /
MIT-BIH), which need data that is not available: parity unpinned for those.
"""
from __future__ import annotations

import numpy as np

PEN_STEP, PEN_LINEAR, PEN_SIGMOID = 0, 1, 2


# --------------------------------------------------------------------------
# inputs
# --------------------------------------------------------------------------
def widen(a):
    """Exact float64 view of an input array (float32, or uint16 bfloat16 bits)."""
    a = np.asarray(a)
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


# --------------------------------------------------------------------------
# SneakPeek posterior and data-aware accuracy (Sec. 4)
# --------------------------------------------------------------------------
def head_logits(x, W1, b1, W2=None, b2=None):
    """Class scores of the SneakPeek head for rows of x.  Logistic: x W1 + b1.
    MLP: relu(x W1 + b1) W2 + b2.  The hidden activations are not rounded."""
    x = widen(x)
    z = x @ widen(W1) + widen(b1)
    if W2 is not None:
        h = np.maximum(z, 0.0)
        z = h @ widen(W2) + widen(b2)
    return z


def posterior(z):
    """theta = softmax(z) along the last axis (SneakPeek probabilities, Def. 4.1.2)."""
    z = np.asarray(z, dtype=np.float64)
    e = np.exp(z - z.max(axis=-1, keepdims=True))
    return e / e.sum(axis=-1, keepdims=True)


def expected_accuracy(theta, recall):
    """eq. (9): EA[i,m] = sum_c theta[i,c] * recall[m,c]."""
    return np.asarray(theta, dtype=np.float64) @ widen(recall).T


def accuracy_from_confusion(Z):
    """eq. (7): profiled accuracy tr(Z) / sum(Z) of a confusion matrix
    (rows = true class, columns = predicted class)."""
    Z = np.asarray(Z, dtype=np.float64)
    return np.trace(Z) / Z.sum()


def class_frequency_from_confusion(Z):
    """theta of the test set: row sums over the grand total (eq. (8))."""
    Z = np.asarray(Z, dtype=np.float64)
    return Z.sum(axis=1) / Z.sum()


def recall_from_confusion(Z):
    """Per-class recall z_ii / sum_j z_ij (eq. (9))."""
    Z = np.asarray(Z, dtype=np.float64)
    return np.diag(Z) / Z.sum(axis=1)


def dirichlet_posterior_mean(alpha, y):
    """Mean of Dirichlet(alpha + y), eq. (10)-(11)."""
    p = np.asarray(alpha, dtype=np.float64) + np.asarray(y, dtype=np.float64)
    return p / p.sum()


def smoothed_posterior(theta, alpha, k):
    """Sec. 4.2: prior Dirichlet(alpha) (eq. 10), evidence a multinomial
    observation of k draws; here the head's softmax output stands for the
    neighbours' votes, y = k * theta, and the estimate is the mean of the
    posterior Dirichlet(alpha + y) (eq. 11), row by row."""
    theta = np.asarray(theta, dtype=np.float64)
    alpha = widen(alpha)
    rows = [dirichlet_posterior_mean(alpha, float(k) * theta[i]) for i in range(theta.shape[0])]
    return np.asarray(rows, dtype=np.float64).reshape(theta.shape)


# --------------------------------------------------------------------------
# priority, penalty, utility (Sec. 3.1, 5.1, 6.1)
# --------------------------------------------------------------------------
def population_variance(v, axis=-1):
    v = np.asarray(v, dtype=np.float64)
    mu = v.mean(axis=axis, keepdims=True)
    return ((v - mu) ** 2).mean(axis=axis)


def request_priority(acc_set, deadline_rel_ms, weight=1.0, timescale_ms=1000.0):
    """eq. (12): (1 + Var[Accuracy(M_a)]) * exp(-d), times the request weight.
    `acc_set` holds the request's accuracies over its application's variants
    along the last axis."""
    var = population_variance(acc_set, axis=-1)
    d = widen(deadline_rel_ms) / float(timescale_ms)
    return widen(weight) * (1.0 + var) * np.exp(-d)


def penalty(kind, deadline, completion):
    """gamma(d, e) of Sec. 6.1; 0 when on time, within [0, 1] when late."""
    d = np.asarray(deadline, dtype=np.float64)
    e = np.asarray(completion, dtype=np.float64)
    d, e = np.broadcast_arrays(d, e)
    late = e > d
    if kind == PEN_STEP:
        return late.astype(np.float64)
    x = 1.0 - (2.0 * d - e) / d          # = (e - d) / d
    g = np.zeros(d.shape, dtype=np.float64)
    if kind == PEN_LINEAR:
        g[late] = np.minimum(1.0, x[late])
        return g
    if kind == PEN_SIGMOID:
        mid = late & (x < 1.0)
        xm = x[mid]
        g[mid] = np.minimum(1.0, 1.0 / (1.0 + (xm / (1.0 - xm)) ** -3.0))
        g[late & (x >= 1.0)] = 1.0
        return g
    raise ValueError(f"unknown penalty kind {kind}")


def utility(accuracy, kind, deadline, completion):
    """eq. (2): Accuracy(m) * [1 - gamma(d, t + l(m))]."""
    return np.asarray(accuracy, dtype=np.float64) * (1.0 - penalty(kind, deadline, completion))


def is_dead(kind, deadline, earliest_completion):
    """A request whose penalty is already 1 on the earliest possible
    completion can no longer earn utility: step -> e > d, else e >= 2 d."""
    d = np.asarray(deadline, dtype=np.float64)
    e = np.asarray(earliest_completion, dtype=np.float64)
    if kind == PEN_STEP:
        return e > d
    return e >= 2.0 * d


# --------------------------------------------------------------------------
# scoring pass over a queue
# --------------------------------------------------------------------------
def score_requests(profile, requests, chunk=16384, return_theta=False):
    """Posterior -> expected accuracy -> priority key for every request.
    Returns EA [N, Mmax] (zero beyond an application's variants) and key [N]."""
    n = int(requests.app.shape[0])
    A = int(profile.n_apps)
    m_max = int(np.max(profile.n_models))
    ea = np.zeros((n, m_max), dtype=np.float64)
    key = np.zeros(n, dtype=np.float64)
    thetas = [None] * n if return_theta else None
    for a in range(A):
        sel = np.nonzero(requests.app == a)[0]
        M = int(profile.n_models[a])
        for s in range(0, sel.shape[0], chunk):
            ids = sel[s:s + chunk]
            z = head_logits(requests.x[ids], profile.W1[a], profile.b1[a], profile.W2[a], profile.b2[a])
            th = posterior(z)
            alpha = None if getattr(profile, "prior_alpha", None) is None else profile.prior_alpha[a]
            if alpha is not None:
                th = smoothed_posterior(th, alpha, profile.evidence_k[a])
            e = expected_accuracy(th, profile.acc[a])
            ea[ids, :M] = e
            key[ids] = request_priority(e, requests.deadline_rel_ms[ids], requests.weight[ids],
                                        profile.prio_timescale_ms)
            if return_theta:
                for j, i in enumerate(ids):
                    thetas[i] = th[j]
    if return_theta:
        return ea, key, thetas
    return ea, key


def split_labels(thetas, threshold=0.5):
    """Sec. 5.3.2 "Enhancements for Grouped Scheduling": a request joins the subgroup of the class its
    SneakPeek probabilities point to (theta_c > 1/2, so at most one class qualifies); with no such class
    it stays in the application's unsplit group.  Returns 1 + class, or 0, per request."""
    out = np.zeros(len(thetas), dtype=np.int64)
    for i, th in enumerate(thetas):
        th = np.asarray(th, dtype=np.float64)
        c = int(np.argmax(th))
        out[i] = 1 + c if th[c] > threshold else 0
    return out


def service_order(app, key, n_apps):
    """Per application, request ids by (key descending, id ascending).  Earliest deadline first is this
    with the negated deadline as the key."""
    out = []
    for a in range(int(n_apps)):
        sel = np.nonzero(np.asarray(app) == a)[0]
        out.append(sel[np.argsort(-np.asarray(key, dtype=np.float64)[sel], kind="stable")])
    return out


# --------------------------------------------------------------------------
# greedy batch-selection rounds
# --------------------------------------------------------------------------
class Window:
    """State of one scheduling window: who is still pending, the worker clock
    t (ms since the window's start), and what has been assigned so far."""

    def __init__(self, profile, requests, ea=None, key=None, policy=None, sub=None):
        self.p = profile
        self.n = int(requests.app.shape[0])
        self.app = np.asarray(requests.app)
        self.D = widen(requests.deadline_rel_ms)
        self.w = widen(requests.weight)
        if ea is None or key is None:
            ea, key = score_requests(profile, requests)
        self.ea = np.asarray(ea, dtype=np.float64)
        self.key = np.asarray(key, dtype=np.float64)
        # policy knobs (Sec. 6.1 baselines, Alg. 1); plain integer codes, 0 everywhere = the default
        g = (lambda name: int(getattr(policy, name, 0))) if policy is not None else (lambda name: 0)
        self.edf, self.group_first, self.whole = g("order") == 1, g("select") == 1, g("batch_rule") == 1
        self.max_accuracy, self.unit_weight = g("choice") == 1, g("weight") == 1
        cap = g("batch_cap")
        self.B = min(int(profile.max_batch), cap) if cap > 0 else int(profile.max_batch)
        # what orders requests inside an application, and what a group's priority averages (eq. 14)
        self.omega = -self.D if self.edf else self.key
        self.wsum = np.ones(self.n) if self.unit_weight else self.key
        # groups: the applications, or (Sec. 5.3.2) every non-empty (application, subgroup) pair in
        # ascending order; everything below that takes a group index g looks its tables up through gapp
        if g("split_groups") == 1:
            assert sub is not None, "group splitting needs the subgroup label of every request (split_labels)"
            pairs = sorted(set(zip(self.app.tolist(), np.asarray(sub).tolist())))
            index = {pr: i for i, pr in enumerate(pairs)}
            self.gapp = [int(pr[0]) for pr in pairs]
            self.gid = np.array([index[(int(a), int(sb))] for a, sb in zip(self.app, np.asarray(sub))], dtype=np.int64)
        else:
            self.gapp = list(range(int(profile.n_apps)))
            self.gid = self.app.astype(np.int64)
        self.G = len(self.gapp)
        self.order = service_order(self.gid, self.omega, self.G)
        self.lat = [widen(l) for l in profile.lat_ms]
        self.lmin = [float(l[:, 0].min()) for l in self.lat]
        # cost of bringing a variant in (Sec. 3.1 counts switching cost as part of a variant's latency;
        # Sec. 5.2 groups requests so that a loaded variant is reused): paid by a batch unless the
        # previous batch of the window ran the same variant of the same application
        swap = getattr(profile, "swap_ms", None)
        self.swap = [None if (swap is None or swap[a] is None) else widen(swap[a]) for a in range(int(profile.n_apps))]
        self.resident = None                 # (application, variant) of the last committed batch
        self.alive = np.ones(self.n, dtype=bool)
        self.t = 0.0
        self.round = 0
        self.next_order = 1
        self.model = np.full(self.n, -1, dtype=np.int32)
        self.round_of = np.full(self.n, -1, dtype=np.int32)
        self.order_of = np.zeros(self.n, dtype=np.int32)
        self.util = np.zeros(self.n, dtype=np.float64)
        self.finish = np.zeros(self.n, dtype=np.float64)
        self.log = []

    # -- who can still be served -------------------------------------------
    def live_queue(self, g):
        """Live requests of group g (an application, or one of its subgroups) in service order."""
        a = self.gapp[g]
        ids = self.order[g]
        ids = ids[self.alive[ids]]
        dead = is_dead(int(self.p.penalty[a]), self.D[ids], self.t + self.lmin[a])
        return ids[~dead]

    def candidate_window(self, g):
        return self.live_queue(g)[: self.B]

    def scoring_penalty(self, a):
        """Penalty kind the candidates are compared under: the application's own (eq. 13), or the step
        penalty when variants are compared by accuracy among those that meet the deadline."""
        return PEN_STEP if self.max_accuracy else int(self.p.penalty[a])

    def group_priority(self, g):
        """eq. (14) over the group's candidate window; None when it is empty."""
        q = self.candidate_window(g)
        return None if q.shape[0] == 0 else float(np.mean(self.omega[q]))

    def start_time(self, a, m):
        """When a batch on variant m of application a starts computing: now, plus the swap-in cost
        unless that variant is the resident one."""
        if self.swap[a] is None or self.resident == (a, m):
            return self.t
        return self.t + self.swap[a][m]

    # -- candidate scores ----------------------------------------------------
    def score_cube(self):
        """Score[a, m, b-1] = sum_{j<=b} key_j * EA[j,m] * (1 - gamma_a(D_j, t + L[a][m][b]))
        over the first b live requests of a; -inf where (a,m,b) is not a candidate."""
        G, B = self.G, int(self.p.max_batch)     # the cube keeps the profile's width; sizes above the cap stay -inf
        m_max = int(np.max(self.p.n_models))
        cube = np.full((G, m_max, B), -np.inf, dtype=np.float64)
        for g in range(G):
            a = self.gapp[g]
            q = self.candidate_window(g)
            nb = q.shape[0]
            if nb == 0:
                continue
            kind = self.scoring_penalty(a)
            for m in range(int(self.p.n_models[a])):
                for b in range(1, nb + 1):
                    if self.whole and b != nb:
                        continue
                    e = self.start_time(a, m) + self.lat[a][m, b - 1]
                    members = q[:b]
                    terms = self.wsum[members] * utility(self.ea[members, m], kind, self.D[members], e)
                    cube[g, m, b - 1] = terms.sum()
        return cube

    def score_cube_fast(self):
        """Same numbers as score_cube with the (b, j) triangle done as one
        masked array per (a, m); kept beside the loop version so that a test
        can check one against the other."""
        G, B = self.G, int(self.p.max_batch)     # the cube keeps the profile's width; sizes above the cap stay -inf
        m_max = int(np.max(self.p.n_models))
        cube = np.full((G, m_max, B), -np.inf, dtype=np.float64)
        for g in range(G):
            a = self.gapp[g]
            q = self.candidate_window(g)
            nb = q.shape[0]
            if nb == 0:
                continue
            kind = self.scoring_penalty(a)
            tri = np.tril(np.ones((nb, nb), dtype=bool))          # [b, j]: j <= b
            for m in range(int(self.p.n_models[a])):
                e = self.start_time(a, m) + self.lat[a][m, :nb]    # [b]
                u = utility(self.ea[q, m][None, :], kind, self.D[q][None, :], e[:, None])
                terms = np.where(tri, self.wsum[q][None, :] * u, 0.0)
                cube[g, m, :nb] = terms.sum(axis=1)
                if self.whole:
                    cube[g, m, : nb - 1] = -np.inf
        return cube

    def decide(self, cube=None):
        """arg max over (a, m, b); exact ties go to the smallest (a, m, b).
        Returns None when no application has a live request."""
        if cube is None:
            cube = self.score_cube_fast()
        if not np.isfinite(cube).any():
            return None
        if self.group_first:
            # Alg. 1: the group with the highest mean priority goes first (ties: smallest application),
            # then the variant (and batch size) is chosen for that group alone
            prio = [self.group_priority(g) for g in range(cube.shape[0])]
            best = max(v for v in prio if v is not None)
            g_star = min(g for g, v in enumerate(prio) if v is not None and v == best)
            masked = np.full_like(cube, -np.inf)
            masked[g_star] = cube[g_star]
            cube = masked
        flat = int(np.argmax(cube))            # first maximum in C order = smallest (group, m, b)
        g, m, bi = np.unravel_index(flat, cube.shape)
        b = int(bi) + 1
        a = self.gapp[int(g)]
        ids = self.candidate_window(int(g))[:b]
        return {"app": a, "group": int(g), "model": int(m), "batch": b, "score": float(cube[g, m, bi]),
                "ids": ids.copy(), "t_start": self.t,
                "t_end": self.start_time(a, int(m)) + self.lat[a][int(m), bi]}

    # -- commit ---------------------------------------------------------------
    def commit(self, a, m, ids):
        """Serve requests `ids` of application a as one batch on variant m."""
        ids = np.asarray(ids, dtype=np.int64)
        b = int(ids.shape[0])
        assert 1 <= b <= self.B
        assert np.all(self.app[ids] == a) and np.all(self.alive[ids])
        t_end = self.start_time(a, m) + self.lat[a][m, b - 1]
        u = utility(self.ea[ids, m], int(self.p.penalty[a]), self.D[ids], t_end)
        self.model[ids] = m
        self.round_of[ids] = self.round
        self.order_of[ids] = np.arange(self.next_order, self.next_order + b)
        self.util[ids] = u
        self.finish[ids] = t_end
        self.alive[ids] = False
        rec = {"app": a, "model": m, "batch": b, "round": self.round, "t_start": self.t, "t_end": t_end,
               "batch_utility": float((self.w[ids] * u).sum()), "ids": ids.copy()}
        self.log.append(rec)
        self.next_order += b
        self.round += 1
        self.t = t_end
        self.resident = (a, m)
        return rec

    def step(self):
        d = self.decide()
        if d is None:
            return None
        rec = self.commit(d["app"], d["model"], d["ids"])
        rec["score"] = d["score"]
        return rec

    def run(self, max_rounds=0):
        """Greedy rounds until nothing is live (or max_rounds > 0 is reached)."""
        while max_rounds <= 0 or self.round < max_rounds:
            if self.step() is None:
                break
        return self.summary()

    def summary(self):
        done = self.model >= 0
        viol = np.maximum(0.0, self.finish[done] - self.D[done])
        return {"total_weighted_utility": float((self.w * self.util).sum()),
                "mean_utility": float(self.util.sum() / self.n) if self.n else 0.0,
                "total_violation_ms": float(viol.sum()),
                "n_rounds": int(self.round), "n_scheduled": int(done.sum()),
                "n_dropped": int(self.n - done.sum())}
