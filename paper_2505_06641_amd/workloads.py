"""Seeded synthetic workloads shaped like the paper's applications.

This module only draws random inputs (profiles and pending requests) and holds
none of the method's arithmetic: no posterior, no expected accuracy, no
utility, no ordering.  Both the CPU checker and the HIP library are fed from
the arrays produced here, so the two sides see identical bytes.

The shapes follow the paper's evaluation set-up (a few applications with a
handful of classes and two to five model variants each, skewed label mixes,
deadlines of tens to hundreds of milliseconds against variant latencies of
tens of milliseconds; Sec. 6.1, Table 1), scaled up to GPU-sized queues.  The
paper's datasets and served models are not used; these inputs stand in for
them.

Draw order (fixed, so a seed names one workload): for each application in
turn -- head weights, per-class accuracy table, latency coefficients
(alpha, beta), then (skewed configs only) the Dirichlet label mix and the
per-class unit directions; afterwards for the whole queue -- the application
permutation, labels, features, deadlines, weights.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

PEN_STEP, PEN_LINEAR, PEN_SIGMOID = 0, 1, 2
F32, BF16 = 0, 1


@dataclass
class Profile:
    """Registered applications: SneakPeek head, per-class recall and latency
    tables of every model variant (Sec. 2.2 "System Model", Sec. 3.2)."""
    n_apps: int
    feat_dim: int
    hidden_dim: int                 # 0 -> logistic head
    max_batch: int
    feat_dtype: int                 # F32 or BF16 (features and head weights)
    n_classes: np.ndarray           # int32 [A]
    n_models: np.ndarray            # int32 [A]
    W1: List[np.ndarray]            # per app [d,H] or [d,C]; float32, or uint16 bf16 bits
    b1: List[np.ndarray]            # per app float32 [H] or [C]
    W2: List[Optional[np.ndarray]]  # per app [H,C] or None
    b2: List[Optional[np.ndarray]]  # per app float32 [C] or None
    acc: List[np.ndarray]           # per app float32 [M_a, C_a]
    theta_test: List[Optional[np.ndarray]]  # per app float32 [C_a] or None
    lat_ms: List[np.ndarray]        # per app float32 [M_a, B]
    penalty: np.ndarray             # int32 [A]
    prio_timescale_ms: float = 1000.0
    max_requests: int = 0
    # optional Dirichlet prior per application (Sec. 4.2): alpha float32 [C_a] or None, and the weight k
    # (number of multinomial draws) the head's output carries as evidence
    prior_alpha: Optional[List[Optional[np.ndarray]]] = None
    evidence_k: Optional[np.ndarray] = None   # float32 [A]
    # optional swap-in cost per variant (Sec. 3.1 "context switch time"): float32 [M_a] per app or None
    swap_ms: Optional[List[Optional[np.ndarray]]] = None


# Scheduling policy knobs (Sec. 6.1 "Baselines and Metrics", Alg. 1).  Plain codes shared by the C ABI,
# the binding and the oracle; no arithmetic here.
ORDER_PRIORITY, ORDER_EDF = 0, 1            # service order inside an application: eq. (12) key, or earliest deadline first
SELECT_JOINT, SELECT_GROUP_FIRST = 0, 1     # one arg max over (a, m, b), or first the group by its mean priority (eq. 14)
BATCH_FREE, BATCH_WHOLE = 0, 1              # any batch size up to the cap, or the whole candidate window (groups run whole)
CHOICE_UTILITY, CHOICE_MAX_ACCURACY = 0, 1  # variants compared by utility (eq. 13), or by accuracy among those on time
WEIGHT_KEY, WEIGHT_UNIT = 0, 1              # utilities of a batch summed with the requests' keys as weights, or plainly


@dataclass
class Policy:
    order: int = ORDER_PRIORITY
    select: int = SELECT_JOINT
    batch_rule: int = BATCH_FREE
    choice: int = CHOICE_UTILITY
    weight: int = WEIGHT_KEY
    batch_cap: int = 0                      # > 0: batches of at most this many requests
    split_groups: int = 0                   # 1: data-aware subgroups per predicted class (Sec. 5.3.2)


def named_policy(name: str) -> Policy:
    """The approaches of Sec. 6.1 in terms of the knobs above (the data-oblivious ones additionally
    replace the posterior by the profiling label mix: a prior with no evidence)."""
    return {
        "sneakpeek": Policy(),
        "alg1": Policy(select=SELECT_GROUP_FIRST, batch_rule=BATCH_WHOLE, weight=WEIGHT_UNIT),
        "lo_priority": Policy(select=SELECT_GROUP_FIRST, batch_cap=1),
        "lo_edf": Policy(order=ORDER_EDF, select=SELECT_GROUP_FIRST, batch_cap=1),
        "maxacc_edf": Policy(order=ORDER_EDF, select=SELECT_GROUP_FIRST, choice=CHOICE_MAX_ACCURACY, batch_cap=1),
    }[name]


@dataclass
class Requests:
    """Pending requests of one scheduling window (Sec. 3.1)."""
    x: np.ndarray                   # [N,d] float32, or uint16 bf16 bits
    app: np.ndarray                 # int32 [N]
    deadline_rel_ms: np.ndarray     # float32 [N], d_i - now > 0
    weight: np.ndarray              # float32 [N], >= 0
    label: Optional[np.ndarray] = None   # int32 [N] hidden class (generator bookkeeping only)

    @property
    def n(self) -> int:
        return int(self.app.shape[0])


@dataclass
class Workload:
    name: str
    seed: int
    profile: Profile
    requests: Requests
    rounds: int                     # <=0: run until the queue is exhausted
    notes: dict = field(default_factory=dict)


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even conversion of float32 to bfloat16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns to float32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def split_counts(n: int, fractions) -> np.ndarray:
    """floor(n*f) per application; the remainder goes to the first ones."""
    c = np.floor(np.asarray(fractions, dtype=np.float64) * n + 1e-9).astype(np.int64)
    rem = n - int(c.sum())
    for i in range(rem):
        c[i % len(c)] += 1
    return c


@dataclass
class Recipe:
    name: str
    seed: int
    n_requests: int
    classes: tuple
    models: tuple
    fractions: tuple
    feat_dim: int
    hidden_dim: int
    feat_dtype: int
    max_batch: int
    head_init: str                  # "normal0.1" | "he"
    acc_dist: tuple                 # ("uniform", lo, hi) | ("beta", a, b)
    alpha: tuple                    # ("fixed", values) | ("uniform", lo, hi)
    beta: tuple
    deadline: tuple                 # (lo, hi) ms
    weight_dist: str                # "uniform" | "pareto2"
    dirichlet: float                # 0 -> no label shift
    rounds: int
    penalty: int = PEN_SIGMOID


def _equal(n):
    return tuple([1.0 / n] * n)


RECIPES = {
    "cfg1": Recipe("cfg1", 0, 256, (10,), (3,), (1.0,), 32, 0, F32, 16, "normal0.1",
                   ("uniform", 0.5, 0.99), ("fixed", (2.0, 5.0, 12.0)), ("fixed", (0.3, 0.8, 2.0)),
                   (10.0, 100.0), "uniform", 0.0, 1),
    "cfg2": Recipe("cfg2", 1, 4096, (10, 7, 2), (4, 4, 4), (0.5, 0.3, 0.2), 128, 64, F32, 32, "he",
                   ("uniform", 0.4, 0.99), ("uniform", 1.0, 15.0), ("uniform", 0.2, 2.5),
                   (20.0, 200.0), "uniform", 0.0, 0),
    "cfg3": Recipe("cfg3", 2, 16384, (10, 7, 2), (4, 4, 4), (0.5, 0.3, 0.2), 128, 64, F32, 32, "he",
                   ("uniform", 0.4, 0.99), ("uniform", 1.0, 15.0), ("uniform", 0.2, 2.5),
                   (5.0, 30.0), "uniform", 0.0, 0),
    "cfg4": Recipe("cfg4", 3, 65536, (100,) * 8, (8,) * 8, _equal(8), 512, 256, BF16, 64, "he",
                   ("beta", 8.0, 2.0), ("uniform", 1.0, 20.0), ("uniform", 0.1, 3.0),
                   (10.0, 150.0), "uniform", 0.3, 64),
    "cfg5": Recipe("cfg5", 4, 1048576, (1000,) * 32, (16,) * 32, _equal(32), 256, 0, F32, 128, "normal0.1",
                   ("beta", 6.0, 3.0), ("uniform", 0.5, 30.0), ("uniform", 0.05, 4.0),
                   (5.0, 500.0), "pareto2", 0.1, 64),
}


def _draw_table(rng, dist, shape):
    if dist[0] == "uniform":
        return rng.uniform(dist[1], dist[2], size=shape)
    if dist[0] == "beta":
        return rng.beta(dist[1], dist[2], size=shape)
    raise ValueError(dist)


def _draw_coeff(rng, spec, m):
    if spec[0] == "fixed":
        v = np.asarray(spec[1], dtype=np.float64)
        assert v.shape[0] == m
        return v
    return rng.uniform(spec[1], spec[2], size=m)


def generate(recipe: Recipe, n_requests: Optional[int] = None, seed: Optional[int] = None) -> Workload:
    """Draw one workload.  `n_requests` / `seed` override the recipe's (used
    by tests that want the same shape at a smaller queue length)."""
    r = recipe
    n = r.n_requests if n_requests is None else int(n_requests)
    seed = r.seed if seed is None else int(seed)
    rng = np.random.Generator(np.random.PCG64(seed))
    A, d, H, B = len(r.classes), r.feat_dim, r.hidden_dim, r.max_batch
    W1, b1, W2, b2, acc, lat, mix, dirs = [], [], [], [], [], [], [], []

    def cast_w(w):
        w = w.astype(np.float32)
        return f32_to_bf16_bits(w) if r.feat_dtype == BF16 else w

    for a in range(A):
        C, M = r.classes[a], r.models[a]
        if H == 0:
            std = 0.1 if r.head_init == "normal0.1" else np.sqrt(2.0 / d)
            W1.append(cast_w(rng.normal(0.0, std, size=(d, C))))
            b1.append(np.zeros(C, dtype=np.float32))
            W2.append(None)
            b2.append(None)
        else:
            W1.append(cast_w(rng.normal(0.0, np.sqrt(2.0 / d), size=(d, H))))
            b1.append(np.zeros(H, dtype=np.float32))
            W2.append(cast_w(rng.normal(0.0, np.sqrt(2.0 / H), size=(H, C))))
            b2.append(np.zeros(C, dtype=np.float32))
        acc.append(_draw_table(rng, r.acc_dist, (M, C)).astype(np.float32))
        alpha = _draw_coeff(rng, r.alpha, M)
        beta = _draw_coeff(rng, r.beta, M)
        bsz = np.arange(1, B + 1, dtype=np.float64)
        lat.append((alpha[:, None] + beta[:, None] * bsz[None, :]).astype(np.float32))
        if r.dirichlet > 0:
            mix.append(rng.dirichlet(np.full(C, r.dirichlet)))
            u = rng.standard_normal((C, d))
            u /= np.linalg.norm(u, axis=1, keepdims=True)
            dirs.append(u.astype(np.float32))

    counts = split_counts(n, r.fractions)
    app = np.repeat(np.arange(A, dtype=np.int32), counts)
    app = app[rng.permutation(n)].astype(np.int32)

    label = np.zeros(n, dtype=np.int32)
    if r.dirichlet > 0:
        for a in range(A):
            sel = np.nonzero(app == a)[0]
            p = mix[a] / mix[a].sum()
            label[sel] = rng.choice(r.classes[a], size=sel.shape[0], p=p).astype(np.int32)

    x = rng.standard_normal((n, d), dtype=np.float32)
    if r.dirichlet > 0:
        step = 1 << 16
        for a in range(A):
            sel = np.nonzero(app == a)[0]
            for s in range(0, sel.shape[0], step):
                ids = sel[s:s + step]
                x[ids] += dirs[a][label[ids]]
    if r.feat_dtype == BF16:
        x = f32_to_bf16_bits(x)

    D = rng.uniform(r.deadline[0], r.deadline[1], size=n).astype(np.float32)
    if r.weight_dist == "uniform":
        w = rng.uniform(0.0, 1.0, size=n)
    elif r.weight_dist == "pareto2":
        w = rng.pareto(2.0, size=n)
        w = w / w.max()
    else:
        raise ValueError(r.weight_dist)
    w = w.astype(np.float32)

    prof = Profile(
        n_apps=A, feat_dim=d, hidden_dim=H, max_batch=B, feat_dtype=r.feat_dtype,
        n_classes=np.asarray(r.classes, dtype=np.int32), n_models=np.asarray(r.models, dtype=np.int32),
        W1=W1, b1=b1, W2=W2, b2=b2, acc=acc, theta_test=[None] * A, lat_ms=lat,
        penalty=np.full(A, r.penalty, dtype=np.int32), prio_timescale_ms=1000.0, max_requests=n)
    req = Requests(x=x, app=app, deadline_rel_ms=D, weight=w, label=label)
    return Workload(name=r.name, seed=seed, profile=prof, requests=req, rounds=r.rounds,
                    notes={"counts": counts.tolist()})


def make(name: str, n_requests: Optional[int] = None, seed: Optional[int] = None) -> Workload:
    return generate(RECIPES[name], n_requests=n_requests, seed=seed)


def tiny(seed: int, n: int, classes=(3,), models=(2,), max_batch=4, feat_dim=4, hidden_dim=0,
         penalty=PEN_SIGMOID, deadline=(5.0, 40.0), alpha=(1.0, 6.0), beta=(0.2, 2.0),
         feat_dtype=F32, fractions=None) -> Workload:
    """Small random workload with free shape parameters (ragged class and
    variant counts allowed) for brute-force and edge-case tests."""
    A = len(classes)
    rec = Recipe(f"tiny{seed}", seed, n, tuple(classes), tuple(models),
                 tuple(fractions) if fractions is not None else _equal(A), feat_dim, hidden_dim,
                 feat_dtype, max_batch, "he", ("uniform", 0.3, 0.99), ("uniform",) + tuple(alpha),
                 ("uniform",) + tuple(beta), tuple(deadline), "uniform", 0.0, 0, penalty)
    return generate(rec)


def attach_priors(profile: Profile, seed: int, kinds=("jeffreys", "weak", "strong", None), window: int = 24) -> Profile:
    """Gives every application a prior of the kinds Sec. 6.3.3 ("Choice of Prior") compares, cycling through `kinds`:
    "jeffreys" alpha_c = 0.5; "weak" alpha = an expected label frequency vector; "strong" alpha =
    expected label counts in a scheduling window of `window` requests; None = no prior.  The evidence
    weight k is drawn from {1, 5, 10, 20}.  Seeded; holds no arithmetic of the method."""
    rng = np.random.Generator(np.random.PCG64(seed))
    alphas, ks = [], np.zeros(profile.n_apps, dtype=np.float32)
    for a in range(profile.n_apps):
        C = int(profile.n_classes[a])
        kind = kinds[a % len(kinds)]
        freq = rng.dirichlet(np.full(C, 0.7))
        ks[a] = np.float32(rng.choice([1.0, 5.0, 10.0, 20.0]))
        if kind is None:
            alphas.append(None)
        elif kind == "jeffreys":
            alphas.append(np.full(C, 0.5, dtype=np.float32))
        elif kind == "weak":
            alphas.append(freq.astype(np.float32))
        else:
            alphas.append((freq * window).astype(np.float32))
    profile.prior_alpha = alphas
    profile.evidence_k = ks
    return profile


def attach_swap_costs(profile: Profile, seed: int, lo: float = 0.5, hi: float = 8.0, skip_every: int = 0) -> Profile:
    """Uniform(lo, hi) ms of swap-in cost for every variant (every `skip_every`-th application gets none)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    out = []
    for a in range(profile.n_apps):
        v = rng.uniform(lo, hi, int(profile.n_models[a])).astype(np.float32)
        out.append(None if (skip_every and a % skip_every == skip_every - 1) else v)
    profile.swap_ms = out
    return profile
