"""CPU reference for the scheduling front-end (TEST INFRASTRUCTURE ONLY).

The paper's components, in the order a request meets them (Sec. 3, Fig. 5):

  Impact Estimator   (Sec. 3.3)  cost of a request from its size: ordinary least squares
                                 for text, quantile regression at the 90th percentile for
                                 image / video requests
  Request Classifier (Sec. 3.4)  "naive": modality -> class; "smart": a clustering model
                                 with three clusters on the estimator's two outputs
  Queue Manager      (Sec. 3.5)  one FCFS queue per class
  Priority Regulator (Sec. 3.6)  Priority_c = Static_c + (1 - exp(-k_c * wait^p_c)),
                                 Score_c = -log(Priority_c), lowest score is served next;
                                 constants of Sec. 4.1 ("Configuration")

Each function is the definition written out: least squares in closed form, the
quantile regression as the linear program it is defined by (solved by
scipy.optimize.linprog, a library primitive used as a step), the regulator's two
formulas, and a plain event loop for one non-preemptive server.

Readings where the paper is silent (all stated again in the design notes):
  * the clustering model is k-means (Lloyd's iterations, k = 3) on the two features
    after log(1 + v) and per-feature standardisation; the initial centroids are the
    requests at the 1/6, 3/6 and 5/6 quantiles of the first feature (deterministic);
    clusters are named motorcycle / car / truck by increasing centroid of the first
    feature; ties in the assignment go to the lower cluster index;
  * Score at Priority 0 (a truck that has not waited) is +infinity; equal scores are
    served in arrival order;
  * inside a class the oldest request is served first (its priority is the highest
    of its class, because the age term grows with the wait).

Pins (tests/test_oracle_scheduler.py): least squares against numpy.polyfit and exact
recovery of a line; quantile regression against exhaustive search over all lines
through two data points, the quantile property of its residuals, and the sample
quantile for constant x; regulator values against hand-evaluated numbers for the
paper's constants (tests/golden/priority_regulator.txt), its limits at wait 0 and
infinity and the ordering of the three classes the paper describes; the server loop
against a hand-worked trace, against the Pollaczek-Khinchine mean wait of an M/D/1
queue, and policy-independent invariants (work conservation); clustering against
brute-force optimal partitions on small inputs.
"""
from __future__ import annotations

import math
from typing import Sequence

import numpy as np
from scipy.optimize import linprog

MOTORCYCLE, CAR, TRUCK = 0, 1, 2
FCFS, STATIC, REGULATED = 0, 1, 2

# Sec. 4.1, "Configuration": StaticPriority, k and p for motorcycles, cars, trucks
PAPER_REGULATOR = {"static": (0.1, 0.05, 0.0), "k": (0.05, 0.003, 0.00075), "p": (3.5, 2.5, 1.1)}


# ---- Impact Estimator (Sec. 3.3) ----------------------------------------------------------
def fit_linear(x, y):
    """Least squares line y ~ intercept + slope * x; returns (slope, intercept)."""
    x = np.asarray(x, np.float64)
    y = np.asarray(y, np.float64)
    xm, ym = x.mean(), y.mean()
    sxx = ((x - xm) ** 2).sum()
    if sxx == 0.0:
        return 0.0, float(ym)
    slope = ((x - xm) * (y - ym)).sum() / sxx
    return float(slope), float(ym - slope * xm)


def pinball_loss(x, y, q, slope, intercept):
    """Sum over the points of rho_q(r), r = y - (intercept + slope*x), rho_q(r) = q*r for
    r >= 0 and (q-1)*r otherwise."""
    r = np.asarray(y, np.float64) - (intercept + slope * np.asarray(x, np.float64))
    return float(np.where(r >= 0, q * r, (q - 1.0) * r).sum())


def fit_quantile(x, y, q):
    """Quantile regression at level q: the line minimising the pinball loss, as the linear
    program  min q*sum(u) + (1-q)*sum(v)  s.t.  intercept + slope*x_i + u_i - v_i = y_i,
    u, v >= 0.  Returns (slope, intercept, loss).  The minimiser need not be unique; the
    loss is."""
    x = np.asarray(x, np.float64)
    y = np.asarray(y, np.float64)
    n = len(x)
    c = np.concatenate([[0.0, 0.0], np.full(n, q), np.full(n, 1.0 - q)])
    a_eq = np.hstack([np.ones((n, 1)), x[:, None], np.eye(n), -np.eye(n)])
    bounds = [(None, None), (None, None)] + [(0, None)] * (2 * n)
    res = linprog(c, A_eq=a_eq, b_eq=y, bounds=bounds, method="highs")
    if res.status != 0:
        raise RuntimeError(res.message)
    intercept, slope = float(res.x[0]), float(res.x[1])
    return slope, intercept, pinball_loss(x, y, q, slope, intercept)


def fit_linear2(x1, x2, y):
    """Least squares plane y ~ c0 + c1*x1 + c2*x2; returns (c0, c1, c2).  The second regressor is meant for the
    sum of squared attention-segment lengths of a request: the encoder's attention work grows with it while the
    rest grows with the token count, so a model that is "simple" in the sense of Sec. 3.3 but has both terms
    follows long videos where a line in the token count cannot.  Regressors that carry no information of their own
    (constant, or proportional to each other after centring) get the minimum-norm solution of the centred and
    scaled problem, which puts no weight on a constant column."""
    x1 = np.asarray(x1, np.float64)
    x2 = np.asarray(x2, np.float64)
    y = np.asarray(y, np.float64)
    m = np.array([x1.mean(), x2.mean()])
    z = np.stack([x1, x2], 1) - m
    sc = np.sqrt((z ** 2).sum(0))
    sc[sc == 0.0] = 1.0
    coef, *_ = np.linalg.lstsq(z / sc, y - y.mean(), rcond=1e-10)
    c = coef / sc
    return float(y.mean() - c @ m), float(c[0]), float(c[1])


def pinball_loss2(x1, x2, y, q, c):
    r = np.asarray(y, np.float64) - (c[0] + c[1] * np.asarray(x1, np.float64) + c[2] * np.asarray(x2, np.float64))
    return float(np.where(r >= 0, q * r, (q - 1.0) * r).sum())


def fit_quantile2(x1, x2, y, q):
    """Quantile regression at level q with two regressors, as the same linear program as fit_quantile with one
    more free variable.  Returns ((c0, c1, c2), loss); only the loss is unique."""
    x1 = np.asarray(x1, np.float64)
    x2 = np.asarray(x2, np.float64)
    y = np.asarray(y, np.float64)
    n = len(y)
    # scaled columns keep the program well conditioned (x2 reaches 1e9)
    s1 = max(np.abs(x1).max(), 1e-300)
    s2 = max(np.abs(x2).max(), 1e-300)
    c = np.concatenate([[0.0, 0.0, 0.0], np.full(n, q), np.full(n, 1.0 - q)])
    a_eq = np.hstack([np.ones((n, 1)), (x1 / s1)[:, None], (x2 / s2)[:, None], np.eye(n), -np.eye(n)])
    bounds = [(None, None)] * 3 + [(0, None)] * (2 * n)
    res = linprog(c, A_eq=a_eq, b_eq=y, bounds=bounds, method="highs")
    if res.status != 0:
        raise RuntimeError(res.message)
    coef = (float(res.x[0]), float(res.x[1] / s1), float(res.x[2] / s2))
    return coef, pinball_loss2(x1, x2, y, q, coef)


# ---- Request Classifier (Sec. 3.4) --------------------------------------------------------
def classify_naive(modality: int) -> int:
    """text -> motorcycle, image -> car, video -> truck (modality codes 0, 1, 2)."""
    return {0: MOTORCYCLE, 1: CAR, 2: TRUCK}[int(modality)]


def _features(f):
    return np.log1p(np.asarray(f, np.float64))


def cluster_fit(features, max_iter: int = 100):
    """features [n, 2] = (estimated time, tokens), both >= 0.  Returns a dict with the
    standardisation (mean, scale) and the three centroids in standardised log space,
    ordered by their first coordinate."""
    z = _features(features)
    mean = z.mean(axis=0)
    scale = z.std(axis=0)
    scale = np.where(scale > 0, scale, 1.0)
    z = (z - mean) / scale
    n = len(z)
    order = np.argsort(z[:, 0], kind="stable")
    cent = np.stack([z[order[min(n - 1, (2 * j + 1) * n // 6)]] for j in range(3)])
    assign = None
    for _ in range(max_iter):
        d2 = ((z[:, None, :] - cent[None, :, :]) ** 2).sum(axis=2)
        new = np.argmin(d2, axis=1)                      # first minimum = lower index on ties
        if assign is not None and np.array_equal(new, assign):
            break
        assign = new
        for j in range(3):
            if np.any(assign == j):
                cent[j] = z[assign == j].mean(axis=0)    # an empty cluster keeps its centroid
    cent = cent[np.argsort(cent[:, 0], kind="stable")]
    return {"mean": mean, "scale": scale, "centroid": cent}


def cluster_assign(model, time, tokens) -> int:
    z = (_features([time, tokens]) - model["mean"]) / model["scale"]
    return int(np.argmin(((model["centroid"] - z) ** 2).sum(axis=1)))


# ---- Priority Regulator (Sec. 3.6) --------------------------------------------------------
def priority(cls: int, wait: float, reg=PAPER_REGULATOR) -> float:
    return reg["static"][cls] + (1.0 - math.exp(-reg["k"][cls] * wait ** reg["p"][cls]))


def score(cls: int, wait: float, reg=PAPER_REGULATOR) -> float:
    pr = priority(cls, wait, reg)
    return math.inf if pr <= 0.0 else -math.log(pr)


# ---- Queue Manager + one server (Sec. 3.5) -------------------------------------------------
def simulate(policy: int, arrival: Sequence[float], service: Sequence[float], cls: Sequence[int],
             reg=PAPER_REGULATOR):
    """One non-preemptive server.  Requests (sorted by arrival time) wait in the queue of
    their class; whenever the server is free it takes, among the waiting requests,
      FCFS       the earliest arrival,
      STATIC     the earliest arrival of the highest non-empty class (motorcycle first),
      REGULATED  the lowest Score at that moment (earliest arrival on ties).
    Returns the start time of every request."""
    n = len(arrival)
    start = [None] * n
    waiting = []                       # indices, in arrival order
    nxt, now, done = 0, 0.0, 0
    while done < n:
        while nxt < n and arrival[nxt] <= now:
            waiting.append(nxt)
            nxt += 1
        if not waiting:
            now = arrival[nxt]
            continue
        if policy == FCFS:
            pick = waiting[0]
        elif policy == STATIC:
            pick = min(waiting, key=lambda i: (cls[i], i))
        else:
            pick = min(waiting, key=lambda i: (score(cls[i], now - arrival[i], reg), i))
        waiting.remove(pick)
        start[pick] = now
        now += service[pick]
        done += 1
    return start
