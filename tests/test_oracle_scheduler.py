"""Pins for oracle/scheduler.py: what the paper and the mathematics fix."""
import itertools
import math
import os

import numpy as np
import pytest

from oracle import scheduler as S

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    out = []
    for line in open(os.path.join(GOLD, name)):
        line = line.split("#")[0].split()
        if line:
            out.append(line)
    return out


# ---- Impact Estimator ------------------------------------------------------------------------
def test_least_squares_against_polyfit_and_exact_line():
    rng = np.random.default_rng(0)
    x = rng.uniform(0, 5000, 200)
    y = 3.0 + 0.02 * x + rng.normal(0, 1.0, 200)
    s, i = S.fit_linear(x, y)
    ps, pi = np.polyfit(x, y, 1)
    assert abs(s - ps) < 1e-12 and abs(i - pi) < 1e-9
    s, i = S.fit_linear(x, 7.0 - 0.5 * x)
    assert abs(s + 0.5) < 1e-12 and abs(i - 7.0) < 1e-9
    assert S.fit_linear([2.0, 2.0, 2.0], [1.0, 2.0, 6.0]) == (0.0, 3.0)


def _best_line_through_two_points(x, y, q):
    best = math.inf
    for a, b in itertools.combinations(range(len(x)), 2):
        if x[a] == x[b]:
            continue
        s = (y[b] - y[a]) / (x[b] - x[a])
        best = min(best, S.pinball_loss(x, y, q, s, y[a] - s * x[a]))
    return best


@pytest.mark.parametrize("q", [0.5, 0.9, 0.25])
def test_quantile_regression_against_vertex_enumeration(q):
    """A linear program attains its optimum at a vertex: a line through two data points."""
    rng = np.random.default_rng(1)
    for n in (3, 8, 25):
        x = rng.uniform(0, 100, n)
        y = 1.0 + 0.3 * x + rng.gamma(2.0, 3.0, n)
        s, i, loss = S.fit_quantile(x, y, q)
        assert abs(loss - _best_line_through_two_points(x, y, q)) <= 1e-8 * max(1.0, loss)
        assert abs(loss - S.pinball_loss(x, y, q, s, i)) <= 1e-12 * max(1.0, loss)


def test_quantile_regression_residual_counts_and_constant_x():
    rng = np.random.default_rng(2)
    x = rng.uniform(0, 8000, 300)
    y = 5.0 + 0.01 * x + rng.gamma(2.0, 2.0, 300)
    for q in (0.9, 0.5):
        s, i, _ = S.fit_quantile(x, y, q)
        r = y - (i + s * x)
        tol = 1e-7
        assert (r < -tol).sum() <= q * len(x) + 1e-9 <= (r <= tol).sum() + 1e-9
    # P90 line lies above the least-squares line over the data range: it must not underestimate (Sec. 3.3)
    s9, i9, _ = S.fit_quantile(x, y, 0.9)
    sl, il = S.fit_linear(x, y)
    assert i9 + s9 * x.mean() > il + sl * x.mean()
    # all x equal: only the level matters and the best level is a sample quantile
    yy = np.array([1.0, 2.0, 3.0, 4.0, 10.0])
    _, _, loss = S.fit_quantile(np.full(5, 3.0), yy, 0.5)
    assert abs(loss - np.abs(yy - 3.0).sum() * 0.5) < 1e-9
    assert S.pinball_loss([0, 0], [1.0, -1.0], 0.9, 0.0, 0.0) == pytest.approx(0.9 + 0.1)


def test_two_regressor_least_squares_against_normal_equations_and_exact_plane():
    rng = np.random.default_rng(3)
    t = rng.uniform(100, 33000, 60)
    x2 = t ** 2                                         # what a one-segment request has: (sum of) squared length
    y = 0.4 + 3e-3 * t + 2e-9 * x2 + rng.normal(0, 0.05, 60)
    c = S.fit_linear2(t, x2, y)
    a = np.stack([np.ones_like(t), t / 1e4, x2 / 1e8], 1)            # textbook normal equations, columns rescaled
    ref = np.linalg.solve(a.T @ a, a.T @ y) / np.array([1.0, 1e4, 1e8])
    assert np.allclose(c, ref, rtol=1e-7, atol=1e-12)
    c = S.fit_linear2(t, x2, 7.0 - 0.5 * t + 1e-6 * x2)
    assert np.allclose(c, (7.0, -0.5, 1e-6), rtol=1e-8)
    # a regressor without information gets no weight: the fit is the one-regressor fit
    s1, i1 = S.fit_linear(t, y)
    assert np.allclose(S.fit_linear2(t, np.full(60, 5.0), y), (i1, s1, 0.0), rtol=1e-9, atol=1e-12)
    # proportional regressors share the slope so that predictions equal the one-regressor fit
    c = S.fit_linear2(t, 3.0 * t, y)
    assert np.allclose(c[0] + c[1] * t + c[2] * 3.0 * t, i1 + s1 * t, rtol=1e-9)


def _best_plane_through_three_points(x1, x2, y, q):
    best = math.inf
    for tri in itertools.combinations(range(len(y)), 3):
        a = np.stack([np.ones(3), x1[list(tri)], x2[list(tri)]], 1)
        if abs(np.linalg.det(a)) < 1e-9:
            continue
        best = min(best, S.pinball_loss2(x1, x2, y, q, np.linalg.solve(a, y[list(tri)])))
    return best


@pytest.mark.parametrize("q", [0.5, 0.9])
def test_two_regressor_quantile_regression_against_vertex_enumeration(q):
    """With three free coefficients a vertex of the linear program is a plane through three data points."""
    rng = np.random.default_rng(4)
    for n in (4, 9, 16):
        x1 = rng.uniform(0, 10, n)
        x2 = x1 ** 2 + rng.uniform(0, 5, n)
        y = 1.0 + 0.3 * x1 + 0.05 * x2 + rng.gamma(2.0, 1.0, n)
        c, loss = S.fit_quantile2(x1, x2, y, q)
        assert abs(loss - _best_plane_through_three_points(x1, x2, y, q)) <= 1e-8 * max(1.0, loss)
        assert abs(loss - S.pinball_loss2(x1, x2, y, q, c)) <= 1e-12 * max(1.0, loss)
        # never worse than the best line in x1 alone, equal to it when the second regressor is constant
        _, _, loss1 = S.fit_quantile(x1, y, q)
        assert loss <= loss1 + 1e-9
        assert S.fit_quantile2(x1, np.full(n, 2.0), y, q)[1] == pytest.approx(loss1, rel=1e-8, abs=1e-10)


def test_two_regressor_quantile_regression_residual_counts_at_request_scale():
    rng = np.random.default_rng(5)
    t = rng.uniform(256, 33000, 120)
    y = 0.5 + 4e-3 * t + 1.2e-7 * t ** 2 * (1 + 0.05 * rng.random(120))
    c, _ = S.fit_quantile2(t, t ** 2, y, 0.9)
    r = y - (c[0] + c[1] * t + c[2] * t ** 2)
    assert (r < -1e-7).sum() <= 0.9 * 120 + 1e-9 <= (r <= 1e-7).sum() + 1e-9
    assert np.abs(r).max() < 0.05 * y.max()             # the square term is followed, a line would miss by far more
    s, i, _ = S.fit_quantile(t, y, 0.9)
    assert np.abs(y - (i + s * t)).max() > 4 * np.abs(r).max()


# ---- Request Classifier ----------------------------------------------------------------------
def test_naive_classifier_follows_modality():
    assert [S.classify_naive(m) for m in (0, 1, 2)] == [S.MOTORCYCLE, S.CAR, S.TRUCK]


def _kmeans_cost(z, labels):
    return sum(((z[labels == j] - z[labels == j].mean(axis=0)) ** 2).sum() for j in set(labels.tolist()))


def test_clustering_recovers_separated_groups_and_matches_the_best_partition():
    rng = np.random.default_rng(3)
    groups = [(2.0, 30), (40.0, 700), (900.0, 16000)]          # (time, tokens) scales: text, image, video
    feats, truth = [], []
    for j, (t, k) in enumerate(groups):
        for _ in range(7):
            feats.append((t * rng.uniform(0.8, 1.25), k * rng.uniform(0.8, 1.25)))
            truth.append(j)
    perm = rng.permutation(len(feats))
    feats, truth = np.asarray(feats)[perm], np.asarray(truth)[perm]
    model = S.cluster_fit(feats)
    got = np.array([S.cluster_assign(model, *f) for f in feats])
    assert np.array_equal(got, truth)
    assert np.all(np.diff(model["centroid"][:, 0]) > 0)
    # exhaustive check on a small one-dimensional-ish input: no 3-partition has a lower cost
    small = feats[:9]
    z = (np.log1p(small) - np.log1p(small).mean(0)) / np.log1p(small).std(0)
    m = S.cluster_fit(small)
    lab = np.array([S.cluster_assign(m, *f) for f in small])
    best = min(_kmeans_cost(z, np.array(l)) for l in itertools.product(range(3), repeat=9) if len(set(l)) == 3)
    assert _kmeans_cost(z, lab) <= best + 1e-9


def test_long_text_and_short_video_can_change_class():
    """Sec. 3.4: resource-aware features let a very long text leave the motorcycles and a short video join
    the cars, which the modality rule cannot do."""
    rng = np.random.default_rng(4)
    feats = np.concatenate([np.c_[rng.uniform(1, 4, 40), rng.uniform(20, 200, 40)],
                            np.c_[rng.uniform(30, 60, 40), rng.uniform(500, 1500, 40)],
                            np.c_[rng.uniform(600, 1500, 40), rng.uniform(10000, 30000, 40)]])
    m = S.cluster_fit(feats)
    assert S.cluster_assign(m, 45.0, 1000.0) == S.CAR          # a short video with an image-like footprint
    assert S.cluster_assign(m, 2.0, 50.0) == S.MOTORCYCLE
    assert S.cluster_assign(m, 1000.0, 20000.0) == S.TRUCK


# ---- Priority Regulator ----------------------------------------------------------------------
def test_regulator_constants_are_the_papers():
    rows = _rows("priority_regulator.txt")
    for c, row in enumerate(rows):
        assert float(row[1]) == S.PAPER_REGULATOR["static"][c]
        assert float(row[2]) == S.PAPER_REGULATOR["k"][c]
        assert float(row[3]) == S.PAPER_REGULATOR["p"][c]


def test_regulator_closed_forms():
    for c in (0, 1, 2):
        st, k, p = (S.PAPER_REGULATOR[n][c] for n in ("static", "k", "p"))
        assert S.priority(c, 0.0) == st                                  # no age yet
        assert S.priority(c, 1e9) == pytest.approx(st + 1.0, abs=1e-12)  # age term saturates at 1
        half = (math.log(2.0) / k) ** (1.0 / p)                          # k * w^p = ln 2  ->  age term 1/2
        assert S.priority(c, half) == pytest.approx(st + 0.5, rel=1e-12)
        w = np.linspace(0, 200, 400)
        pr = np.array([S.priority(c, x) for x in w])
        assert np.all(np.diff(pr) >= 0)
        assert S.score(c, half) == pytest.approx(-math.log(st + 0.5), rel=1e-12)
        # independent evaluation of the same formula
        assert S.priority(c, 7.0) == pytest.approx(st - math.expm1(-k * math.exp(p * math.log(7.0))), rel=1e-12)
    assert S.score(S.TRUCK, 0.0) == math.inf
    assert S.score(S.MOTORCYCLE, 0.0) == pytest.approx(-math.log(0.1))


def test_regulator_ordering_described_by_the_paper():
    """Sec. 3.6: motorcycles gain priority rapidly, cars gradually, trucks very slowly; the waits at which the
    age term reaches one half are about 2 s, 9 s and 8 minutes."""
    half = [(math.log(2.0) / S.PAPER_REGULATOR["k"][c]) ** (1.0 / S.PAPER_REGULATOR["p"][c]) for c in range(3)]
    assert 2.0 < half[0] < 2.3 and 8.5 < half[1] < 9.0 and 480 < half[2] < 520
    for w in (0.0, 0.5, 1.0, 3.0, 10.0, 60.0):
        pr = [S.priority(c, w) for c in range(3)]
        assert pr[0] >= pr[1] >= pr[2]
    # a truck that has waited long enough overtakes a fresh motorcycle: no starvation
    assert S.score(S.TRUCK, 600.0) < S.score(S.MOTORCYCLE, 0.0)


# ---- one server ------------------------------------------------------------------------------
def test_hand_worked_trace():
    rows = [[float(v) for v in r] for r in _rows("server_trace.txt")]
    arr, svc, cls = [r[0] for r in rows], [r[1] for r in rows], [int(r[2]) for r in rows]
    for col, policy in ((3, S.FCFS), (4, S.STATIC), (5, S.REGULATED)):
        assert S.simulate(policy, arr, svc, cls) == [r[col] for r in rows]


def test_fcfs_mean_wait_matches_pollaczek_khinchine():
    """M/D/1: mean wait = lambda * s^2 / (2 * (1 - lambda * s))."""
    rng = np.random.default_rng(5)
    lam, s, n = 2.0, 0.3, 60000
    arr = np.cumsum(rng.exponential(1.0 / lam, n)).tolist()
    start = S.simulate(S.FCFS, arr, [s] * n, [0] * n)
    wait = np.mean(np.asarray(start) - np.asarray(arr))
    assert wait == pytest.approx(lam * s * s / (2 * (1 - lam * s)), rel=0.05)


def test_policies_conserve_work_and_agree_on_a_single_class():
    rng = np.random.default_rng(6)
    n = 400
    arr = np.cumsum(rng.exponential(0.5, n)).tolist()
    svc = rng.choice([0.01, 0.2, 1.5], n, p=[0.7, 0.2, 0.1]).tolist()
    cls = [{0.01: 0, 0.2: 1, 1.5: 2}[v] for v in svc]
    ends = []
    for policy in (S.FCFS, S.STATIC, S.REGULATED):
        st = S.simulate(policy, arr, svc, cls)
        assert all(a <= b for a, b in zip(arr, st))
        iv = sorted(zip(st, svc))
        assert all(iv[i][0] + iv[i][1] <= iv[i + 1][0] + 1e-12 for i in range(n - 1))     # one request at a time
        ends.append(max(a + b for a, b in zip(st, svc)))
    assert ends[0] == pytest.approx(ends[1]) == pytest.approx(ends[2])                     # same busy periods
    one = [1] * n
    assert S.simulate(S.FCFS, arr, svc, one) == S.simulate(S.STATIC, arr, svc, one) == S.simulate(S.REGULATED, arr, svc, one)
    # static priority: no car or truck is started while a motorcycle is waiting
    st = S.simulate(S.STATIC, arr, svc, cls)
    for i in range(n):
        if cls[i] == 0:
            assert not any(cls[j] > 0 and arr[i] <= st[j] < st[i] for j in range(n)), i
