"""The C++ scheduling front-end (libtcmv.so, include/tcms.h) against the CPU reference in
oracle/scheduler.py, on the same seeded inputs.  Host code only: these run without a GPU."""
import math

import numpy as np
import pytest

from oracle import scheduler as S
from paper_2603_26498_amd import sched_binding as T


def _mix(rng, n):
    """Request sizes shaped like the paper's heavy mix: mostly text, some images, few videos; features are
    (time in ms, tokens)."""
    cls = rng.choice(3, n, p=[0.6, 0.3, 0.1])
    tokens = np.where(cls == 0, rng.integers(10, 400, n),
                      np.where(cls == 1, rng.integers(256, 9217, n), rng.integers(8192, 32769, n))).astype(float)
    time = np.where(cls == 0, 0.02 * tokens, np.where(cls == 1, 0.004 * tokens, 2e-7 * tokens ** 2 + 0.003 * tokens))
    time = time * rng.uniform(0.95, 1.3, n)
    return cls, tokens, time


@pytest.mark.parametrize("n", [1, 2, 17, 400])
def test_least_squares(n):
    rng = np.random.default_rng(n)
    x = rng.uniform(0, 30000, n)
    y = 1.5 + 0.004 * x + rng.normal(0, 2, n)
    s, i = T.tcms_fit_linear(x, y)
    rs, ri = S.fit_linear(x, y)
    assert s == pytest.approx(rs, rel=1e-10, abs=1e-14) and i == pytest.approx(ri, rel=1e-9, abs=1e-9)


@pytest.mark.parametrize("q", [0.9, 0.5, 0.1])
@pytest.mark.parametrize("n", [2, 3, 10, 61, 300])
def test_quantile_regression_reaches_the_minimum_of_the_linear_program(q, n):
    rng = np.random.default_rng(100 * n + int(q * 10))
    x = rng.uniform(0, 30000, n)
    y = 2.0 + 0.004 * x + rng.gamma(2.0, 4.0, n)
    s, i, loss = T.tcms_fit_quantile(x, y, q)
    _, _, ref = S.fit_quantile(x, y, q)
    assert loss == pytest.approx(ref, rel=1e-8, abs=1e-8)                 # the minimum is unique
    assert S.pinball_loss(x, y, q, s, i) == pytest.approx(loss, rel=1e-12)   # and the returned line attains it
    assert T.tcms_pinball_loss(x, y, q, s, i) == pytest.approx(loss, rel=1e-12)
    r = y - (i + s * x)
    tol = 1e-9 * max(1.0, np.abs(y).max())
    assert (r < -tol).sum() <= q * n + 1e-9 <= (r <= tol).sum() + 1e-9


@pytest.mark.parametrize("n", [1, 2, 3, 17, 400])
def test_two_regressor_least_squares(n):
    rng = np.random.default_rng(n)
    t = rng.uniform(64, 33000, n)
    y = 1.5 + 0.004 * t + 1.1e-7 * t ** 2 + rng.normal(0, 2, n)
    for x2 in (t ** 2, np.full(n, 9.0), 3.0 * t):          # informative, constant, proportional
        c = T.tcms_fit_linear2(t, x2, y)
        ref = S.fit_linear2(t, x2, y)
        pred, pref = c[0] + c[1] * t + c[2] * x2, ref[0] + ref[1] * t + ref[2] * x2
        assert np.allclose(pred, pref, rtol=1e-8, atol=1e-8)
        if n >= 3:
            assert np.allclose(c, ref, rtol=1e-6, atol=1e-9 * max(1.0, abs(ref[0])))


@pytest.mark.parametrize("q", [0.9, 0.5])
@pytest.mark.parametrize("n", [1, 2, 3, 10, 61, 150])
def test_two_regressor_quantile_regression_reaches_the_minimum_of_the_linear_program(q, n):
    rng = np.random.default_rng(100 * n + int(q * 10))
    t = np.round(rng.uniform(64, 33000, n))
    x2 = t ** 2 if n % 2 else t ** 2 * rng.uniform(0.3, 1.0, n)       # one segment, or several per request
    y = 2.0 + 0.004 * t + 1.1e-7 * x2 + rng.gamma(2.0, 4.0, n)
    c, loss = T.tcms_fit_quantile2(t, x2, y, q)
    _, ref = S.fit_quantile2(t, x2, y, q)
    assert loss == pytest.approx(ref, rel=1e-8, abs=1e-8)
    assert S.pinball_loss2(t, x2, y, q, c) == pytest.approx(loss, rel=1e-12, abs=1e-12)
    assert T.tcms_pinball_loss2(t, x2, y, q, c) == pytest.approx(loss, rel=1e-12, abs=1e-12)
    # with a constant second regressor it is the one-regressor fit
    c1, loss1 = T.tcms_fit_quantile2(t, np.full(n, 4.0), y, q)
    assert loss1 == pytest.approx(T.tcms_fit_quantile(t, y, q)[2], rel=1e-9, abs=1e-9)
    with pytest.raises(T.TcmsError):
        T.tcms_fit_quantile2(t, x2, y, 1.0)


def test_quantile_regression_degenerate_inputs():
    y = np.array([4.0, 1.0, 3.0, 2.0, 10.0])
    for q in (0.5, 0.9, 0.2):
        s, i, loss = T.tcms_fit_quantile(np.full(5, 7.0), y, q)
        _, _, ref = S.fit_quantile(np.full(5, 7.0), y, q)
        assert s == 0.0 and loss == pytest.approx(ref, abs=1e-9)
    assert T.tcms_fit_quantile([3.0], [5.0], 0.9)[:2] == (0.0, 5.0)
    # repeated x values and exact collinearity
    x = np.array([1.0, 1.0, 2.0, 2.0, 3.0, 3.0])
    s, i, loss = T.tcms_fit_quantile(x, 2 * x + 1, 0.9)
    assert loss == pytest.approx(0.0, abs=1e-12) and s == pytest.approx(2.0) and i == pytest.approx(1.0)
    for bad in (0.0, 1.0, -0.1, float("nan")):
        with pytest.raises(T.TcmsError):
            T.tcms_fit_quantile(x, x, bad)
    with pytest.raises(T.TcmsError):
        T.tcms_fit_linear([1.0, float("inf")], [1.0, 2.0])


def test_classifiers():
    assert [T.tcms_classify_naive(m) for m in (0, 1, 2)] == [S.classify_naive(m) for m in (0, 1, 2)]
    with pytest.raises(T.TcmsError):
        T.tcms_classify_naive(3)
    for seed in range(4):
        rng = np.random.default_rng(seed)
        _, tokens, time = _mix(rng, 500)
        feats = np.c_[time, tokens]
        m = T.tcms_cluster_fit(feats)
        ref = S.cluster_fit(feats)
        assert np.allclose(np.array(m.mean[:]), ref["mean"], rtol=1e-12)
        assert np.allclose(np.array(m.scale[:]), ref["scale"], rtol=1e-12)
        cent = np.array([[m.centroid[j][0], m.centroid[j][1]] for j in range(3)])
        assert np.allclose(cent, ref["centroid"], rtol=1e-9, atol=1e-12)
        _, tk, tm = _mix(np.random.default_rng(100 + seed), 300)
        got = [T.tcms_cluster_assign(m, a, b) for a, b in zip(tm, tk)]
        exp = [S.cluster_assign(ref, a, b) for a, b in zip(tm, tk)]
        assert got == exp
        assert len(set(got)) == 3
    with pytest.raises(T.TcmsError):
        T.tcms_cluster_fit(np.ones((2, 2)))
    with pytest.raises(T.TcmsError):
        T.tcms_cluster_fit(-np.ones((5, 2)))


def test_priority_regulator_values():
    reg = T.tcms_regulator_default()
    for c in range(3):
        assert reg.static_priority[c] == S.PAPER_REGULATOR["static"][c]
        assert reg.k[c] == S.PAPER_REGULATOR["k"][c] and reg.p[c] == S.PAPER_REGULATOR["p"][c]
        for w in (0.0, 1e-3, 0.5, 1.0, 2.0, 3.0, 7.5, 10.0, 60.0, 600.0, 1e6):
            assert T.tcms_priority(reg, c, w) == pytest.approx(S.priority(c, w), rel=1e-14, abs=1e-300)
            a, b = T.tcms_score(reg, c, w), S.score(c, w)
            assert (a == b) if math.isinf(b) else a == pytest.approx(b, rel=1e-13, abs=1e-15)
    assert T.tcms_score(reg, 2, 0.0) == math.inf
    assert math.isnan(T.tcms_priority(reg, 5, 1.0))
    other = {"static": (0.3, 0.2, 0.1), "k": (0.5, 0.01, 0.002), "p": (2.0, 1.5, 1.0)}
    r2 = T.make_regulator(other["static"], other["k"], other["p"])
    for c in range(3):
        for w in (0.0, 0.7, 12.0):
            assert T.tcms_priority(r2, c, w) == pytest.approx(S.priority(c, w, other), rel=1e-14)


@pytest.mark.parametrize("policy", [S.FCFS, S.STATIC, S.REGULATED])
@pytest.mark.parametrize("seed,rate", [(0, 2.0), (1, 6.0), (2, 20.0)])
def test_server_trace_start_times(policy, seed, rate):
    rng = np.random.default_rng(seed)
    n = 600
    cls, _, time_ms = _mix(rng, n)
    arrival = np.cumsum(rng.exponential(1.0 / rate, n))
    service = time_ms / 1e3 * 3
    reg = T.tcms_regulator_default()
    got = T.tcms_simulate(reg, policy, arrival, service, cls)
    exp = np.asarray(S.simulate(policy, arrival.tolist(), service.tolist(), cls.tolist()))
    assert np.array_equal(got, exp)


def test_hand_worked_trace_and_queue_object():
    import os
    rows = [[float(v) for v in l.split("#")[0].split()] for l in
            open(os.path.join(os.path.dirname(__file__), "golden", "server_trace.txt")) if l.split("#")[0].split()]
    arr, svc, cls = [r[0] for r in rows], [r[1] for r in rows], [int(r[2]) for r in rows]
    reg = T.tcms_regulator_default()
    for col, policy in ((3, T.TCMS_FCFS), (4, T.TCMS_STATIC), (5, T.TCMS_REGULATED)):
        assert T.tcms_simulate(reg, policy, arr, svc, cls).tolist() == [r[col] for r in rows]
        # the same trace driven through the queue object by hand
        q = T.tcms_queues_create(reg, policy)
        start, now, nxt = {}, 0.0, 0
        while len(start) < len(arr):
            while nxt < len(arr) and arr[nxt] <= now:
                T.tcms_queues_push(q, nxt, cls[nxt], arr[nxt])
                nxt += 1
            got = T.tcms_queues_pop(q, now)
            if got is None:
                now = arr[nxt]
                continue
            start[got[0]] = now
            assert got[1] == cls[got[0]] and got[2] == arr[got[0]]
            now += svc[got[0]]
        assert [start[i] for i in range(len(arr))] == [r[col] for r in rows]
        assert T.tcms_queues_pop(q, now) is None
        T.tcms_queues_destroy(q)


def test_queue_metrics_and_argument_checks():
    reg = T.tcms_regulator_default()
    q = T.tcms_queues_create(reg, T.TCMS_REGULATED)
    for i, (c, a) in enumerate([(0, 0.0), (2, 1.0), (2, 2.0), (1, 2.5)]):
        T.tcms_queues_push(q, i, c, a)
    ln, mw = T.tcms_queues_stats(q, 4.0)
    assert ln == [1, 1, 2] and mw == pytest.approx([4.0, 1.5, 2.5])
    with pytest.raises(T.TcmsError):
        T.tcms_queues_push(q, 9, 2, 0.5)            # arrivals of a class must not go back in time
    with pytest.raises(T.TcmsError):
        T.tcms_queues_push(q, 9, 3, 5.0)
    T.tcms_queues_destroy(q)
    with pytest.raises(T.TcmsError):
        T.tcms_queues_create(T.make_regulator((0.1, 0.05, 0.0), (0.05, -1.0, 0.1), (1.0, 1.0, 1.0)), 0)
    with pytest.raises(T.TcmsError):
        T.tcms_simulate(reg, 0, [1.0, 0.5], [1.0, 1.0], [0, 0])
