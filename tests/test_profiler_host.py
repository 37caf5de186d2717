"""Host-side parts of the workload profiler / impact estimator / trace tools (no GPU needed): the fits,
the classifier trained on profile records and the policy comparison must agree with the CPU reference."""
import numpy as np
import pytest

from oracle import scheduler as S
from paper_2603_26498_amd import profiler as P
from paper_2603_26498_amd import sched_binding as T
from paper_2603_26498_amd import serve as V


def _records(rng):
    recs = []
    for _ in range(40):
        tok = int(rng.integers(64, 2305)) * 4
        recs.append({"modality": 1, "tokens": tok, "frames": 1, "preprocess_ms": 0.03,
                     "encode_ms": 3.0 + 0.003 * tok + rng.gamma(2.0, 0.3)})
    for f in (4, 8, 16, 24, 32, 48, 64):
        for side in (224, 448):
            tok = f // 2 * (side // 14) ** 2
            recs.append({"modality": 2, "tokens": tok, "frames": f, "preprocess_ms": 0.05,
                         "encode_ms": 2.0 + 0.004 * tok + 2e-7 * tok * tok + rng.gamma(2.0, 0.5)})
    return recs


def test_estimator_fits_match_the_reference():
    recs = _records(np.random.default_rng(0))
    models = P.fit_impact_estimator(recs)
    for m in (1, 2):
        sel = [r for r in recs if r["modality"] == m]
        x = [r["tokens"] for r in sel]
        y = [r["preprocess_ms"] + r["encode_ms"] for r in sel]
        s, i = S.fit_linear(x, y)
        assert models[m]["linear"] == pytest.approx((s, i), rel=1e-9)
        _, _, loss = S.fit_quantile(x, y, 0.9)
        qs, qi = models[m]["quantile"]
        assert S.pinball_loss(x, y, 0.9, qs, qi) == pytest.approx(loss, rel=1e-8)
        assert models[m]["pinball"] == pytest.approx(loss, rel=1e-8)
        under = np.mean(np.asarray(y) > qi + qs * np.asarray(x) + 1e-9)
        assert under <= 0.1 + 1e-9                      # the P90 line under-estimates at most 10 % of the fitted requests
    assert P.predict(models, 0, 123) == 0.0             # text needs nothing from the vision stages
    assert P.predict(models, 1, 4000) > P.predict(models, 1, 400) > 0
    assert len(P.estimator_report(models, recs)) == 4


def test_estimator_with_the_attention_term_follows_the_videos():
    recs = _records(np.random.default_rng(3))
    one = P.fit_impact_estimator(recs)
    two = P.fit_impact_estimator(recs, attention_term=True)
    sel = [r for r in recs if r["modality"] == 2]
    x = np.array([r["tokens"] for r in sel], float)
    y = np.array([r["preprocess_ms"] + r["encode_ms"] for r in sel])
    coef, loss = S.fit_quantile2(x, x ** 2, y, 0.9)
    assert two[2]["pinball"] == pytest.approx(loss, rel=1e-8)
    c = S.fit_linear2(x, x ** 2, y)
    assert two[2]["linear"] == pytest.approx((c[1], c[0], c[2]), rel=1e-6)
    e1 = np.abs([P.predict(one, 2, r["tokens"], "linear") for r in sel] - y).max()
    e2 = np.abs([P.predict(two, 2, r["tokens"], "linear", r["tokens"] ** 2) for r in sel] - y).max()
    assert e2 < 0.25 * e1                               # the records hold a square term; a line cannot follow it
    assert len(P.estimator_report(two, recs)) == 4


def test_classifier_trained_on_profile_separates_the_modalities_of_the_sweep():
    recs = _records(np.random.default_rng(1))
    models = P.fit_impact_estimator(recs)
    cm = P.fit_classifier(models, recs)
    feats = [(P.predict(models, r["modality"], r["tokens"]), float(r["tokens"])) for r in recs] + [(0.0, 0.0)] * 16
    ref = S.cluster_fit(np.asarray(feats))
    for a, b in feats:
        assert T.tcms_cluster_assign(cm, a, b) == S.cluster_assign(ref, a, b)
    assert T.tcms_cluster_assign(cm, 0.0, 0.0) == T.TCMS_MOTORCYCLE
    big = max(recs, key=lambda r: r["tokens"])
    assert T.tcms_cluster_assign(cm, P.predict(models, 2, big["tokens"]), big["tokens"]) == T.TCMS_TRUCK


def test_policy_comparison_matches_the_reference_server_loop():
    recs = _records(np.random.default_rng(2))
    models = P.fit_impact_estimator(recs)
    cm = P.fit_classifier(models, recs)
    res = P.compare_policies(models, cm, rate=150.0, n=1500, seed=5)
    # rebuild the same trace and run the reference loop
    rng = np.random.default_rng(5)
    arrival, mod, tokens = P.make_trace(rng, 1500, 150.0)
    service = np.array([P.predict(models, int(m), t) for m, t in zip(mod, tokens)]) / 1e3
    naive = [S.classify_naive(int(m)) for m in mod]
    start = np.asarray(S.simulate(S.STATIC, arrival.tolist(), service.tolist(), naive))
    wait = (start - arrival) * 1e3
    row = [r for r in res["rows"] if r["policy"] == "static/naive"][0]
    assert row["text"][0] == pytest.approx(wait[mod == 0].mean(), rel=1e-9, abs=1e-9)
    assert row["video"][2] == pytest.approx(wait[mod == 2].max(), rel=1e-9, abs=1e-9)
    assert 0.0 < res["utilisation"] < 2.0
    assert len(P.policy_report(res)) == 2 + 5


def test_trace_replay_loop_with_a_stub_device():
    """The real-time loop (serve.replay) with the device call replaced by a short sleep: every request is
    started after it arrived, finished after it started, text requests leave when scheduled."""
    import time
    rng = np.random.default_rng(3)
    reqs = V.make_requests(rng, 200)
    mod = np.array([r[0] for r in reqs])
    arrival = np.cumsum(np.random.default_rng(4).exponential(1 / 4000.0, 200))
    cls = np.array([T.tcms_classify_naive(int(m)) for m in mod], np.int32)
    orig = V.run_batch
    V.run_batch = lambda enc, pool, batch: time.sleep(1e-4 + 2e-8 * sum(V.tokens_of(r) for r in batch))
    try:
        for policy in (T.TCMS_FCFS, T.TCMS_STATIC, T.TCMS_REGULATED):
            start, finish = V.replay(None, None, reqs, arrival, cls, policy, 8192)
            assert np.all(start >= arrival - 1e-9) and np.all(finish >= start)
            assert np.all(finish[mod == 0] == start[mod == 0])
            assert np.all(finish[mod != 0] > start[mod != 0])
    finally:
        V.run_batch = orig
    assert V.tokens_of((2, 8, 448, 448)) == 4 * 32 * 32 and V.tokens_of((1, 1, 224, 336)) == 16 * 24
