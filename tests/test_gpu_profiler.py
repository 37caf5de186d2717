"""The Workload Profiler and the Impact Estimator (Sec. 3.2, 3.3) on the device: a short sweep of requests, one at
a time, through the real preprocess / encode / project calls; the recorded sizes against the CPU reference's
segment arithmetic and the library's fits against the CPU reference's fits on the recorded points."""
import numpy as np
import pytest

import workloads
from oracle import encoder as oe
from oracle import scheduler as S
from paper_2603_26498_amd import profiler as P
from paper_2603_26498_amd.runtime import VisionEncoder

pytestmark = pytest.mark.gpu


def _sweep():
    rng = np.random.default_rng(21)
    items = []
    for h, w in ((224, 308), (448, 448), (28 * 9, 28 * 31), (28 * 40, 28 * 12)):
        items.append(workloads.Item(P.IMAGE, 1, h, w, h, w, workloads.random_frames(rng, 1, h, w)))
    for f, side in ((4, 224), (8, 224), (8, 336), (16, 448)):
        items.append(workloads.Item(P.VIDEO, f, side, side, side, side, workloads.random_frames(rng, f, side, side)))
    items.append(workloads.Item(P.TEXT, 0, 0, 0, 0, 0, None))
    return items


def test_profile_sweep_records_and_fits():
    wl = workloads.full_config(4, with_frames=False, layers=2)
    desc = wl.desc
    enc = VisionEncoder(desc, wl.weights)
    items = _sweep()
    recs = P.profile_requests(enc, items, reps=2, warmup=1)
    assert len(recs) == len(items)
    for it, r in zip(items, recs):
        assert r["modality"] == it.modality
        if it.n_frames == 0:
            assert r["tokens"] == 0 and r["preprocess_ms"] == 0.0 and r["encode_ms"] == 0.0
            continue
        # a still image fills the temporal patch by repetition; a video is cut into groups of tpatch frames
        gt = max(1, it.n_frames // desc.tpatch)
        cu = oe.cu_seqlens_of([(gt, it.dst_h // desc.patch, it.dst_w // desc.patch)], desc.use_cls)
        assert r["tokens"] == int(cu[-1])
        assert r["seg_sq"] == int((np.diff(cu) ** 2).sum())
        assert r["preprocess_ms"] > 0.0 and r["encode_ms"] > 0.0
        assert r["encode_ms"] < 2000.0
    # larger requests of one modality take longer on the device (two layers: about 0.1 .. 10 ms)
    vid = sorted((r for r in recs if r["modality"] == P.VIDEO), key=lambda r: r["tokens"])
    assert vid[-1]["encode_ms"] > vid[0]["encode_ms"]
    for attention_term in (False, True):
        models = P.fit_impact_estimator(recs, attention_term=attention_term)
        for m in (P.IMAGE, P.VIDEO):
            sel = [r for r in recs if r["modality"] == m]
            x = np.array([r["tokens"] for r in sel], float)
            x2 = np.array([r["seg_sq"] for r in sel], float)
            y = np.array([r["preprocess_ms"] + r["encode_ms"] for r in sel])
            if attention_term:
                c = S.fit_linear2(x, x2, y)
                got = models[m]["linear"]
                pred = got[1] + got[0] * x + got[2] * x2
                assert np.allclose(pred, c[0] + c[1] * x + c[2] * x2, rtol=1e-8, atol=1e-8)
                _, loss = S.fit_quantile2(x, x2, y, 0.9)
            else:
                s, i = S.fit_linear(x, y)
                assert models[m]["linear"] == pytest.approx((s, i), rel=1e-8, abs=1e-8)
                _, _, loss = S.fit_quantile(x, y, 0.9)
            assert models[m]["pinball"] == pytest.approx(loss, rel=1e-8, abs=1e-8)
            # a model fitted at the 90th percentile under-estimates at most every tenth fitted request
            p = np.array([P.predict(models, m, r["tokens"], "quantile", r["seg_sq"]) for r in sel])
            assert (y > p + 1e-9).mean() <= 0.1 + 1.0 / len(sel)
        assert P.predict(models, P.TEXT, 0) == 0.0
