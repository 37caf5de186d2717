"""Workload Profiler and Impact Estimator on this library's own encoder, and a policy
comparison on a synthetic arrival trace.

The paper's Workload Profiler (Sec. 3.2) runs requests of increasing size one at a time and
records, per request, the preprocessing time, the encoder time and the number of tokens; the
Impact Estimator (Sec. 3.3) fits simple per-modality models on those records (a linear
regression, and a quantile regression at the 90th percentile for image and video requests)
and reports the prediction error (Fig. 7).  The Request Classifier (Sec. 3.4), the Queue
Manager and the Priority Regulator (Sec. 3.5, 3.6) then order the requests.

Everything measured here runs through libtcmv.so: the GPU kernels for the records, the C++
front-end (include/tcms.h) for fits, classification and the one-server trace model.  Inputs
are synthetic (seeded): the paper's datasets only provide request sizes, and sizes are what
this sweep varies.

    python -m paper_2603_26498_amd.profiler [--layers L] [--reps R] [--out FILE]
"""
from __future__ import annotations

import argparse
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import workloads  # noqa: E402

from . import sched_binding as T  # noqa: E402

TEXT, IMAGE, VIDEO = 0, 1, 2


def sweep_items(seed=7, n_images=48, video_frames=(4, 8, 16, 24, 32, 48, 64), video_sides=(224, 336, 448)):
    """Requests of increasing size: images with both sides drawn from 28*{8..48} (the dynamic-resolution
    rule of the image workloads), videos of several lengths and resolutions."""
    rng = np.random.default_rng(seed)
    items = []
    hs = rng.integers(8, 49, n_images) * 28
    ws = rng.integers(8, 49, n_images) * 28
    for h, w in zip(hs, ws):
        items.append(workloads.Item(IMAGE, 1, int(h), int(w), int(h), int(w), workloads.random_frames(rng, 1, int(h), int(w))))
    for side in video_sides:
        for f in video_frames:
            items.append(workloads.Item(VIDEO, f, side, side, side, side, workloads.random_frames(rng, f, side, side)))
    return items


def profile_requests(enc, items, reps=3, warmup=1):
    """One request at a time (no interference): median preprocess and encode(+merge/project) time."""
    import torch
    recs = []
    for it in items:
        if it.n_frames == 0:
            recs.append({"modality": it.modality, "tokens": 0, "seg_sq": 0, "preprocess_ms": 0.0, "encode_ms": 0.0})
            continue
        plan = enc.plan([it])
        cu = plan.cu_seqlens
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
        pre, encd = [], []
        for r in range(warmup + reps):
            ev[0].record()
            patches = enc.preprocess(plan)
            ev[1].record()
            hidden = enc.encode(plan, patches)
            if enc.desc.out_dim:
                enc.merge_project(plan, hidden)
            ev[2].record()
            torch.cuda.synchronize()
            if r >= warmup:
                pre.append(ev[0].elapsed_time(ev[1]))
                encd.append(ev[1].elapsed_time(ev[2]))
        recs.append({"modality": it.modality, "tokens": int(plan.info.n_tokens), "frames": it.n_frames,
                     "seg_sq": int(sum((b - a) ** 2 for a, b in zip(cu[:-1], cu[1:]))),
                     "preprocess_ms": float(np.median(pre)), "encode_ms": float(np.median(encd))})
        plan.close()
    return recs


def _seg_sq(r):
    """Sum of the squared attention-segment lengths of a profiled request (one segment when not recorded)."""
    return float(r.get("seg_sq", r["tokens"] ** 2))


def fit_impact_estimator(recs, q=0.9, attention_term=False):
    """Per modality: least-squares and q-quantile fits of (preprocess + encode) time against the tokens of the
    request.  The paper's estimator keeps the models simple (Sec. 3.3): one regressor.  With attention_term the
    sum of the squared attention-segment lengths joins as a second regressor - the encoder's attention work grows
    with it, and for long videos it is most of the time."""
    models = {}
    for m in (IMAGE, VIDEO):
        sel = [r for r in recs if r["modality"] == m]
        if len(sel) < 2:
            continue
        x = np.array([r["tokens"] for r in sel], float)
        y = np.array([r["preprocess_ms"] + r["encode_ms"] for r in sel], float)
        if attention_term:
            x2 = np.array([_seg_sq(r) for r in sel], float)
            lin = T.tcms_fit_linear2(x, x2, y)
            qc, ql = T.tcms_fit_quantile2(x, x2, y, q)
            models[m] = {"linear": (lin[1], lin[0], lin[2]), "quantile": (qc[1], qc[0], qc[2]), "q": q,
                         "n": len(sel), "pinball": ql}
        else:
            ls, li = T.tcms_fit_linear(x, y)
            qs, qi, ql = T.tcms_fit_quantile(x, y, q)
            models[m] = {"linear": (ls, li), "quantile": (qs, qi), "q": q, "n": len(sel), "pinball": ql}
    return models


def predict(models, modality, tokens, kind="quantile", seg_sq=None):
    """Estimated stage time in ms; models hold (slope, intercept[, coefficient of the squared-segment term])."""
    if modality == TEXT or modality not in models:
        return 0.0
    c = models[modality][kind]
    t = c[1] + c[0] * tokens
    if len(c) > 2:
        t += c[2] * (tokens ** 2 if seg_sq is None else seg_sq)
    return max(0.0, t)


def estimator_report(models, recs):
    """Errors of the fitted lines on records (the quantity of the paper's estimator-accuracy figure)."""
    lines = []
    for m, name in ((IMAGE, "image"), (VIDEO, "video")):
        sel = [r for r in recs if r["modality"] == m]
        if not sel or m not in models:
            continue
        y = np.array([r["preprocess_ms"] + r["encode_ms"] for r in sel])
        for kind in ("linear", "quantile"):
            p = np.array([predict(models, m, r["tokens"], kind, _seg_sq(r)) for r in sel])
            err = p - y
            c = models[m][kind]
            sq = f", {c[2] * 1e9:8.4f} ns/token^2" if len(c) > 2 else ""
            lines.append(f"  {name:5s} {kind:8s}: slope {c[0] * 1e3:8.4f} us/token, intercept "
                         f"{c[1]:8.3f} ms{sq}; n={len(sel)}; |err| mean {np.abs(err).mean():7.3f} ms, "
                         f"max {np.abs(err).max():7.3f} ms; under-estimated {100.0 * (err < 0).mean():5.1f} % of requests; "
                         f"request times {y.min():.2f}..{y.max():.2f} ms")
    return lines


def make_trace(rng, n, rate, mix=(200, 24, 2)):
    """Arrivals are a Poisson process, as in the evaluation set-up of Sec. 4.1; modality drawn with the
    proportions text : image : video = mix; sizes as in the mixed workload (images 28*{8..48} per side,
    videos of 8..64 frames at 448x448)."""
    p = np.asarray(mix, float) / sum(mix)
    mod = rng.choice(3, n, p=p)
    arrival = np.cumsum(rng.exponential(1.0 / rate, n))
    tokens = np.zeros(n)
    for i in range(n):
        if mod[i] == IMAGE:
            tokens[i] = int(rng.integers(8, 49)) * 2 * int(rng.integers(8, 49)) * 2
        elif mod[i] == VIDEO:
            tokens[i] = int(rng.integers(4, 33)) * 1024          # frame pairs x 32x32 tokens
    return arrival, mod, tokens


def fit_classifier(models, recs, n_text=16):
    """The clustering classifier is trained on profiling data (Sec. 3.4): the estimator's outputs for the
    profiled requests, plus text requests, which need no work from the vision stages."""
    feats = [(predict(models, r["modality"], r["tokens"]), float(r["tokens"])) for r in recs if r["modality"] != TEXT]
    feats += [(0.0, 0.0)] * n_text
    return T.tcms_cluster_fit(np.asarray(feats, float))


def compare_policies(models, cm, rate, n=20000, seed=11, mix=(200, 24, 2)):
    """Waiting time in front of the encoder stage per class of request under FCFS, static priority and the
    regulated priority, with the naive and the clustering classifier.  Service time = estimated stage time
    (text requests need no encoder work); one non-preemptive server."""
    rng = np.random.default_rng(seed)
    arrival, mod, tokens = make_trace(rng, n, rate, mix)
    service = np.array([predict(models, int(m), t) for m, t in zip(mod, tokens)]) / 1e3
    reg = T.tcms_regulator_default()
    naive = np.array([T.tcms_classify_naive(int(m)) for m in mod], np.int32)
    feats = np.c_[service * 1e3, tokens]
    smart = np.array([T.tcms_cluster_assign(cm, a, b) for a, b in feats], np.int32)
    out = {"utilisation": float(service.sum() / arrival[-1]), "rate": rate, "n": n,
           "class_counts_naive": np.bincount(naive, minlength=3).tolist(),
           "class_counts_smart": np.bincount(smart, minlength=3).tolist(), "rows": []}
    for label, policy, cls in (("FCFS", T.TCMS_FCFS, naive), ("static/naive", T.TCMS_STATIC, naive),
                               ("static/smart", T.TCMS_STATIC, smart), ("regulated/naive", T.TCMS_REGULATED, naive),
                               ("regulated/smart", T.TCMS_REGULATED, smart)):
        t0 = time.perf_counter()
        start = T.tcms_simulate(reg, policy, arrival, service, cls)
        dt = time.perf_counter() - t0
        wait = (start - arrival) * 1e3
        row = {"policy": label, "sim_s": dt}
        for m, name in ((TEXT, "text"), (IMAGE, "image"), (VIDEO, "video")):
            w = wait[mod == m]
            row[name] = (float(w.mean()), float(np.percentile(w, 90)), float(w.max())) if len(w) else (0.0, 0.0, 0.0)
        out["rows"].append(row)
    return out


def policy_report(res):
    lines = [f"  rate {res['rate']:.1f} req/s, {res['n']} requests, encoder utilisation {res['utilisation']:.3f}; classes "
             f"(motorcycle, car, truck): naive {res['class_counts_naive']}, clustering {res['class_counts_smart']}",
             "  policy/classifier     wait in ms: text mean / P90 / max        image mean / P90 / max        video mean / P90 / max"]
    for r in res["rows"]:
        f = lambda t: f"{t[0]:9.2f} {t[1]:9.2f} {t[2]:9.2f}"
        lines.append(f"  {r['policy']:18s}  {f(r['text'])}   {f(r['image'])}   {f(r['video'])}")
    return lines


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--layers", type=int, default=None)
    ap.add_argument("--reps", type=int, default=3)
    ap.add_argument("--out", default=None)
    args = ap.parse_args()
    import torch
    from .runtime import VisionEncoder
    if not torch.cuda.is_available():
        print("profiler: no GPU visible; the vision path has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    wl = workloads.full_config(4, with_frames=False, layers=args.layers)
    enc = VisionEncoder(wl.desc, wl.weights)
    items = sweep_items()
    print(f"profiling {len(items)} requests one at a time ...", flush=True)
    recs = profile_requests(enc, items, reps=args.reps)
    # fit on every second request of each modality, report on the others as well
    train = [r for i, r in enumerate(recs) if i % 2 == 0]
    test = [r for i, r in enumerate(recs) if i % 2 == 1]
    models = fit_impact_estimator(train)
    lines = ["Workload profile and impact estimator of the vision stages (preprocess + encode + merge/project),",
             f"encoder: {wl.desc.layers} layers, d={wl.desc.d}, heads={wl.desc.heads}, mlp={wl.desc.mlp}, projector to {wl.desc.out_dim};",
             "MI355X, one request at a time, median of %d runs; synthetic frames." % args.reps,
             "command: python -m paper_2603_26498_amd.profiler" + (f" --layers {args.layers}" if args.layers is not None else ""),
             "", "records (modality, frames, tokens, preprocess ms, encode ms):"]
    for r in recs:
        lines.append(f"  {('text', 'image', 'video')[r['modality']]:5s} {r.get('frames', 0):3d} {r['tokens']:6d} "
                     f"{r['preprocess_ms']:8.3f} {r['encode_ms']:9.3f}")
    lines += ["", "fits on every second record, errors on the fitted records:"] + estimator_report(models, train)
    lines += ["errors on the held-out records:"] + estimator_report(models, test)
    models2 = fit_impact_estimator(train, attention_term=True)
    lines += ["", "the same with the sum of squared attention-segment lengths as a second regressor,",
              "errors on the fitted records:"] + estimator_report(models2, train)
    lines += ["errors on the held-out records:"] + estimator_report(models2, test)
    lines += ["", "policies on a Poisson trace (text : image : video = 200 : 24 : 2), service time = P90 estimate:"]
    full = fit_impact_estimator(recs)
    cm = fit_classifier(full, recs)
    probe = compare_policies(full, cm, 2.0)
    # the paper's rate, then rates that load the encoder stage to about 80 % and 95 %
    for rate in (2.0, 2.0 * 0.8 / max(probe["utilisation"], 1e-9), 2.0 * 0.95 / max(probe["utilisation"], 1e-9)):
        lines += policy_report(compare_policies(full, cm, rate))
    text = "\n".join(lines) + "\n"
    print(text)
    if args.out:
        with open(args.out, "w") as f:
            f.write(text)


if __name__ == "__main__":
    main()
