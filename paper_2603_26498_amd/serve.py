"""Replay of an arrival trace against the vision stages on the GPU, with the scheduling
front-end deciding which requests enter the next encoder batch.

This joins the pieces: the Impact Estimator's fitted lines give every arriving request an
estimated stage time, the Request Classifier puts it into one of the three queues, and each
time the GPU is free the Queue Manager / Priority Regulator (Sec. 3.5, 3.6) hand out requests
until a token budget is filled; the batch then runs preprocess + encode + merge/project as one
plan.  Text requests need nothing from the vision stages and leave as soon as they are
scheduled.  Measured per request: waiting time (arrival -> start of its batch) and time in the
stage (arrival -> batch finished), in real time on the device.

    python -m paper_2603_26498_amd.serve [--requests N] [--utilisation U] [--budget TOKENS] [--out FILE]

Inputs are synthetic (seeded); request sizes follow the mixed workload.  Frames are shared
between requests of equal size (pixel values do not change the timing).
"""
from __future__ import annotations

import argparse
import sys
import time

import numpy as np

import workloads

from . import profiler as P
from . import sched_binding as T

TEXT, IMAGE, VIDEO = 0, 1, 2


def make_requests(rng, n, mix=(200, 24, 2)):
    """Modality and size of n requests: images with sides from 28*{8..24}, videos of 8..32 frames at 448x448."""
    p = np.asarray(mix, float) / sum(mix)
    mod = rng.choice(3, n, p=p)
    reqs = []
    for m in mod:
        if m == TEXT:
            reqs.append((TEXT, 0, 0, 0))
        elif m == IMAGE:
            reqs.append((IMAGE, 1, int(rng.integers(8, 25)) * 28, int(rng.integers(8, 25)) * 28))
        else:
            reqs.append((VIDEO, int(rng.integers(4, 17)) * 2, 448, 448))
    return reqs


def tokens_of(req):
    m, f, h, w = req
    if m == TEXT:
        return 0
    return (1 if f == 1 else f // 2) * (h // 14) * (w // 14)


class FramePool:
    """One device tensor per (frames, h, w): uploaded once, shared by all requests of that size."""

    def __init__(self, device):
        self.device, self.pool = device, {}

    def get(self, f, h, w):
        import torch
        key = (f, h, w)
        if key not in self.pool:
            g = torch.Generator(device="cpu")
            g.manual_seed(f * 1000003 + h * 1009 + w)
            self.pool[key] = torch.randint(0, 256, (f, h, w, 3), generator=g, dtype=torch.uint8).to(self.device)
        return self.pool[key]


def run_batch(enc, pool, batch):
    """batch: list of requests (modality, frames, h, w) -> one plan, three stage calls, synchronised."""
    import torch
    from . import binding as B
    rows, keep = [], []
    for (m, f, h, w) in batch:
        t = pool.get(f, h, w)
        keep.append(t)
        rows.append((m, f, h, w, h, w, t.data_ptr()))
    from .runtime import Plan
    plan = Plan(enc, rows, keep)
    out = enc.run(plan)
    torch.cuda.synchronize()
    plan.close()
    return out


def replay(enc, pool, reqs, arrival, cls, policy, budget):
    """Real-time replay.  Returns (start, finish) per request, in seconds from the start of the replay."""
    reg = T.tcms_regulator_default()
    q = T.tcms_queues_create(reg, policy)
    n = len(reqs)
    start, finish = np.zeros(n), np.zeros(n)
    nxt = done = 0
    t0 = time.perf_counter()
    now = lambda: time.perf_counter() - t0
    waiting = 0
    while done < n:
        t = now()
        while nxt < n and arrival[nxt] <= t:
            T.tcms_queues_push(q, nxt, int(cls[nxt]), float(arrival[nxt]))
            nxt += 1
            waiting += 1
        if waiting == 0:
            # nothing to do until the next arrival
            while now() < arrival[nxt]:
                pass
            continue
        batch, ids, tok = [], [], 0
        t = now()
        while waiting:
            got = T.tcms_queues_pop(q, t)
            rid = got[0]
            waiting -= 1
            start[rid] = t
            if reqs[rid][0] == TEXT:
                finish[rid] = t
                done += 1
                continue
            batch.append(reqs[rid])
            ids.append(rid)
            tok += tokens_of(reqs[rid])
            if tok >= budget:
                break
        if batch:
            run_batch(enc, pool, batch)
            t = now()
            for rid in ids:
                finish[rid] = t
            done += len(ids)
    T.tcms_queues_destroy(q)
    return start, finish


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--requests", type=int, default=3000)
    ap.add_argument("--utilisation", type=float, default=0.8)
    ap.add_argument("--budget", type=int, default=16384, help="visual tokens per encoder batch")
    ap.add_argument("--layers", type=int, default=None)
    ap.add_argument("--out", default=None)
    args = ap.parse_args()
    import torch
    from .runtime import VisionEncoder
    if not torch.cuda.is_available():
        print("serve: no GPU visible; the vision path has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    wl = workloads.full_config(4, with_frames=False, layers=args.layers)
    enc = VisionEncoder(wl.desc, wl.weights)
    pool = FramePool("cuda:0")
    rng = np.random.default_rng(21)
    reqs = make_requests(rng, args.requests)
    toks = np.array([tokens_of(r) for r in reqs], float)
    mod = np.array([r[0] for r in reqs])

    # Workload Profiler + Impact Estimator on a size sweep of the same kinds of request
    sweep = []
    srng = np.random.default_rng(22)
    for _ in range(24):
        h, w = int(srng.integers(8, 25)) * 28, int(srng.integers(8, 25)) * 28
        sweep.append(workloads.Item(IMAGE, 1, h, w, h, w, workloads.random_frames(srng, 1, h, w)))
    for f in (8, 12, 16, 20, 24, 28, 32):
        sweep.append(workloads.Item(VIDEO, f, 448, 448, 448, 448, workloads.random_frames(srng, f, 448, 448)))
    recs = P.profile_requests(enc, sweep, reps=3)
    models = P.fit_impact_estimator(recs)
    est_ms = np.array([P.predict(models, int(m), t) for m, t in zip(mod, toks)])
    cm = P.fit_classifier(models, recs)
    smart = np.array([T.tcms_cluster_assign(cm, a, b) for a, b in zip(est_ms, toks)], np.int32)
    naive = np.array([T.tcms_classify_naive(int(m)) for m in mod], np.int32)

    # batched service is cheaper than the per-request estimate; calibrate the rate on a short FCFS burst
    burst = [r for r in reqs[:400] if r[0] != TEXT]
    for r in burst:
        pool.get(r[1], r[2], r[3])
    t0 = time.perf_counter()
    i = 0
    while i < len(burst):
        b, tok = [], 0
        while i < len(burst) and tok < args.budget:
            b.append(burst[i]); tok += tokens_of(burst[i]); i += 1
        run_batch(enc, pool, b)
    busy = time.perf_counter() - t0
    per_request = busy / 400.0                     # seconds of GPU per arriving request (text included)
    rate = args.utilisation / per_request
    for r in reqs:
        if r[0] != TEXT:
            pool.get(r[1], r[2], r[3])
    arrival = np.cumsum(np.random.default_rng(23).exponential(1.0 / rate, args.requests))

    lines = ["Replay of a Poisson arrival trace against the vision stages on the GPU (preprocess + encode + merge/project),",
             f"encoder: {wl.desc.layers} layers, d={wl.desc.d}; {args.requests} requests, text : image : video = 200 : 24 : 2,",
             f"images 224..672 px per side, videos 8..32 frames at 448x448; token budget per batch {args.budget};",
             f"arrival rate {rate:.1f} requests/s = {args.utilisation:.2f} of the measured batched capacity "
             f"({per_request * 1e3:.3f} ms of GPU per arriving request).",
             "command: python -m paper_2603_26498_amd.serve" + (f" --layers {args.layers}" if args.layers is not None else ""),
             f"classes (motorcycle, car, truck): modality rule {np.bincount(naive, minlength=3).tolist()}, clustering "
             f"{np.bincount(smart, minlength=3).tolist()}",
             "",
             "policy/classifier     wait in ms: text mean / P90 / max        image mean / P90 / max        video mean / P90 / max     makespan s"]
    for label, policy, cls in (("FCFS", T.TCMS_FCFS, naive), ("static/naive", T.TCMS_STATIC, naive),
                               ("static/smart", T.TCMS_STATIC, smart), ("regulated/smart", T.TCMS_REGULATED, smart)):
        start, finish = replay(enc, pool, reqs, arrival, cls, policy, args.budget)
        wait = (start - arrival) * 1e3
        f = lambda w: f"{w.mean():9.2f} {np.percentile(w, 90):9.2f} {w.max():9.2f}" if len(w) else " " * 29
        lines.append(f"{label:18s}  {f(wait[mod == TEXT])}   {f(wait[mod == IMAGE])}   {f(wait[mod == VIDEO])}   {finish.max():8.2f}")
        print(lines[-1], flush=True)
    text = "\n".join(lines) + "\n"
    print(text)
    if args.out:
        with open(args.out, "w") as fh:
            fh.write(text)


if __name__ == "__main__":
    main()
