#!/usr/bin/env python3
"""Writes tests/golden/full_cfg<N>.npz: sampled rows of the CPU reference's final
output for a FULL-SIZE workload (all layers).  Calls only `oracle` and the
seeded input generators; nothing here touches the GPU library.

    python tests/golden/make_full_size_golden.py --config 4

The reference is evaluated in float32 here (a full float64 pass over 200-400
TFLOP of work is out of reach of a CPU); float32 rounding (~1e-6 relative per
operation) is three orders of magnitude below the bf16 tolerance the values are
compared at.  Takes from minutes (config 2) to about an hour (configs 3-5)."""
import argparse
import os
import sys
import time

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

import oracle  # noqa: E402
import workloads  # noqa: E402


def sample_rows(cu, n_rows_total, per_seg_div, n_random=64):
    """First, middle and last output row of EVERY segment, plus seeded random rows.

    (Files written before this rule hold 24 rows: first/last rows of the first, longest,
    shortest and last segment plus random ones.  A file records the rows it holds, so the
    test reads either kind.)"""
    rng = np.random.default_rng(12345)
    seg = [(int(a) // per_seg_div, int(b) // per_seg_div) for a, b in zip(cu[:-1], cu[1:]) if b > a]
    pick = set()
    for a, b in seg:
        pick |= {a, (a + b) // 2, b - 1}
    want = min(len(pick) + n_random, n_rows_total)
    while len(pick) < want:
        pick.add(int(rng.integers(0, n_rows_total)))
    return np.array(sorted(pick), np.int64)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, required=True, choices=[1, 2, 3, 4, 5, 6, 7, 8, 9])
    ap.add_argument("--out", default=None)
    ap.add_argument("--workers", type=int, default=1, help="threads over attention heads (arithmetic unchanged)")
    args = ap.parse_args()
    t0 = time.time()
    wl = workloads.full_config(args.config)
    print(f"[{time.time() - t0:7.1f}s] generated {wl.name}", flush=True)
    dt = np.float64 if args.config == 1 else np.float32
    res = oracle.run(wl, dtype=dt, progress=lambda l: print(f"[{time.time() - t0:7.1f}s] layer {l} done", flush=True),
                     workers=args.workers)
    m2 = wl.desc.merge ** 2 if wl.desc.out_dim else 1
    final = res["out"] if wl.desc.out_dim else res["hidden"]
    rows = sample_rows(res["cu_seqlens"], final.shape[0], m2)
    out = args.out or os.path.join(HERE, f"full_cfg{args.config}.npz")
    np.savez_compressed(out, rows=rows, values=final[rows].astype(np.float32),
                        n_rows=np.int64(final.shape[0]), cu_seqlens=res["cu_seqlens"],
                        mean_abs=np.float64(np.abs(final).mean()), workload=np.array(wl.name),
                        oracle_seconds=np.float64(time.time() - t0), oracle_dtype=np.array(np.dtype(dt).name))
    print(f"[{time.time() - t0:7.1f}s] wrote {out}: {len(rows)} rows of {final.shape}", flush=True)


if __name__ == "__main__":
    main()
