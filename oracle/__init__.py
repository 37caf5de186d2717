"""CPU reference ("oracle") for the vision preprocess + ViT-encode path.

TEST INFRASTRUCTURE ONLY.  Plain, slow numpy code that defines the expected
result of every stage; it shares no code with the GPU library and must never be
imported by it.  Only tests, the smoke check and the benchmark's CPU-baseline
leg use it.
"""
from __future__ import annotations

import numpy as np

from . import preprocess, encoder, naive  # noqa: F401


def run(workload, dtype=np.float64, stages=("preprocess", "encode", "merge"), progress=None, workers=1):
    """Run the whole path for a workload (see workloads.Workload).

    Returns a dict with 'patches' (list per request), 'cu_seqlens', 'hidden'
    ([T, d]) and, when the model has a projector, 'out' ([T/merge^2, out_dim])."""
    desc, items, w = workload.desc, workload.items, workload.weights
    res = {}
    grids = encoder.grids_of(items, desc)
    res["grids"] = grids
    res["cu_seqlens"] = encoder.cu_seqlens_of(grids, desc.use_cls)
    res["patches"] = [preprocess.preprocess_item(it, desc) for it in items]
    if "encode" in stages:
        res["hidden"] = encoder.encode(res["patches"], grids, desc, w, dtype, progress, workers)
        if "merge" in stages and desc.out_dim:
            res["out"] = encoder.merge_project(res["hidden"], desc, w, dtype)
    return res
