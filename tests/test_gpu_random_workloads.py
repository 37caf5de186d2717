"""Randomised differential test: encoder descriptions drawn from every family the library has (CLS + learned
positions in bf16 and fp32, temporal patch + 2x2 merge + separable positions, windows + rotary + RMSNorm + gated MLP,
merge-free rotary, head size 72 / odd mlp widths reached by padding, no positions at all) with random widths, head
sizes, depths and normalisation constants, and request lists with text, stills and videos at native and resampled
sizes.  Every case goes through the three stages on the GPU and is compared with the CPU reference as in
test_gpu_e2e.py: patches bit for bit, hidden states and projector output per token."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from workloads import IMAGE, TEXT, VIDEO, Item, ModelDesc, Workload, make_weights, random_frames
from paper_2603_26498_amd.runtime import VisionEncoder
from util import assert_tokens_close

pytestmark = pytest.mark.gpu

HEADS_FOR = {32: [2, 4], 64: [1, 2, 3, 4], 80: [4], 96: [2, 4]}     # bf16: heads * head size is a multiple of 64


def random_case(seed):
    rng = np.random.default_rng(seed)
    fam = int(rng.integers(0, 6))
    layers = int(rng.integers(1, 4))
    kw = {}
    if rng.integers(0, 3) == 0:
        kw = {"mean": tuple(float(np.float32(x)) for x in rng.uniform(0.3, 0.6, 3)),
              "std": tuple(float(np.float32(x)) for x in rng.uniform(0.2, 0.5, 3))}
    if fam == 0:
        if rng.integers(0, 2):
            dtype, dh = "bf16", int(rng.choice([32, 64]))
            heads, mlp = int(rng.choice(HEADS_FOR[dh])), 64 * int(rng.integers(1, 9))
        else:
            dtype, dh = "f32", int(rng.choice([16, 32, 48, 64, 128]))
            heads, mlp = int(rng.integers(1, 5)), 32 * int(rng.integers(1, 12))
        desc = ModelDesc(dtype=dtype, layers=layers, d=dh * heads, heads=heads, mlp=mlp, patch=int(rng.choice([14, 16])),
                         tpatch=1, merge=1, use_cls=int(rng.integers(0, 2)), pos="learned1d", max_pos=0,
                         final_ln=int(rng.integers(0, 2)), **kw)
    elif fam in (1, 2):
        dh = int(rng.choice([32, 64, 80, 96]))
        heads = int(rng.choice(HEADS_FOR[dh]))
        mlp, out_dim = 64 * int(rng.integers(1, 10)), 8 * int(rng.integers(1, 40))
        if fam == 1:
            desc = ModelDesc(dtype="bf16", layers=layers, d=dh * heads, heads=heads, mlp=mlp, patch=14, tpatch=2, merge=2,
                             out_dim=out_dim, pos="sep2d", max_pos=40, **kw)
        else:
            desc = ModelDesc(dtype="bf16", layers=layers + 1, d=dh * heads, heads=heads, mlp=mlp, patch=14, tpatch=2,
                             merge=2, out_dim=out_dim, pos="rope2d", norm="rms", gated=1,
                             window=int(rng.choice([2, 4, 6, 8])), full_every=int(rng.integers(0, 4)), **kw)
    elif fam == 3:
        dh = int(rng.choice([32, 64, 96]))
        heads = 2 if dh != 64 else int(rng.integers(1, 5))
        desc = ModelDesc(dtype="bf16", layers=layers, d=dh * heads, heads=heads, mlp=64 * int(rng.integers(1, 9)), patch=16,
                         tpatch=1, merge=1, out_dim=8 * int(rng.integers(1, 40)), pos="rope2d", norm="rms", gated=1, **kw)
    elif fam == 4:
        desc = ModelDesc(dtype="bf16", layers=layers, d=576, heads=8, mlp=8 * int(rng.integers(5, 60)), patch=14, tpatch=1,
                         merge=1, pos="learned1d", max_pos=0, final_ln=1, **kw)
    else:
        desc = ModelDesc(dtype="bf16", layers=layers, d=64 * int(rng.integers(1, 4)), heads=1, mlp=64 * int(rng.integers(1, 9)),
                         patch=int(rng.choice([8, 14])), tpatch=int(rng.choice([1, 2])), merge=2,
                         out_dim=8 * int(rng.integers(1, 30)), pos="none", **kw)
        desc.heads = desc.d // 64
    step = desc.patch * desc.merge
    big = int(rng.integers(0, 4)) == 0
    gmax, cap = (40 if big else 20) // desc.merge, (7000 if big else 2200)
    items, tokens, longest = [], 0, 0
    for _ in range(int(rng.integers(1, 13 if big else 7))):
        kind = int(rng.integers(0, 10))
        if kind == 0:
            items.append(Item(TEXT, 0, 0, 0, 0, 0, None))
            continue
        video = kind >= 8 and not desc.use_cls
        n = desc.tpatch * int(rng.integers(1, 4)) if video else 1
        gh, gw = int(rng.integers(1, gmax + 1)), int(rng.integers(1, gmax + 1))
        t = (gh * desc.merge) * (gw * desc.merge) * max(1, (n + desc.tpatch - 1) // desc.tpatch)
        if tokens + t > cap:
            continue
        sh, sw = (gh * step, gw * step) if rng.integers(0, 2) else (int(rng.integers(3, 400)), int(rng.integers(3, 400)))
        items.append(Item(VIDEO if video else IMAGE, n, sh, sw, gh * step, gw * step, random_frames(rng, n, sh, sw)))
        tokens, longest = tokens + t, max(longest, t + desc.use_cls)
    if desc.pos == "learned1d":
        desc.max_pos = max(longest, 1) + int(rng.integers(0, 5))
    wl = Workload(f"random{seed}", desc, items)
    wl.weights = make_weights(desc, 5000 + seed, random_affine=bool(rng.integers(0, 2)))
    return wl


@pytest.mark.parametrize("first", [0, 40, 80, 120, 160])
def test_random_descriptions_and_request_lists(first):
    for seed in range(first, first + 40):
        wl = random_case(seed)
        d = wl.desc
        tag = (f"seed {seed}: {d.dtype} L{d.layers} d{d.d} h{d.heads} mlp{d.mlp} p{d.patch} tp{d.tpatch} m{d.merge} out{d.out_dim} "
               f"cls{d.use_cls} {d.pos} win{d.window}/{d.full_every} "
               f"items {[(i.modality, i.n_frames, i.src_h, i.src_w, i.dst_h, i.dst_w) for i in wl.items]}")
        ref = oracle.run(wl)
        enc = VisionEncoder(d, wl.weights)
        pl = enc.plan(wl.items)
        patches = enc.preprocess(pl)
        hidden = enc.encode(pl, patches)
        out = enc.merge_project(pl, hidden) if d.out_dim else None
        torch.cuda.synchronize()
        assert pl.cu_seqlens == ref["cu_seqlens"].tolist(), tag
        got = patches.float().cpu().numpy()
        exp = np.concatenate(ref["patches"], 0) if got.shape[0] else np.zeros((0, d.k), np.float32)
        assert got.shape[0] == exp.shape[0], tag
        assert np.array_equal(got[:, :d.k].view(np.uint32), exp.view(np.uint32)), "patches differ: " + tag
        assert not got[:, d.k:].any(), "padding columns: " + tag
        rel, cos = (1e-4, 0.999999) if d.dtype == "f32" else (2e-2, 0.999)
        if hidden.shape[0]:
            assert_tokens_close(hidden.cpu().numpy(), ref["hidden"], rel, cos, "hidden, " + tag)
            if out is not None:
                assert_tokens_close(out.float().cpu().numpy(), ref["out"], rel, cos, "out, " + tag)
