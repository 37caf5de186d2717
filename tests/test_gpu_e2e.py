"""GPU parity of the three stages (through the C ABI) against the CPU
reference on reduced versions of the five workloads, plus the adversarial
end-to-end variants (non-zero biases, random gamma/beta) they are built with.

Tolerances.  Preprocessing and patch indexing: bit-exact.  fp32 model: 1e-4 of
the row maximum.  bf16 model: per token max|err|/max|ref| <= 2e-2 and cosine
>= 0.999 (the bar of the target), checked on every output row."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from paper_2603_26498_amd import binding as B
from paper_2603_26498_amd.runtime import VisionEncoder
from util import assert_tokens_close

pytestmark = pytest.mark.gpu


def run_gpu(wl):
    enc = VisionEncoder(wl.desc, wl.weights)
    pl = enc.plan(wl.items)
    patches = enc.preprocess(pl)
    hidden = enc.encode(pl, patches)
    out = enc.merge_project(pl, hidden) if wl.desc.out_dim else None
    torch.cuda.synchronize()
    return enc, pl, patches, hidden, out


def check_patches(wl, ref, patches):
    k = wl.desc.k
    got = patches.float().cpu().numpy()
    exp = np.concatenate([p for p in ref["patches"]], 0) if got.shape[0] else np.zeros((0, k), np.float32)
    assert got.shape[0] == exp.shape[0]
    assert np.array_equal(got[:, :k].view(np.uint32), exp.view(np.uint32)), "patches differ (must be bit-exact)"
    assert not got[:, k:].any(), "padding columns must be zero"


@pytest.mark.parametrize("idx", [1, 2, 3, 4, 5, 6, 7, 8, 9])
@pytest.mark.parametrize("affine", [False, True])
def test_small_workloads(idx, affine):
    wl = workloads.small_config(idx, random_affine=affine)
    ref = oracle.run(wl)
    enc, pl, patches, hidden, out = run_gpu(wl)
    assert pl.cu_seqlens == ref["cu_seqlens"].tolist()
    check_patches(wl, ref, patches)
    rel, cos = (1e-4, 0.999999) if wl.desc.dtype == "f32" else (2e-2, 0.999)
    assert_tokens_close(hidden.cpu().numpy(), ref["hidden"], rel, cos, f"small{idx} hidden")
    if out is not None:
        assert_tokens_close(out.float().cpu().numpy(), ref["out"], rel, cos, f"small{idx} out")


def test_resize_paths_bit_exact_many_sizes():
    """Up- and down-scaling, odd source sizes, several items per launch."""
    desc = workloads.ModelDesc(dtype="bf16", layers=0, d=128, heads=2, mlp=128, patch=14, tpatch=2, merge=2)
    rng = np.random.default_rng(77)
    items = []
    for (n, sh, sw, dh, dw) in [(1, 37, 53, 28, 56), (2, 240, 426, 56, 84), (1, 31, 17, 84, 140), (4, 5, 1, 28, 28),
                                (1, 1080, 1920, 224, 448), (1, 56, 56, 56, 56), (2, 100, 100, 112, 28)]:
        items.append(workloads.Item(2 if n > 1 else 1, n, sh, sw, dh, dw, workloads.random_frames(rng, n, sh, sw)))
    wl = workloads.Workload("resize", desc, items, workloads.make_weights(desc, 1))
    enc = VisionEncoder(desc, wl.weights)
    pl = enc.plan(items)
    patches = enc.preprocess(pl)
    torch.cuda.synchronize()
    ref = oracle.run(wl, stages=("preprocess",))
    check_patches(wl, ref, patches)


@pytest.mark.parametrize("dtype,patch,tpatch,merge", [("f32", 16, 1, 1), ("f32", 7, 3, 1), ("bf16", 14, 1, 1),
                                                      ("bf16", 8, 2, 2), ("f32", 14, 2, 2)])
def test_preprocess_layouts_and_general_normalisation(dtype, patch, tpatch, merge):
    mean = tuple(float(np.float32(m)) for m in (0.485, 0.456, 0.406))
    std = tuple(float(np.float32(s)) for s in (0.229, 0.224, 0.225))
    desc = workloads.ModelDesc(dtype=dtype, layers=0, d=128, heads=2, mlp=128, patch=patch, tpatch=tpatch, merge=merge,
                               mean=mean, std=std)
    rng = np.random.default_rng(5)
    pm = patch * merge
    items = [workloads.Item(1, 1, 3 * pm, 2 * pm, 3 * pm, 2 * pm, workloads.random_frames(rng, 1, 3 * pm, 2 * pm)),
             workloads.Item(0, 0, 0, 0, 0, 0, None),
             workloads.Item(2, 2 * tpatch, pm, 4 * pm, pm, 4 * pm, workloads.random_frames(rng, 2 * tpatch, pm, 4 * pm))]
    wl = workloads.Workload("layout", desc, items, workloads.make_weights(desc, 1))
    enc = VisionEncoder(desc, wl.weights)
    pl = enc.plan(items)
    patches = enc.preprocess(pl)
    torch.cuda.synchronize()
    check_patches(wl, oracle.run(wl, stages=("preprocess",)), patches)


def _fma_form_reproduces_table(mean, std):
    """Whether bf16(fma(v, 1/(255 std), -mean/std)) in fp32 equals the contract's bf16(fp32((v/255 - mean)/std)) for
    every pixel value (the product v * scale fits a double exactly, so rounding the double sum once to fp32 is the
    fused multiply-add)."""
    v = np.arange(256, dtype=np.float64)
    table = workloads.snap_to_bf16_grid(((v / 255.0 - mean) / std).astype(np.float32))
    sc, of = np.float32(1.0 / (255.0 * std)), np.float32(-mean / std)
    return np.array_equal(table, workloads.snap_to_bf16_grid((v * np.float64(sc) + np.float64(of)).astype(np.float32)))


@pytest.mark.parametrize("first_channel,computed", [((0.5, 0.5), True), ((0.3121532201766968, 0.4928024709224701), False)])
def test_bf16_normalisation_computed_or_looked_up_is_the_table(first_channel, computed):
    """The bf16 strip kernel computes the normalised value with one fused multiply-add where that gives the table's
    768 values, and looks it up where it does not (here: one entry of the first channel differs).  Either way the
    patches are the reference's, bit for bit; copied and resampled strips, a video and still images."""
    mean = (first_channel[0], float(np.float32(0.456)), float(np.float32(0.406)))
    std = (first_channel[1], float(np.float32(0.224)), float(np.float32(0.225)))
    assert all(_fma_form_reproduces_table(m, s) for m, s in zip(mean, std)) == computed
    desc = workloads.ModelDesc(dtype="bf16", layers=0, d=128, heads=2, mlp=128, patch=14, tpatch=2, merge=2,
                               mean=mean, std=std)
    rng = np.random.default_rng(6)
    items = [workloads.Item(1, 1, 84, 532, 84, 532, workloads.random_frames(rng, 1, 84, 532)),       # 38 tokens wide: strips of 16, 16, 6
             workloads.Item(2, 4, 56, 476, 56, 476, workloads.random_frames(rng, 4, 56, 476)),       # 34 wide: 16, 16, 2
             workloads.Item(1, 1, 61, 333, 56, 308, workloads.random_frames(rng, 1, 61, 333)),       # resampled
             workloads.Item(2, 2, 100, 90, 84, 112, workloads.random_frames(rng, 2, 100, 90))]
    # every pixel value occurs in every channel of the first image
    items[0].frames.reshape(-1, 3)[:256] = np.arange(256, dtype=np.uint8)[:, None]
    wl = workloads.Workload("normalisation", desc, items, workloads.make_weights(desc, 1))
    enc = VisionEncoder(desc, wl.weights)
    pl = enc.plan(items)
    patches = enc.preprocess(pl)
    torch.cuda.synchronize()
    check_patches(wl, oracle.run(wl, stages=("preprocess",)), patches)


def test_text_only_and_empty_batches_launch_nothing():
    wl = workloads.small_config(5)
    enc = VisionEncoder(wl.desc, wl.weights)
    for items in ([], [workloads.Item(0, 0, 0, 0, 0, 0, None)] * 4):
        pl = enc.plan(items)
        p = enc.preprocess(pl)
        h = enc.encode(pl, p)
        o = enc.merge_project(pl, h)
        torch.cuda.synchronize()
        assert p.shape[0] == 0 and h.shape[0] == 0 and o.shape[0] == 0


def test_text_requests_do_not_disturb_other_requests():
    wl = workloads.small_config(5)
    only_visual = [it for it in wl.items if it.n_frames > 0]
    enc = VisionEncoder(wl.desc, wl.weights)
    res = []
    for items in (wl.items, only_visual):
        pl = enc.plan(items)
        h = enc.encode(pl, enc.preprocess(pl))
        res.append(enc.merge_project(pl, h).float().cpu().numpy())
    assert np.array_equal(res[0], res[1])


def test_permutation_equivariance_without_positions():
    """Permuting the patch rows of a segment permutes the encoder output rows."""
    desc = workloads.ModelDesc(dtype="bf16", layers=2, d=128, heads=2, mlp=256, patch=14, tpatch=1, merge=1)
    w = workloads.make_weights(desc, 3, random_affine=True)
    rng = np.random.default_rng(3)
    it = workloads.Item(1, 1, 70, 84, 70, 84, workloads.random_frames(rng, 1, 70, 84))
    enc = VisionEncoder(desc, w)
    pl = enc.plan([it])
    patches = enc.preprocess(pl)
    perm = torch.from_numpy(rng.permutation(patches.shape[0])).to(patches.device)
    a = enc.encode(pl, patches).clone()
    b = enc.encode(pl, patches[perm].contiguous())
    torch.cuda.synchronize()
    assert_tokens_close(b.cpu().numpy(), a[perm].cpu().numpy(), 2e-2, 0.999, "permutation")


def test_workspace_too_small_and_missing_projector_are_reported():
    wl = workloads.small_config(2)
    enc = VisionEncoder(wl.desc, wl.weights)
    pl = enc.plan(wl.items)
    patches = enc.preprocess(pl)
    small = enc.workspace(256)
    hidden = torch.empty((pl.info.n_tokens, wl.desc.d), device="cuda:0")
    with pytest.raises(B.TcmvError) as e:
        B.tcmv_encode(enc.ctx, pl.handle, pl.meta, patches, hidden, small, small.numel())
    assert e.value.code == B.TCMV_E_WORKSPACE_TOO_SMALL
    with pytest.raises(B.TcmvError) as e:
        B.tcmv_merge_project(enc.ctx, pl.handle, hidden, hidden, small, small.numel())
    assert e.value.code == B.TCMV_E_UNSUPPORTED


def test_results_are_deterministic_run_to_run():
    wl = workloads.small_config(3)
    a = run_gpu(wl)[4].float().cpu().numpy()
    b = run_gpu(wl)[4].float().cpu().numpy()
    assert np.array_equal(a, b)


def test_per_request_pipeline_matches_plan_by_plan_runs():
    """One plan per request, preprocessing of the next request overlapped with the
    encoding of the current one on a second stream: outputs must be the ones of
    running the requests one after the other, and each request's output must be
    its rows of the batched run (requests do not interact)."""
    for idx in (5, 6):
        wl = workloads.small_config(idx)
        enc = VisionEncoder(wl.desc, wl.weights)
        plans = [enc.plan([it]) for it in wl.items]
        seq = [enc.run(p).float().cpu().numpy() for p in plans]
        for _ in range(2):
            pip = enc.run_pipelined(plans)
            torch.cuda.synchronize()
            for a, b in zip(seq, pip):
                assert np.array_equal(a, b.float().cpu().numpy())
        whole = enc.plan(wl.items)
        out = enc.run(whole).float().cpu().numpy()
        m2 = wl.desc.merge ** 2
        r0 = 0
        for a, plan in zip(seq, plans):
            assert plan.info.n_out_tokens == a.shape[0] == plan.info.n_tokens // m2
            assert_tokens_close(out[r0:r0 + a.shape[0]], a, 2e-2, 0.999, f"{wl.name} request rows")
            r0 += a.shape[0]
        assert r0 == out.shape[0]


@pytest.mark.parametrize("std", [0.02, 0.08])
def test_long_segments_take_the_norm_bounded_attention_path(std):
    """Segments of 4096 and 2304 tokens make the library compute key norms and run attention without a softmax
    reference where the bound allows it; the result must not depend on which copy of the kernel ran."""
    desc = workloads.qwen_like_desc(layers=2, d=320, heads=4, mlp=640, out_dim=192, max_grid=48)
    rng = np.random.default_rng(9)
    items = [workloads.Item(2, 8, 448, 448, 448, 448, workloads.random_frames(rng, 8, 448, 448)),
             workloads.Item(1, 1, 672, 672, 672, 672, workloads.random_frames(rng, 1, 672, 672))]
    wl = workloads.Workload("long", desc, items, workloads.make_weights(desc, 31, std=std, random_affine=True))
    ref = oracle.run(wl, workers=4)
    enc, pl, patches, hidden, out = run_gpu(wl)
    assert pl.cu_seqlens == [0, 4096, 4096 + 2304]
    assert_tokens_close(hidden.cpu().numpy(), ref["hidden"], 2e-2, 0.999, "long segments hidden")
    assert_tokens_close(out.float().cpu().numpy(), ref["out"], 2e-2, 0.999, "long segments out")


@pytest.mark.parametrize("dh", [80, 64])
def test_windows_of_up_to_64_tokens_with_ragged_edges(dh):
    """Windows of 8 x 8 patches on grids that are not multiples of 8: window sizes 64, 48, 32, 24, 16, 8 ... in
    one batch, every layer windowed (the short-window attention kernel: second wave idle below 33 tokens, keys
    masked beyond the window), then with every second layer over the whole request."""
    rng = np.random.default_rng(31)
    sizes = [(168, 140), (196, 252), (224, 224), (112, 28), (28, 364)]      # patch grids 12x10, 14x18, 16x16, 8x2, 2x26
    items = [workloads.Item(workloads.IMAGE, 1, h, w, h, w, workloads.random_frames(rng, 1, h, w)) for h, w in sizes]
    items.insert(2, workloads.Item(workloads.VIDEO, 4, 140, 196, 140, 196, workloads.random_frames(rng, 4, 140, 196)))
    for full_every in (0, 2):
        desc = workloads.windowed_desc(layers=2, d=4 * dh, heads=4, mlp=640, out_dim=192, window=8, full_every=full_every)
        wl = workloads.Workload("ragged_windows", desc, items, workloads.make_weights(desc, 3100 + dh, random_affine=True))
        ref = oracle.run(wl)
        enc, pl, patches, hidden, out = run_gpu(wl)
        check_patches(wl, ref, patches)
        assert_tokens_close(hidden.cpu().numpy(), ref["hidden"], 2e-2, 0.999, f"ragged windows dh={dh} hidden")
        assert_tokens_close(out.float().cpu().numpy(), ref["out"], 2e-2, 0.999, f"ragged windows dh={dh} out")


def test_single_small_request_with_long_mlp_contraction():
    """One small request through a model whose fc2 contraction is long (mlp 2048 over 320 rows of tokens): the
    library computes that product in four slices of k and adds them in a fixed order.  Result within the usual
    bar, identical from run to run, and equal to what the same request gets inside a large batch (where the
    product is computed undivided) up to fp32 summation order."""
    rng = np.random.default_rng(41)
    desc = workloads.qwen_like_desc(layers=2, d=320, heads=4, mlp=2048, out_dim=192, max_grid=16)
    item = workloads.Item(workloads.IMAGE, 1, 224, 140, 224, 140, workloads.random_frames(rng, 1, 224, 140))
    wl = workloads.Workload("one_small_request", desc, [item], workloads.make_weights(desc, 4100, random_affine=True))
    ref = oracle.run(wl)
    enc, pl, patches, hidden, out = run_gpu(wl)
    assert_tokens_close(hidden.cpu().numpy(), ref["hidden"], 2e-2, 0.999, "single request hidden")
    assert_tokens_close(out.float().cpu().numpy(), ref["out"], 2e-2, 0.999, "single request out")
    again = enc.encode(pl, patches)
    torch.cuda.synchronize()
    assert torch.equal(hidden, again)
    # the same request as the first of a batch large enough for the undivided product
    others = [workloads.Item(workloads.IMAGE, 1, 224, 224, 224, 224, workloads.random_frames(rng, 1, 224, 224))
              for _ in range(40)]
    plb = enc.plan([item] + others)
    hb = enc.encode(plb, enc.preprocess(plb))
    torch.cuda.synchronize()
    n = hidden.shape[0]
    assert_tokens_close(hb[:n].cpu().numpy(), hidden.cpu().numpy().astype(np.float64), 2e-3, 0.99999, "batch vs alone")
