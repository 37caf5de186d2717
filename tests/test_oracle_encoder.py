"""Pins for the CPU reference of the encoder / projector: closed forms,
invariants, special cases that reduce to a library routine, brute force."""
import math

import numpy as np
import pytest
import torch

import workloads
import oracle
from oracle import encoder as oe
from oracle import naive


def _rand(rng, *s, scale=1.0):
    return rng.normal(0, scale, size=s)


def test_softmax_rows_sum_to_one_and_special_cases():
    rng = np.random.default_rng(0)
    T, d, heads = 37, 24, 3
    q, k, v = _rand(rng, T, d, scale=3), _rand(rng, T, d, scale=3), _rand(rng, T, d)
    cu = [0, 1, 1, 20, 37]                       # single-key, empty, ragged segments
    out, probs = oe.attention(q, k, v, cu, heads, q_block=7, return_probs=True)
    for p in probs:
        assert np.abs(p.sum(-1) - 1).max() <= 1e-12 and p.min() >= 0
    assert np.array_equal(out[0], v[0])           # one key: the output is that key's value row
    o0 = oe.attention(np.zeros_like(q), k, v, cu, heads)
    for a, b in [(1, 20), (20, 37)]:              # zero queries: uniform weights -> mean of V
        assert np.allclose(o0[a:b], v[a:b].mean(0, keepdims=True), atol=1e-13)
    # query blocking does not change anything
    assert np.array_equal(out, oe.attention(q, k, v, cu, heads, q_block=1000))


def test_attention_matches_pure_python_loops():
    rng = np.random.default_rng(1)
    T, d, heads = 29, 16, 2
    q, k, v = _rand(rng, T, d, scale=2), _rand(rng, T, d, scale=2), _rand(rng, T, d)
    cu = [0, 5, 5, 18, 29]
    ref = np.array(naive.attention_loops(q.tolist(), k.tolist(), v.tolist(), cu, heads))
    assert np.abs(oe.attention(q, k, v, cu, heads) - ref).max() <= 1e-12


def test_attention_matches_library_sdpa():
    rng = np.random.default_rng(2)
    T, d, heads = 48, 32, 4
    q, k, v = _rand(rng, T, d), _rand(rng, T, d), _rand(rng, T, d)
    got = oe.attention(q, k, v, [0, T], heads)
    tq, tk, tv = (torch.from_numpy(a).view(T, heads, d // heads).transpose(0, 1) for a in (q, k, v))
    lib = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv).transpose(0, 1).reshape(T, d).numpy()
    assert np.abs(got - lib).max() <= 1e-12


def test_attention_peaked_scores_pick_argmax_value():
    rng = np.random.default_rng(3)
    T, d = 16, 8
    k = _rand(rng, T, d); v = _rand(rng, T, d)
    q = 200.0 * k                                  # each query overwhelmingly matches its own key
    out = oe.attention(q, k, v, [0, T], 1)
    s = q @ k.T
    assert np.allclose(out, v[s.argmax(1)], atol=1e-9)


def test_layernorm_statistics_and_library():
    rng = np.random.default_rng(4)
    x = _rand(rng, 11, 96, scale=5) + 3
    y = oe.layernorm(x, np.ones(96), np.zeros(96), 0.0)
    assert np.abs(y.mean(-1)).max() <= 1e-13 and np.abs(y.var(-1) - 1).max() <= 1e-12
    g, b = _rand(rng, 96), _rand(rng, 96)
    lib = torch.nn.functional.layer_norm(torch.from_numpy(x), (96,), torch.from_numpy(g), torch.from_numpy(b), 1e-6)
    assert np.abs(oe.layernorm(x, g, b, 1e-6) - lib.numpy()).max() <= 1e-12
    # eps matters for a constant row: output is exactly beta
    c = np.full((1, 96), 2.5)
    assert np.allclose(oe.layernorm(c, g, b, 1e-6), b)


def test_gelu_identities_and_tabulated_values():
    x = np.linspace(-6, 6, 241)
    assert np.abs(oe.gelu(x) - oe.gelu(-x) - x).max() <= 1e-15
    assert oe.gelu(np.array(0.0)) == 0.0
    # Phi(1) = 0.841344746068543 (standard normal CDF, tabulated), Phi(2) = 0.977249868051821
    assert abs(oe.gelu(np.array(1.0)) - 0.841344746068543) <= 1e-14
    assert abs(oe.gelu(np.array(2.0)) - 2 * 0.977249868051821) <= 1e-14
    assert abs(oe.gelu(np.array(-1.0)) - (-(1 - 0.841344746068543))) <= 1e-14
    ref = np.array([0.5 * t * (1 + math.erf(t / math.sqrt(2))) for t in x])
    assert np.abs(oe.gelu(x) - ref).max() <= 1e-15
    # the tanh approximation is a different function: it must NOT be what is implemented
    tanh_form = 0.5 * x * (1 + np.tanh(math.sqrt(2 / math.pi) * (x + 0.044715 * x ** 3)))
    assert np.abs(oe.gelu(x) - tanh_form).max() > 1e-4


def _tiny(pos="none", use_cls=0, layers=2, merge=1, out_dim=0, tpatch=1):
    desc = workloads.ModelDesc(dtype="f32", layers=layers, d=32, heads=2, mlp=64, patch=4, tpatch=tpatch,
                               merge=merge, out_dim=out_dim, use_cls=use_cls, pos=pos, max_pos=40, final_ln=0)
    return desc


def test_depth_zero_is_one_library_gemm():
    desc = _tiny(layers=0)
    w = workloads.make_weights(desc, 5, random_affine=True)
    rng = np.random.default_rng(5)
    p = [rng.normal(size=(12, desc.k)), rng.normal(size=(6, desc.k))]
    grids = [(1, 3, 4), (1, 2, 3)]
    got = oe.encode(p, grids, desc, w)
    ref = torch.addmm(torch.from_numpy(w["b_pe"]).double(), torch.from_numpy(np.concatenate(p)),
                      torch.from_numpy(w["w_pe"]).double().T).numpy()
    assert np.abs(got - ref).max() <= 1e-13


def test_zero_output_projections_make_blocks_identity():
    desc = _tiny(layers=3)
    w = workloads.make_weights(desc, 6, random_affine=True)
    for l in range(3):
        for n in ("w_o", "b_o", "w_2", "b_2"):
            w[f"l{l}.{n}"] = np.zeros_like(w[f"l{l}.{n}"])
    rng = np.random.default_rng(6)
    p = [rng.normal(size=(12, desc.k))]
    a = oe.encode(p, [(1, 3, 4)], desc, w)
    d0 = _tiny(layers=0)
    assert np.array_equal(a, oe.encode(p, [(1, 3, 4)], d0, w))


def test_block_residual_wiring_against_torch_modules():
    """One pre-LN block assembled from torch.nn library layers."""
    desc = _tiny(layers=1)
    w = workloads.make_weights(desc, 7, random_affine=True, std=0.2)
    rng = np.random.default_rng(7)
    x = rng.normal(size=(10, desc.d))
    got = oe.encoder_block(x, np.array([0, 10]), desc, w, 0)
    t = lambda n: torch.from_numpy(w["l0." + n]).double()
    X = torch.from_numpy(x)
    mha = torch.nn.MultiheadAttention(desc.d, desc.heads, bias=True, batch_first=True, dtype=torch.float64)
    with torch.no_grad():
        mha.in_proj_weight.copy_(t("w_qkv")); mha.in_proj_bias.copy_(t("b_qkv"))
        mha.out_proj.weight.copy_(t("w_o")); mha.out_proj.bias.copy_(t("b_o"))
        h = torch.nn.functional.layer_norm(X, (desc.d,), t("ln1_g"), t("ln1_b"), desc.ln_eps)
        X = X + mha(h[None], h[None], h[None], need_weights=False)[0][0]
        h = torch.nn.functional.layer_norm(X, (desc.d,), t("ln2_g"), t("ln2_b"), desc.ln_eps)
        h = torch.nn.functional.gelu(torch.nn.functional.linear(h, t("w_1"), t("b_1")))
        X = X + torch.nn.functional.linear(h, t("w_2"), t("b_2"))
    assert np.abs(got - X.numpy()).max() <= 1e-12


def test_permutation_equivariance_without_position_terms():
    desc = _tiny(layers=2)
    w = workloads.make_weights(desc, 8, random_affine=True, std=0.3)
    rng = np.random.default_rng(8)
    p = rng.normal(size=(12, desc.k))
    perm = rng.permutation(12)
    a = oe.encode([p], [(1, 3, 4)], desc, w)
    b = oe.encode([p[perm]], [(1, 3, 4)], desc, w)
    assert np.abs(a[perm] - b).max() <= 1e-12
    # and with a position term the equivariance must break
    desc_p = _tiny(pos="learned1d", layers=2)
    wp = workloads.make_weights(desc_p, 8, random_affine=True, std=0.3)
    a = oe.encode([p], [(1, 3, 4)], desc_p, wp)
    b = oe.encode([p[perm]], [(1, 3, 4)], desc_p, wp)
    assert np.abs(a[perm] - b).max() > 1e-3


def test_segments_are_independent():
    desc = _tiny(pos="sep2d", layers=2, merge=2, out_dim=24, tpatch=2)
    w = workloads.make_weights(desc, 9, random_affine=True, std=0.3)
    rng = np.random.default_rng(9)
    pa, pb = rng.normal(size=(16, desc.k)), rng.normal(size=(8, desc.k))
    ga, gb = (1, 4, 4), (2, 2, 2)
    both = oe.encode([pa, np.zeros((0, desc.k)), pb], [ga, (0, 0, 0), gb], desc, w)
    assert np.abs(both[:16] - oe.encode([pa], [ga], desc, w)).max() <= 1e-13
    assert np.abs(both[16:] - oe.encode([pb], [gb], desc, w)).max() <= 1e-13
    # poisoning the other segment must not move this one
    poisoned = oe.encode([pa, 1e6 * pb], [ga, gb], desc, w)
    assert np.abs(poisoned[:16] - both[:16]).max() <= 1e-13


def test_position_terms_and_cls():
    desc = _tiny(pos="sep2d", layers=0, merge=2, tpatch=2)
    w = workloads.make_weights(desc, 10)
    p = np.zeros((16, desc.k))
    x = oe.encode([p], [(2, 2, 4)], desc, w)       # zero patches, zero bias: output is the position term
    from oracle.preprocess import token_coords
    co = token_coords(2, 2, 4, 2)
    for r in range(16):
        assert np.allclose(x[r], w["pos0"][co[r, 1]].astype(np.float64) + w["pos1"][co[r, 2]])
    assert np.array_equal(x[:8], x[8:])             # shared by all frame groups of a video
    desc = _tiny(pos="learned1d", use_cls=1, layers=0)
    w = workloads.make_weights(desc, 11)
    x = oe.encode([np.zeros((6, desc.k)), np.zeros((4, desc.k))], [(1, 2, 3), (1, 2, 2)], desc, w)
    assert x.shape == (12, desc.d)
    assert np.allclose(x[0], w["cls"].astype(np.float64) + w["pos0"][0]) and np.allclose(x[7], x[0])
    assert np.allclose(x[1:7], w["pos0"][1:7]) and np.allclose(x[8:12], w["pos0"][1:5])


def test_merge_view_against_brute_force_gather():
    desc = _tiny(pos="none", layers=0, merge=2, out_dim=24, tpatch=1)
    w = workloads.make_weights(desc, 12, random_affine=True, std=0.2)
    rng = np.random.default_rng(12)
    gh, gw = 4, 6
    x = rng.normal(size=(gh * gw, desc.d))
    out = oe.merge_project(x, desc, w)
    from oracle.preprocess import token_coords
    co = token_coords(1, gh, gw, 2)
    row_of = {(h, ww): r for r, (_, h, ww) in enumerate(co)}
    y = oe.layernorm(x, w["lnm_g"].astype(np.float64), w["lnm_b"].astype(np.float64), desc.ln_eps)
    g = 0
    for hb in range(gh // 2):
        for wb in range(gw // 2):
            cat = np.concatenate([y[row_of[(2 * hb + hi, 2 * wb + wi)]] for hi in range(2) for wi in range(2)])
            hid = oe.gelu(w["w_m1"].astype(np.float64) @ cat + w["b_m1"])
            ref = w["w_m2"].astype(np.float64) @ hid + w["b_m2"]
            assert np.abs(out[g] - ref).max() <= 1e-12
            g += 1
    assert g == out.shape[0]


def test_weight_layout_is_out_by_in():
    desc = _tiny(layers=1)
    w = workloads.make_weights(desc, 13)
    assert w["w_pe"].shape == (desc.d, desc.k) and w["l0.w_qkv"].shape == (3 * desc.d, desc.d)
    assert w["l0.w_1"].shape == (desc.mlp, desc.d) and w["l0.w_2"].shape == (desc.d, desc.mlp)


def test_fp32_and_fp64_evaluations_agree_on_small_workloads():
    for idx in (1, 3, 5):
        wl = workloads.small_config(idx)
        a = oracle.run(wl, np.float64)
        b = oracle.run(wl, np.float32)
        key = "out" if "out" in a else "hidden"
        scale = np.abs(a[key]).max()
        assert np.abs(a[key] - b[key]).max() <= 2e-5 * scale
        for pa, pb in zip(a["patches"], b["patches"]):
            assert np.array_equal(pa, pb)


def test_attention_energy_note():
    """With N(0, 0.02) weights the scores are near-uniform, so end-to-end parity
    is nearly blind to attention errors; this documents why adversarial
    (peaked) attention tests exist on the GPU side."""
    wl = workloads.small_config(4, random_affine=False)
    r = oracle.run(wl)
    assert np.isfinite(r["out"]).all()


def test_row_subset_evaluation_equals_full_evaluation():
    """The row-subset mode used for full-size checks returns exactly the rows of the full result."""
    desc = _tiny(pos="none", layers=1)
    w = workloads.make_weights(desc, 21, random_affine=True, std=0.3)
    rng = np.random.default_rng(21)
    x = rng.normal(size=(40, desc.d))
    cu = np.array([0, 7, 7, 25, 40])
    rows = [0, 6, 7, 24, 25, 39]
    full = oe.encoder_block(x, cu, desc, w, 0)
    part = oe.encoder_block(x, cu, desc, w, 0, rows=rows)
    assert np.abs(full[rows] - part).max() <= 1e-13


def test_threaded_heads_give_identical_results():
    rng = np.random.default_rng(31)
    q, k, v = _rand(rng, 50, 48), _rand(rng, 50, 48), _rand(rng, 50, 48)
    cu = [0, 13, 50]
    assert np.array_equal(oe.attention(q, k, v, cu, 4), oe.attention(q, k, v, cu, 4, workers=3))


@pytest.mark.parametrize("kind", ["image_cls_learned", "video_sep2d"])
def test_whole_encoder_against_torch_transformer(kind):
    """The whole path frames -> hidden against a model put together from torch.nn library modules only:
    Conv2d / Conv3d with kernel = stride = patch as the patch embedding (which also fixes the element
    order inside a patch row and the raster order of the rows), nn.TransformerEncoder with
    norm_first=True and exact GELU as the blocks, nn.LayerNorm as the final norm."""
    rng = np.random.default_rng(5)
    if kind == "image_cls_learned":
        desc = workloads.ModelDesc(dtype="f32", layers=3, d=64, heads=4, mlp=128, patch=16, tpatch=1, merge=1, use_cls=1,
                         pos="learned1d", max_pos=13, final_ln=1)
        frames = workloads.random_frames(rng, 1, 48, 64)
        item = workloads.Item(workloads.IMAGE, 1, 48, 64, 48, 64, frames)
    else:
        desc = workloads.ModelDesc(dtype="f32", layers=2, d=48, heads=3, mlp=96, patch=8, tpatch=2, merge=1, use_cls=0,
                         pos="sep2d", max_pos=6, final_ln=0)
        frames = workloads.random_frames(rng, 4, 24, 40)
        item = workloads.Item(workloads.VIDEO, 4, 24, 40, 24, 40, frames)
    w = workloads.make_weights(desc, 77, random_affine=True)
    wl = workloads.Workload(kind, desc, [item], w)
    got = oracle.run(wl, dtype=np.float64)["hidden"]

    t = lambda a: torch.from_numpy(np.asarray(a, np.float64))
    d, P, tp = desc.d, desc.patch, desc.tpatch
    mean, std = t(desc.mean).view(1, 3, 1, 1), t(desc.std).view(1, 3, 1, 1)
    x = (t(frames).permute(0, 3, 1, 2) / 255.0 - mean) / std          # [n, 3, H, W]
    x = x.float().double()                                            # the stage stores fp32 patch values
    if tp == 1:
        conv = torch.nn.Conv2d(3, d, P, stride=P, dtype=torch.float64)
        conv.weight.data = t(w["w_pe"][:, :desc.k]).view(d, 3, P, P)
        conv.bias.data = t(w["b_pe"])
        tok = conv(x).flatten(2).transpose(1, 2)                      # [1, gh*gw, d], rows in (h, w) order
    else:
        conv = torch.nn.Conv3d(3, d, (tp, P, P), stride=(tp, P, P), dtype=torch.float64)
        conv.weight.data = t(w["w_pe"][:, :desc.k]).view(d, 3, tp, P, P)
        conv.bias.data = t(w["b_pe"])
        vol = x.permute(1, 0, 2, 3).unsqueeze(0)                      # [1, 3, n, H, W]
        tok = conv(vol).flatten(2).transpose(1, 2)                    # rows in (t, h, w) order
    if desc.use_cls:
        tok = torch.cat([t(w["cls"]).view(1, 1, d), tok], 1)
        tok = tok + t(w["pos0"])[: tok.shape[1]].unsqueeze(0)
    else:
        gt, gh, gw = frames.shape[0] // tp, frames.shape[1] // P, frames.shape[2] // P
        pos = (t(w["pos0"])[:gh, None, :] + t(w["pos1"])[None, :gw, :]).reshape(1, gh * gw, d).repeat(1, gt, 1)
        tok = tok + pos
    layer = torch.nn.TransformerEncoderLayer(d, desc.heads, desc.mlp, dropout=0.0, activation="gelu",
                                             layer_norm_eps=desc.ln_eps, batch_first=True, norm_first=True,
                                             dtype=torch.float64)
    final = torch.nn.LayerNorm(d, eps=desc.ln_eps, dtype=torch.float64) if desc.final_ln else None
    model = torch.nn.TransformerEncoder(layer, desc.layers, norm=final, enable_nested_tensor=False)
    for l, lay in enumerate(model.layers):
        g = lambda k: t(w[f"l{l}.{k}"])
        lay.self_attn.in_proj_weight.data, lay.self_attn.in_proj_bias.data = g("w_qkv"), g("b_qkv")
        lay.self_attn.out_proj.weight.data, lay.self_attn.out_proj.bias.data = g("w_o"), g("b_o")
        lay.linear1.weight.data, lay.linear1.bias.data = g("w_1"), g("b_1")
        lay.linear2.weight.data, lay.linear2.bias.data = g("w_2"), g("b_2")
        lay.norm1.weight.data, lay.norm1.bias.data = g("ln1_g"), g("ln1_b")
        lay.norm2.weight.data, lay.norm2.bias.data = g("ln2_g"), g("ln2_b")
    if final is not None:
        final.weight.data, final.bias.data = t(w["lnf_g"]), t(w["lnf_b"])
    model.eval()
    with torch.no_grad():
        ref = model(tok)[0].numpy()
    assert got.shape == ref.shape
    assert np.abs(got - ref).max() <= 1e-9 * max(1.0, np.abs(ref).max())


def test_merged_family_against_torch_modules_and_unfold():
    """The 2x2-merge family end to end (frames -> hidden -> projector output): Conv3d patch embedding and
    nn.TransformerEncoder on raster-ordered tokens, then torch.nn.functional.unfold (kernel = stride = 2) as
    the library's own definition of the 2x2 grouping; the reference's rows come in merge-group order, so its
    hidden matrix viewed as [T/4, 4d] must equal the unfolded raster result group by group."""
    rng = np.random.default_rng(6)
    desc = workloads.ModelDesc(dtype="f32", layers=2, d=32, heads=2, mlp=64, patch=8, tpatch=2, merge=2, out_dim=40,
                               use_cls=0, pos="sep2d", max_pos=6, final_ln=0)
    frames = workloads.random_frames(rng, 4, 32, 48)
    w = workloads.make_weights(desc, 78, random_affine=True)
    wl = workloads.Workload("merged", desc, [workloads.Item(workloads.VIDEO, 4, 32, 48, 32, 48, frames)], w)
    res = oracle.run(wl, dtype=np.float64)

    t = lambda a: torch.from_numpy(np.asarray(a, np.float64))
    d, P, tp = desc.d, desc.patch, desc.tpatch
    gt, gh, gw = 2, 4, 6
    x = ((t(frames).permute(0, 3, 1, 2) / 255.0 - 0.5) / 0.5).float().double()
    conv = torch.nn.Conv3d(3, d, (tp, P, P), stride=(tp, P, P), dtype=torch.float64)
    conv.weight.data, conv.bias.data = t(w["w_pe"][:, :desc.k]).view(d, 3, tp, P, P), t(w["b_pe"])
    tok = conv(x.permute(1, 0, 2, 3).unsqueeze(0)).flatten(2).transpose(1, 2)          # [1, gt*gh*gw, d] raster
    pos = (t(w["pos0"])[:gh, None, :] + t(w["pos1"])[None, :gw, :]).reshape(1, gh * gw, d).repeat(1, gt, 1)
    layer = torch.nn.TransformerEncoderLayer(d, desc.heads, desc.mlp, dropout=0.0, activation="gelu",
                                             layer_norm_eps=desc.ln_eps, batch_first=True, norm_first=True,
                                             dtype=torch.float64)
    model = torch.nn.TransformerEncoder(layer, desc.layers, enable_nested_tensor=False)
    for l, lay in enumerate(model.layers):
        g = lambda k: t(w[f"l{l}.{k}"])
        lay.self_attn.in_proj_weight.data, lay.self_attn.in_proj_bias.data = g("w_qkv"), g("b_qkv")
        lay.self_attn.out_proj.weight.data, lay.self_attn.out_proj.bias.data = g("w_o"), g("b_o")
        lay.linear1.weight.data, lay.linear1.bias.data = g("w_1"), g("b_1")
        lay.linear2.weight.data, lay.linear2.bias.data = g("w_2"), g("b_2")
        lay.norm1.weight.data, lay.norm1.bias.data = g("ln1_g"), g("ln1_b")
        lay.norm2.weight.data, lay.norm2.bias.data = g("ln2_g"), g("ln2_b")
    model.eval()

    def groups(h):          # [gt*gh*gw, d] raster -> [gt*(gh/2)*(gw/2), 4*d], group rows ordered (h%2, w%2)
        img = h.view(gt, gh, gw, d).permute(0, 3, 1, 2)                                 # [gt, d, gh, gw]
        u = torch.nn.functional.unfold(img, kernel_size=2, stride=2)                    # [gt, d*4, L], (c, kh, kw)
        return u.view(gt, d, 4, -1).permute(0, 3, 2, 1).reshape(-1, 4 * d)

    with torch.no_grad():
        hid = model(tok + pos)[0]
        ref_hidden = groups(hid).numpy()
        y = torch.nn.functional.layer_norm(hid, (d,), t(w["lnm_g"]), t(w["lnm_b"]), desc.ln_eps)
        y = torch.nn.functional.gelu(torch.nn.functional.linear(groups(y), t(w["w_m1"]), t(w["b_m1"])))
        ref_out = torch.nn.functional.linear(y, t(w["w_m2"]), t(w["b_m2"])).numpy()
    got_hidden = res["hidden"].reshape(-1, 4 * d)
    assert got_hidden.shape == ref_hidden.shape and res["out"].shape == ref_out.shape
    assert np.abs(got_hidden - ref_hidden).max() <= 1e-9 * max(1.0, np.abs(ref_hidden).max())
    assert np.abs(res["out"] - ref_out).max() <= 1e-9 * max(1.0, np.abs(ref_out).max())
