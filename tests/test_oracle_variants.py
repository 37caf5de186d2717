"""Pins for the encoder variants of the CPU reference (RMSNorm, gated MLP, rotary 2-D positions,
windowed attention): library routines, closed forms, independent formulations, brute force."""
import numpy as np
import pytest
import torch

import workloads
from oracle import encoder as oe
from oracle import preprocess as op


def test_rmsnorm_properties_and_library_routine():
    rng = np.random.default_rng(0)
    x = rng.normal(0.3, 2.0, (7, 64))
    g = rng.normal(1.0, 0.2, 64)
    y = oe.rmsnorm(x, np.ones(64), 0.0)
    assert np.allclose((y ** 2).mean(axis=1), 1.0, atol=1e-12)
    assert np.allclose(oe.rmsnorm(3.7 * x, g, 0.0), oe.rmsnorm(x, g, 0.0), atol=1e-12)
    z = x - x.mean(axis=1, keepdims=True)
    assert np.allclose(oe.rmsnorm(z, g, 1e-6), oe.layernorm(z, g, np.zeros(64), 1e-6), atol=1e-12)
    ref = torch.nn.functional.rms_norm(torch.from_numpy(x), (64,), torch.from_numpy(g), 1e-6).numpy()
    assert np.allclose(oe.rmsnorm(x, g, 1e-6), ref, atol=1e-12)
    desc = workloads.ModelDesc(norm="rms")
    assert np.array_equal(oe.norm(desc, x, g, 5.0 + g), oe.rmsnorm(x, g, desc.ln_eps))     # beta is not used


def test_silu_identities_and_library_routine():
    x = np.linspace(-12, 12, 97)
    assert np.allclose(oe.silu(x) - oe.silu(-x), x, atol=1e-12)
    assert oe.silu(np.array([0.0]))[0] == 0.0
    assert np.allclose(oe.silu(x), torch.nn.functional.silu(torch.from_numpy(x)).numpy(), atol=1e-14)
    assert oe.silu(np.array([1.0]))[0] == pytest.approx(1.0 / (1.0 + np.exp(-1.0)))


def test_gated_block_against_torch_modules():
    desc = workloads.ModelDesc(dtype="f32", layers=1, d=32, heads=2, mlp=48, norm="rms", gated=1)
    w = workloads.make_weights(desc, 5, std=0.2, random_affine=True)
    assert w["l0.w_1"].shape == (96, 32) and w["l0.b_1"].shape == (96,)
    w["l0.w_o"][:] = 0
    w["l0.b_o"][:] = 0                                   # attention branch contributes nothing
    rng = np.random.default_rng(1)
    x = rng.normal(0, 1, (9, 32))
    got = oe.encoder_block(x, np.array([0, 9]), desc, w, 0)
    t = lambda a: torch.from_numpy(np.asarray(a, np.float64))
    xt = t(x)
    h = torch.nn.functional.rms_norm(xt, (32,), t(w["l0.ln2_g"]), desc.ln_eps)
    gate = torch.nn.functional.linear(h, t(w["l0.w_1"][:48]), t(w["l0.b_1"][:48]))
    up = torch.nn.functional.linear(h, t(w["l0.w_1"][48:]), t(w["l0.b_1"][48:]))
    ref = xt + torch.nn.functional.linear(torch.nn.functional.silu(gate) * up, t(w["l0.w_2"]), t(w["l0.b_2"]))
    assert np.allclose(got, ref.numpy(), atol=1e-12)


def test_rotary_against_complex_multiplication_and_invariants():
    rng = np.random.default_rng(2)
    heads, dh, T = 3, 8, 11
    x = rng.normal(0, 1, (T, heads * dh))
    hw = rng.integers(0, 40, (T, 2))
    ang = oe.rope_angles(hw, dh, 10000.0)
    assert ang.shape == (T, dh // 2)
    # angle table: pair p < dh/4 follows h, the others w, frequency theta^(-j/(dh/4))
    for r in range(T):
        for p in range(dh // 2):
            ax, j = (0, p) if p < dh // 4 else (1, p - dh // 4)
            assert ang[r, p] == pytest.approx(hw[r, ax] * 10000.0 ** (-j / (dh // 4)), rel=1e-13)
    y = oe.rope_rotate(x, ang, heads)
    z = x.reshape(T, heads, dh // 2, 2)
    zc = (z[..., 0] + 1j * z[..., 1]) * np.exp(1j * ang)[:, None, :]
    assert np.allclose(y.reshape(T, heads, dh // 2, 2)[..., 0], zc.real, atol=1e-13)
    assert np.allclose(y.reshape(T, heads, dh // 2, 2)[..., 1], zc.imag, atol=1e-13)
    assert np.allclose((y ** 2).reshape(T, -1, 2).sum(-1), (x ** 2).reshape(T, -1, 2).sum(-1), atol=1e-12)
    assert np.array_equal(oe.rope_rotate(x, oe.rope_angles(np.zeros((T, 2)), dh, 10000.0), heads), x)
    # scores depend on coordinate differences only: shifting every token by the same offset changes nothing
    q, k = rng.normal(0, 1, (T, heads * dh)), rng.normal(0, 1, (T, heads * dh))
    s0 = oe.rope_rotate(q, ang, heads) @ oe.rope_rotate(k, ang, heads).T
    ang2 = oe.rope_angles(hw + np.array([5, 9]), dh, 10000.0)
    s1 = oe.rope_rotate(q, ang2, heads) @ oe.rope_rotate(k, ang2, heads).T
    assert np.allclose(s0, s1, atol=1e-10)
    with pytest.raises(ValueError):
        oe.rope_angles(hw, 6, 10000.0)


@pytest.mark.parametrize("gt,gh,gw,merge,win", [(1, 6, 6, 2, 4), (2, 8, 12, 2, 4), (1, 10, 6, 2, 4), (3, 5, 7, 1, 3),
                                                (1, 4, 4, 2, 8)])
def test_window_major_token_order(gt, gh, gw, merge, win):
    co = op.token_coords(gt, gh, gw, merge, win)
    assert sorted(map(tuple, co.tolist())) == [(t, h, w) for t in range(gt) for h in range(gh) for w in range(gw)]
    lens = op.window_lengths(gt, gh, gw, win)
    assert sum(lens) == gt * gh * gw and len(lens) == gt * -(-gh // win) * -(-gw // win)
    r = 0
    seen = []
    for n in lens:                                    # every window is a contiguous run with one window index
        blk = co[r:r + n]
        key = {(t, h // win, w // win) for t, h, w in blk.tolist()}
        assert len(key) == 1
        seen.append(key.pop())
        r += n
    assert seen == sorted(seen)                       # frame group, then window row, then window column
    if merge == 2:                                    # merge groups are still four consecutive rows
        g = co.reshape(-1, 4, 3)
        assert np.all(g[:, :, 0] == g[:, :1, 0]) and np.all(g[:, :, 1] // 2 == g[:, :1, 1] // 2)
        assert np.all(g[:, :, 2] // 2 == g[:, :1, 2] // 2)
    if win >= max(gh, gw):
        assert np.array_equal(co, op.token_coords(gt, gh, gw, merge))
    with pytest.raises(ValueError):
        op.token_coords(1, 4, 4, 2, 3)


def test_windowed_attention_against_dense_mask():
    rng = np.random.default_rng(3)
    desc = workloads.ModelDesc(dtype="f32", layers=1, d=16, heads=2, mlp=16, merge=2, window=4, full_every=0)
    grids = [(2, 6, 10), (1, 4, 4)]
    cu = oe.cu_seqlens_of(grids, 0)
    cu_win = oe.window_cu_seqlens_of(grids, desc)
    T = int(cu[-1])
    q, k, v = (rng.normal(0, 1, (T, 16)) for _ in range(3))
    got = oe.attention(q, k, v, cu_win, 2)
    # brute force: a query sees a key iff same request, same frame group, same window
    ident = []
    for i, (gt, gh, gw) in enumerate(grids):
        for t, h, w in op.token_coords(gt, gh, gw, 2, 4).tolist():
            ident.append((i, t, h // 4, w // 4))
    ref = np.zeros_like(q)
    for hd in range(2):
        c = slice(hd * 8, hd * 8 + 8)
        s = q[:, c] @ k[:, c].T / np.sqrt(8)
        for a in range(T):
            m = np.array([ident[b] == ident[a] for b in range(T)])
            e = np.where(m, np.exp(s[a] - s[a][m].max()), 0.0)
            ref[a, c] = (e / e.sum()) @ v[:, c]
    assert np.allclose(got, ref, atol=1e-12)
    assert cu_win[-1] == T and set(cu.tolist()) <= set(cu_win.tolist())


def test_layer_schedule_and_single_window_equals_full_attention():
    desc = workloads.ModelDesc(window=4, full_every=4, layers=8)
    assert [oe.layer_is_windowed(desc, l) for l in range(8)] == [True, True, True, False, True, True, True, False]
    assert not any(oe.layer_is_windowed(workloads.ModelDesc(window=0, full_every=2), l) for l in range(4))
    assert all(oe.layer_is_windowed(workloads.ModelDesc(window=4, full_every=0), l) for l in range(4))
    # one image whose grid fits in one window: the windowed model is the unwindowed one
    import oracle
    base = dict(dtype="f32", layers=2, d=32, heads=2, mlp=64, patch=4, tpatch=2, merge=2, out_dim=24, pos="rope2d",
                norm="rms", gated=1)
    rng = np.random.default_rng(4)
    it = workloads.Item(1, 1, 24, 16, 24, 16, workloads.random_frames(rng, 1, 24, 16))
    outs = []
    for win in (0, 8):
        desc = workloads.ModelDesc(window=win, **base)
        wl = workloads.Workload("t", desc, [it], workloads.make_weights(desc, 9, std=0.1, random_affine=True))
        outs.append(oracle.run(wl)["out"])
    assert np.array_equal(outs[0], outs[1])
    # and with a smaller window the result changes
    desc = workloads.ModelDesc(window=2, **base)
    wl = workloads.Workload("t", desc, [it], workloads.make_weights(desc, 9, std=0.1, random_affine=True))
    o2 = oracle.run(wl)
    assert o2["out"].shape == outs[0].shape and not np.allclose(o2["out"], outs[0], atol=1e-3)
