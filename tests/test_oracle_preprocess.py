"""Pins for the CPU reference of preprocessing: every check compares it with
something fixed outside it (hand-worked values, closed forms, a library
routine, brute force, invariants)."""
import os

import numpy as np
import pytest
import torch

from oracle import preprocess as op

GOLD = os.path.join(os.path.dirname(__file__), "golden", "resize_examples.txt")


def _cases():
    lines = [l.strip() for l in open(GOLD) if l.strip() and not l.startswith("#")]
    i, out = 0, []
    while i < len(lines):
        tok = lines[i].split()
        assert tok[0] == "case"
        name, sh, sw, dh, dw = tok[1], *map(int, tok[2:])
        src = np.array([list(map(int, lines[i + 1 + r].split())) for r in range(sh)])
        dst = np.array([list(map(int, lines[i + 1 + sh + r].split())) for r in range(dh)])
        assert src.shape == (sh, sw) and dst.shape == (dh, dw)
        out.append((name, src, dst))
        i += 1 + sh + dh
    return out


@pytest.mark.parametrize("name,src,dst", _cases())
def test_resize_hand_worked(name, src, dst):
    f = np.repeat(src[None, :, :, None], 3, axis=3).astype(np.uint8)
    got = op.resize_bilinear_u8(f, *dst.shape)
    for c in range(3):
        assert np.array_equal(got[0, :, :, c], dst), name


def test_resize_identity_and_constant():
    rng = np.random.default_rng(0)
    f = rng.integers(0, 256, (2, 17, 23, 3), dtype=np.uint8)
    assert np.array_equal(op.resize_bilinear_u8(f, 17, 23), f)
    for v in (0, 1, 127, 254, 255):
        c = np.full((1, 9, 13, 3), v, np.uint8)
        assert np.all(op.resize_bilinear_u8(c, 28, 5) == v)


def test_resize_exact_2x_is_block_mean():
    rng = np.random.default_rng(1)
    f = rng.integers(0, 256, (1, 12, 20, 3), dtype=np.uint8)
    got = op.resize_bilinear_u8(f, 6, 10)
    s = f.astype(np.int64).reshape(1, 6, 2, 10, 2, 3).sum(axis=(2, 4))
    assert np.array_equal(got, ((s + 2) >> 2).astype(np.uint8))


def _float_bilinear(f, dh, dw):
    """Textbook real-valued bilinear sampling at half-pixel centres with clamping."""
    n, hs, ws, _ = f.shape
    ys = np.clip((np.arange(dh) + 0.5) * hs / dh - 0.5, 0, hs - 1)
    xs = np.clip((np.arange(dw) + 0.5) * ws / dw - 0.5, 0, ws - 1)
    y0 = np.floor(ys).astype(int); x0 = np.floor(xs).astype(int)
    y1 = np.minimum(y0 + 1, hs - 1); x1 = np.minimum(x0 + 1, ws - 1)
    wy = (ys - y0)[None, :, None, None]; wx = (xs - x0)[None, None, :, None]
    g = f.astype(np.float64)
    top = g[:, y0][:, :, x0] * (1 - wx) + g[:, y0][:, :, x1] * wx
    bot = g[:, y1][:, :, x0] * (1 - wx) + g[:, y1][:, :, x1] * wx
    return top * (1 - wy) + bot * wy


@pytest.mark.parametrize("shape", [((37, 53), (28, 56)), ((240, 426), (56, 84)), ((31, 17), (84, 140)),
                                   ((5, 1), (14, 14)), ((1080, 1920), (28, 28))])
def test_resize_close_to_real_valued_bilinear(shape):
    (hs, ws), (dh, dw) = shape
    rng = np.random.default_rng(hs * 131 + ws)
    f = rng.integers(0, 256, (1, hs, ws, 3), dtype=np.uint8)
    got = op.resize_bilinear_u8(f, dh, dw).astype(np.float64)
    ref = _float_bilinear(f, dh, dw)
    # rounding (0.5) + weight quantisation to 1/2048 (two axes, <= 255*2/4096 each)
    assert np.abs(got - ref).max() <= 0.5 + 255 * 4 / 4096 + 1e-9
    # library routine with the same sampling convention
    t = torch.from_numpy(f).permute(0, 3, 1, 2).double()
    lib = torch.nn.functional.interpolate(t, size=(dh, dw), mode="bilinear", align_corners=False,
                                          antialias=False).permute(0, 2, 3, 1).numpy()
    assert np.abs(got - lib).max() <= 0.5 + 255 * 4 / 4096 + 1e-6


def test_resize_within_tap_range():
    rng = np.random.default_rng(5)
    f = rng.integers(0, 256, (1, 19, 11, 3), dtype=np.uint8)
    dh, dw = 42, 28
    got = op.resize_bilinear_u8(f, dh, dw)
    r0, r1, _ = op.resize_axis_taps(19, dh)
    c0, c1, _ = op.resize_axis_taps(11, dw)
    taps = np.stack([f[0][r0][:, c0], f[0][r0][:, c1], f[0][r1][:, c0], f[0][r1][:, c1]])
    assert np.all(got[0] >= taps.min(0)) and np.all(got[0] <= taps.max(0))


def test_axis_taps_properties():
    for ns, nd in [(2, 4), (4, 2), (7, 7), (240, 448), (1080, 224), (3, 1344)]:
        i0, i1, fr = op.resize_axis_taps(ns, nd)
        assert np.all((0 <= i0) & (i0 <= i1) & (i1 <= ns - 1) & (i1 - i0 <= 1))
        assert np.all((0 <= fr) & (fr <= 2048))
        pos = i0 + fr / 2048.0
        assert np.all(np.diff(pos) >= -1e-12)            # monotone sampling positions
        # mirror symmetry of half-pixel sampling: pos[i] + pos[nd-1-i] == ns-1 (up to quantisation)
        assert np.abs(pos + pos[::-1] - (ns - 1)).max() <= 1.0 / 2048 + 1e-12
        if ns == nd:
            assert np.array_equal(i0, np.arange(ns)) and np.all(fr == 0)


def test_normalise_closed_form_all_values():
    v = np.arange(256, dtype=np.uint8)
    u = np.stack([v, v, v], -1)
    x = op.normalise(u, (0.5,) * 3, (0.5,) * 3, "f32")
    closed = (2.0 * v.astype(np.float64) / 255.0 - 1.0).astype(np.float32)
    for c in range(3):
        assert np.array_equal(x[:, c], closed)
    assert x[0, 0] == -1.0 and x[255, 0] == 1.0
    assert np.all(np.diff(x[:, 0]) > 0)
    # antisymmetry of the closed form: x(v) = -x(255 - v)
    assert np.array_equal(x[:, 0], -x[::-1, 0])
    # general mean / std: compare with exact rationals
    from fractions import Fraction
    mean, std = (0.485, 0.456, 0.406), (0.229, 0.224, 0.225)
    y = op.normalise(u, mean, std, "f32")
    for c in range(3):
        for vv in (0, 1, 77, 128, 255):
            exact = (Fraction(vv, 255) - Fraction(mean[c])) / Fraction(std[c])
            assert abs(float(y[vv, c]) - float(exact)) <= abs(float(exact)) * 2 ** -23 + 1e-12


def test_bf16_rounding_against_torch_and_cases():
    rng = np.random.default_rng(3)
    x = np.concatenate([rng.normal(0, 1, 4096), rng.normal(0, 1e-3, 1024), [0.0, -0.0, 1.0, -1.0]]).astype(np.float32)
    got = op.round_to_bf16(x)
    lib = torch.from_numpy(x).to(torch.bfloat16).float().numpy()
    assert np.array_equal(got.view(np.uint32), lib.view(np.uint32))
    # ties to even: 1 + 2^-8 is halfway between 1 and 1 + 2^-7 -> 1 ; 1 + 3*2^-8 -> 1 + 2^-6
    assert op.round_to_bf16(np.float32(1 + 2 ** -8)) == np.float32(1.0)
    assert op.round_to_bf16(np.float32(1 + 3 * 2 ** -8)) == np.float32(1 + 2 ** -6)
    # normalised pixels in bf16 take at most 256 values and stay monotone
    v = np.arange(256, dtype=np.uint8)
    xb = op.normalise(np.stack([v] * 3, -1), (0.5,) * 3, (0.5,) * 3, "bf16")[:, 0]
    assert np.all(np.diff(xb) >= 0) and np.all((xb.view(np.uint32) & 0xFFFF) == 0)


@pytest.mark.parametrize("patch,tpatch,merge,n,h,w", [(14, 1, 1, 1, 42, 70), (16, 1, 1, 3, 48, 32),
                                                      (14, 2, 2, 4, 56, 84), (14, 2, 2, 6, 28, 28),
                                                      (4, 2, 2, 2, 24, 8), (2, 3, 1, 6, 6, 10)])
def test_patchify_roundtrip_bit_exact(patch, tpatch, merge, n, h, w):
    rng = np.random.default_rng(7)
    x = rng.integers(0, 256, (n, h, w, 3), dtype=np.uint8)
    rows = op.patchify(x, patch, tpatch, merge)
    assert rows.shape == ((n // tpatch) * (h // patch) * (w // patch), 3 * tpatch * patch * patch)
    back = op.unpatchify(rows, n, h, w, patch, tpatch, merge)
    assert np.array_equal(back, x)


def test_patchify_image_is_duplicated_to_temporal_patch():
    rng = np.random.default_rng(8)
    x = rng.integers(0, 256, (1, 28, 56, 3), dtype=np.uint8)
    rows = op.patchify(x, 14, 2, 2).reshape(-1, 3, 2, 14, 14)
    assert np.array_equal(rows[:, :, 0], rows[:, :, 1])
    assert np.array_equal(rows[:, :, 0].reshape(-1, 3 * 14 * 14), op.patchify(x, 14, 1, 2))


def test_patch_row_layout_brute_force():
    """Element k of token row r is pixel (frame, y, x, c) given by explicit index arithmetic."""
    patch, tpatch, merge, n, h, w = 4, 2, 2, 4, 16, 24
    x = np.arange(n * h * w * 3, dtype=np.int64).reshape(n, h, w, 3)
    rows = op.patchify(x, patch, tpatch, merge)
    gh, gw = h // patch, w // patch
    r = 0
    for t in range(n // tpatch):
        for hb in range(gh // 2):
            for wb in range(gw // 2):
                for hi in range(2):
                    for wi in range(2):
                        ph, pw = 2 * hb + hi, 2 * wb + wi
                        for c in range(3):
                            for tt in range(tpatch):
                                for py in range(patch):
                                    for px in range(patch):
                                        k = ((c * tpatch + tt) * patch + py) * patch + px
                                        assert rows[r, k] == x[t * tpatch + tt, ph * patch + py, pw * patch + px, c]
                        r += 1
    assert r == rows.shape[0]


def test_merge_groups_are_consecutive_rows():
    co = op.token_coords(3, 4, 6, 2)
    assert co.shape == (72, 3)
    for g in range(18):
        blk = co[4 * g:4 * g + 4]
        assert len(set(blk[:, 0])) == 1
        hb, wb = blk[0, 1] // 2, blk[0, 2] // 2
        assert sorted(map(tuple, blk[:, 1:])) == [(2 * hb, 2 * wb), (2 * hb, 2 * wb + 1),
                                                  (2 * hb + 1, 2 * wb), (2 * hb + 1, 2 * wb + 1)]
    # raster order for merge=1, every coordinate exactly once in both orders
    co1 = op.token_coords(2, 3, 5, 1)
    assert [tuple(c) for c in co1] == [(t, h, w) for t in range(2) for h in range(3) for w in range(5)]
    assert len({tuple(c) for c in co}) == 72


def test_token_counts_of_the_workloads():
    """Fixed-resolution images give a constant token count (the near-vertical
    line of Sec. 2.2); text requests give none."""
    import workloads
    from oracle import encoder
    wl = workloads.full_config(1, with_frames=False, with_weights=False)
    assert encoder.cu_seqlens_of(encoder.grids_of(wl.items, wl.desc), 1).tolist() == [0, 197]
    wl = workloads.full_config(2, with_frames=False, with_weights=False)
    cu = encoder.cu_seqlens_of(encoder.grids_of(wl.items, wl.desc), 0)
    assert np.all(np.diff(cu) == 576) and cu[-1] == 18432
    wl = workloads.full_config(3, with_frames=False, with_weights=False)
    cu = encoder.cu_seqlens_of(encoder.grids_of(wl.items, wl.desc), 0)
    assert cu[-1] == sum((i.dst_h // 14) * (i.dst_w // 14) for i in wl.items)
    assert np.diff(cu).min() >= 256 and np.diff(cu).max() <= 9216 and np.all(np.diff(cu) % 4 == 0)
    wl = workloads.full_config(4, with_frames=False, with_weights=False)
    assert encoder.cu_seqlens_of(encoder.grids_of(wl.items, wl.desc), 0).tolist() == [0, 32768]
    wl = workloads.full_config(5, with_frames=False, with_weights=False)
    cu = encoder.cu_seqlens_of(encoder.grids_of(wl.items, wl.desc), 0)
    assert cu[1] == 16384 and cu[2] == 32768 and np.all(np.diff(cu)[26:] == 0) and len(cu) == 227


def test_video_as_frames_shares_patch_halves_with_the_video():
    """Feeding a video frame by frame (Sec. 4.1, "Models") repeats every frame over the
    temporal patch; the video pairs consecutive frames.  So row r of the video's
    frame pair j holds, in its first temporal slot, what image 2j holds there, and
    in its second slot what image 2j+1 holds there."""
    import workloads
    vid, seq = workloads.small_config(4), workloads.small_config(6)
    assert len(seq.items) == vid.items[0].n_frames
    pv = op.preprocess_item(vid.items[0], vid.desc)
    P, tp = vid.desc.patch, vid.desc.tpatch
    n = (vid.items[0].dst_h // P) * (vid.items[0].dst_w // P)        # rows per frame pair / per image
    pv = pv.reshape(-1, n, 3, tp, P * P)
    for j in range(pv.shape[0]):
        a = op.preprocess_item(seq.items[2 * j], seq.desc).reshape(n, 3, tp, P * P)
        b = op.preprocess_item(seq.items[2 * j + 1], seq.desc).reshape(n, 3, tp, P * P)
        assert np.array_equal(pv[j][:, :, 0], a[:, :, 0]) and np.array_equal(pv[j][:, :, 1], b[:, :, 1])
        assert np.array_equal(a[:, :, 0], a[:, :, 1])
    wl = workloads.full_config(6, with_frames=False, with_weights=False)
    from oracle import encoder
    cu = encoder.cu_seqlens_of(encoder.grids_of(wl.items, wl.desc), 0)
    assert len(cu) == 65 and np.all(np.diff(cu) == 1024)


def test_bad_shapes_raise():
    with pytest.raises(ValueError):
        op.token_grid(1, 1, 30, 28, 14, 2, 2)
    with pytest.raises(ValueError):
        op.token_grid(2, 3, 28, 28, 14, 2, 2)
    assert op.token_grid(0, 0, 0, 0, 14, 2, 2) == (0, 0, 0)
