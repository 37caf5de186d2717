"""CPU reference for vision preprocessing (TEST INFRASTRUCTURE ONLY).

This is the checker for the "vision preprocessing" stage the paper places in
front of the vision encoder (Sec. 2.1 "Multimodal LLM Architecture", Fig. 1;
the Workload Profiler of Sec. 3.2 times it separately).  The paper fixes no
arithmetic for it; the readings implemented here are:

  resize     integer bilinear, half-pixel centres, edge clamp, no antialias,
             11-bit fractional weights, one rounding at the end;
  normalise  x = (v/255 - mean_c)/std_c evaluated in double, rounded once to
             fp32 and, for bf16 models, once more to bf16 (ties to even);
  patchify   Sec. 2.2 has the image cut into a grid of equally sized patches:
             frames are taken in groups of `tpatch` (a still image is repeated
             `tpatch` times); tokens are ordered (t, h, w) for merge=1 and
             (t, h//2, w//2, h%2, w%2) for merge=2 so that each 2x2 merge group
             is four consecutive rows; inside a row the element order is
             (channel, frame-in-group, patch row, patch column).

Plain numpy, written for legibility, not speed.  Nothing here is used by the
GPU library; only tests, the smoke check and the benchmark's CPU-baseline leg
may import it.

Pins (tests/test_oracle_preprocess.py): identity resize, constant images,
tap-range bound, hand-worked 2x2->4x4 and 4x4->2x2 examples
(tests/golden/resize_examples.txt), exact-2x downscale = rounded block mean,
normalise == 2v/255-1 closed form, patchify/unpatchify round trip and a
brute-force index map.
"""
from __future__ import annotations

import numpy as np

FRAC_BITS = 11
ONE = 1 << FRAC_BITS


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """fp32 -> nearest bf16 (ties to even), returned as fp32."""
    u = np.asarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    u = (u + 0x7FFF + lsb) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32)


def resize_axis_taps(n_src: int, n_dst: int):
    """For each destination index: the two source indices and the weight of the
    second one in units of 1/2048.  Destination pixel centre (i+0.5) maps to
    source coordinate (i+0.5)*n_src/n_dst - 0.5, clamped to [0, n_src-1]."""
    i0 = np.zeros(n_dst, np.int64)
    i1 = np.zeros(n_dst, np.int64)
    fr = np.zeros(n_dst, np.int64)
    den = 2 * n_dst
    for i in range(n_dst):
        num = max(0, (2 * i + 1) * n_src - n_dst)
        a = num // den
        f = ((num % den) * ONE + den // 2) // den
        if a >= n_src - 1:
            a, b, f = n_src - 1, n_src - 1, 0
        else:
            b = a + 1
        i0[i], i1[i], fr[i] = a, b, f
    return i0, i1, fr


def resize_bilinear_u8(frames: np.ndarray, dst_h: int, dst_w: int) -> np.ndarray:
    """frames uint8 [n, Hs, Ws, 3] -> uint8 [n, dst_h, dst_w, 3]."""
    n, hs, ws, c = frames.shape
    r0, r1, fy = resize_axis_taps(hs, dst_h)
    c0, c1, fx = resize_axis_taps(ws, dst_w)
    fy = fy[:, None, None]
    fx = fx[None, :, None]
    out = np.empty((n, dst_h, dst_w, c), np.uint8)
    for k in range(n):                      # frame by frame only to bound memory
        f = frames[k].astype(np.int64)
        a = f[r0][:, c0]
        b = f[r0][:, c1]
        cc = f[r1][:, c0]
        e = f[r1][:, c1]
        acc = (a * (ONE - fx) * (ONE - fy) + b * fx * (ONE - fy)
               + cc * (ONE - fx) * fy + e * fx * fy + (1 << (2 * FRAC_BITS - 1)))
        out[k] = (acc >> (2 * FRAC_BITS)).astype(np.uint8)
    return out


def normalise(u8: np.ndarray, mean, std, dtype: str) -> np.ndarray:
    """uint8 [..., 3] -> fp32 values of (v/255 - mean_c)/std_c (bf16-rounded for
    dtype == 'bf16')."""
    v = u8.astype(np.float64) / 255.0
    x = (v - np.asarray(mean, np.float64)) / np.asarray(std, np.float64)
    x = x.astype(np.float32)
    if dtype == "bf16":
        x = round_to_bf16(x)
    return x


def token_grid(modality: int, n_frames: int, h: int, w: int, patch: int, tpatch: int, merge: int):
    """(gt, gh, gw) for one item; raises ValueError for shapes the method does
    not define (non-multiples, odd video length)."""
    if n_frames == 0:
        return (0, 0, 0)
    if h % (patch * merge) or w % (patch * merge) or h <= 0 or w <= 0:
        raise ValueError("target size must be a positive multiple of patch*merge")
    if n_frames == 1:
        gt = 1
    else:
        if n_frames % tpatch:
            raise ValueError("video length must be a multiple of the temporal patch")
        gt = n_frames // tpatch
    return (gt, h // patch, w // patch)


def token_coords(gt: int, gh: int, gw: int, merge: int, window: int = 0) -> np.ndarray:
    """[T, 3] int array: (t, h, w) patch coordinate of every token row, in token order.
    window == 0: per frame group, merge groups in raster order, rows of a group consecutive.
    window > 0 (a multiple of merge): per frame group, windows of window x window patches in
    raster order (clipped at the right and bottom edges), the same merge-group order inside
    each window; every window is then a contiguous run of rows."""
    out = []
    if window and window % merge:
        raise ValueError("window must be a multiple of merge")
    wh = window if window else max(gh, 1)
    ww = window if window else max(gw, 1)
    for t in range(gt):
        for h0 in range(0, gh, wh):
            for w0 in range(0, gw, ww):
                h1, w1 = min(gh, h0 + wh), min(gw, w0 + ww)
                for hb in range(h0, h1, merge):
                    for wb in range(w0, w1, merge):
                        for hi in range(merge):
                            for wi in range(merge):
                                out.append((t, hb + hi, wb + wi))
    return np.asarray(out, np.int64).reshape(-1, 3)


def window_lengths(gt: int, gh: int, gw: int, window: int):
    """Number of tokens of every window of one request, in token order."""
    out = []
    for _ in range(gt):
        for h0 in range(0, gh, window):
            for w0 in range(0, gw, window):
                out.append((min(gh, h0 + window) - h0) * (min(gw, w0 + window) - w0))
    return out


def patchify(x: np.ndarray, patch: int, tpatch: int, merge: int, window: int = 0) -> np.ndarray:
    """x [n_frames, H, W, 3] (any dtype) -> [T, 3*tpatch*patch*patch].
    A single frame is repeated tpatch times."""
    n, h, w, c = x.shape
    assert c == 3
    if n == 1 and tpatch > 1:
        x = np.repeat(x, tpatch, axis=0)
        n = tpatch
    gt, gh, gw = n // tpatch, h // patch, w // patch
    coords = token_coords(gt, gh, gw, merge, window)
    rows = np.empty((coords.shape[0], 3 * tpatch * patch * patch), x.dtype)
    for r, (t, ph, pw) in enumerate(coords):
        blk = x[t * tpatch:(t + 1) * tpatch, ph * patch:(ph + 1) * patch, pw * patch:(pw + 1) * patch, :]
        rows[r] = blk.transpose(3, 0, 1, 2).reshape(-1)     # (c, tt, py, px)
    return rows


def unpatchify(rows: np.ndarray, n_frames: int, h: int, w: int, patch: int, tpatch: int, merge: int) -> np.ndarray:
    """Inverse of patchify for n_frames that is a multiple of tpatch."""
    gt, gh, gw = n_frames // tpatch, h // patch, w // patch
    coords = token_coords(gt, gh, gw, merge)
    x = np.empty((n_frames, h, w, 3), rows.dtype)
    for r, (t, ph, pw) in enumerate(coords):
        blk = rows[r].reshape(3, tpatch, patch, patch).transpose(1, 2, 3, 0)
        x[t * tpatch:(t + 1) * tpatch, ph * patch:(ph + 1) * patch, pw * patch:(pw + 1) * patch, :] = blk
    return x


def preprocess_item(item, desc) -> np.ndarray:
    """One request -> normalised patch rows [T_patches, K] (fp32 container)."""
    gt, gh, gw = token_grid(item.modality, item.n_frames, item.dst_h, item.dst_w,
                            desc.patch, desc.tpatch, desc.merge)
    if gt == 0:
        return np.zeros((0, desc.k), np.float32)
    f = item.frames
    if (item.src_h, item.src_w) != (item.dst_h, item.dst_w):
        f = resize_bilinear_u8(f, item.dst_h, item.dst_w)
    x = normalise(f, desc.mean, desc.std, desc.dtype)
    return patchify(x, desc.patch, desc.tpatch, desc.merge, getattr(desc, "window", 0))
