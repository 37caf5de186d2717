"""CPU reference for the vision encoder and the merge/projector
(TEST INFRASTRUCTURE ONLY).

The paper's "vision encoding" stage (Sec. 2.1, Fig. 1) turns preprocessed
patches into embeddings "in a unified format" for the LLM; the encoders it
serves are ViT variants (Table 1).  The paper gives no arithmetic, so this file
is the textbook pre-LN ViT written out, evaluated in one floating-point type
(`dtype`, default float64) with no intermediate rounding:

  embed     X = patches @ W_pe.T + b_pe ; optional CLS row first in each
            segment ; position term added per row
  block     x = x + Attn(LN1(x)) @ W_o.T + b_o
            x = x + GELU(LN2(x) @ W_1.T + b_1) @ W_2.T + b_2        (x L)
  LN        (x - mean)/sqrt(var + eps) * gamma + beta, biased variance over d
  Attn      [q|k|v] = h @ W_qkv.T + b_qkv, head j = columns [j*dh, (j+1)*dh) of
            each third; softmax(q k^T / sqrt(dh)) v over the keys of the SAME
            segment (request) only, all keys visible (bidirectional)
  GELU      x/2 * (1 + erf(x/sqrt 2))
  final LN  optional
  merge     LN_m(x); each group of merge^2 consecutive rows is concatenated
            into one row of width merge^2*d; out = GELU(Y @ W_m1.T + b_m1) @ W_m2.T + b_m2

Variants (encoder families of Table 1 differ in these; every switch is a field of
the model description, the defaults give the block above):
  norm = "rms"     RMSNorm  x / sqrt(mean(x^2) + eps) * gamma  wherever LN stands above
  gated = 1        MLP  (silu(h W_g^T + b_g) * (h W_u^T + b_u)) W_2^T + b_2, silu(x) = x/(1+e^-x);
                   w_1 holds W_g in its first mlp rows and W_u in the last mlp rows
  pos = "rope2d"   no additive position term; instead q and k of every head are rotated:
                   element pairs (2p, 2p+1), p < dh/2; the first dh/4 pairs turn by
                   h * theta^(-p/(dh/4)), the others by w * theta^(-(p-dh/4)/(dh/4)),
                   (h, w) = patch coordinate of the token (all frames of a video share it)
  window = W       tokens are ordered window by window (oracle/preprocess.token_coords);
                   layers attend inside each W x W window of a frame group, except layers l
                   with (l+1) % full_every == 0, which attend over the whole segment

Library primitives used as steps: numpy matmul, scipy.special.erf.  Attention
is evaluated in blocks of query rows only to bound memory; every row still
gets a full-row, max-subtracted softmax.

Pins (tests/test_oracle_encoder.py): softmax rows sum to 1; single-key segment
returns V; zero queries return mean(V); agreement with a pure-Python triple
loop (oracle/naive.py); permutation equivariance without position terms;
segment independence; LN output statistics; GELU identities and tabulated erf
values; L=0 reduces to one library GEMM; zeroed W_o / W_2 make blocks the
identity; merge view against a brute-force gather; and the whole path frames ->
hidden -> projector output against models put together from torch.nn library
modules only (Conv2d / Conv3d patch embedding, nn.TransformerEncoder with
norm_first and exact GELU, nn.LayerNorm, unfold for the 2x2 grouping), for the
CLS + learned-position family, the separable-position video family and the
2x2-merge + projector family.  The variant switches have their own pins
(tests/test_oracle_variants.py).  The paper prints no output values of any
encoder, so there is nothing of the paper's to compare with beyond these.
"""
from __future__ import annotations

from typing import Dict, List, Sequence

import numpy as np
from scipy.special import erf

from .preprocess import token_coords, token_grid


def layernorm(x, gamma, beta, eps):
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps) * gamma + beta


def rmsnorm(x, gamma, eps):
    return x / np.sqrt((x ** 2).mean(axis=-1, keepdims=True) + eps) * gamma


def norm(desc, x, gamma, beta):
    """The normalisation the model uses (LayerNorm or RMSNorm; RMSNorm has no beta)."""
    if getattr(desc, "norm", "layer") == "rms":
        return rmsnorm(x, gamma, desc.ln_eps)
    return layernorm(x, gamma, beta, desc.ln_eps)


def gelu(x):
    return 0.5 * x * (1.0 + erf(x / np.sqrt(2.0)))


def silu(x):
    return x / (1.0 + np.exp(-x))


def rope_angles(coords_hw, dh, theta):
    """[T, dh/2] rotation angle of every element pair of a head, from the (h, w) patch
    coordinate of every row: first dh/4 pairs follow h, the others w."""
    if dh % 4:
        raise ValueError("rotary positions need a head size that is a multiple of 4")
    n_ax = dh // 4
    freq = theta ** (-np.arange(n_ax, dtype=np.float64) / n_ax)
    hw = np.asarray(coords_hw, np.float64)
    return np.concatenate([hw[:, 0:1] * freq[None, :], hw[:, 1:2] * freq[None, :]], axis=1)


def rope_rotate(x, angles, heads):
    """x [T, d]: rotates pairs (2p, 2p+1) of every head by angles[:, p]."""
    T, d = x.shape
    dh = d // heads
    xr = x.reshape(T, heads, dh // 2, 2)
    c = np.cos(angles)[:, None, :].astype(x.dtype)
    sn = np.sin(angles)[:, None, :].astype(x.dtype)
    out = np.empty_like(xr)
    out[..., 0] = xr[..., 0] * c - xr[..., 1] * sn
    out[..., 1] = xr[..., 0] * sn + xr[..., 1] * c
    return out.reshape(T, d)


def softmax_rows(s):
    s = s - s.max(axis=-1, keepdims=True)
    p = np.exp(s)
    return p / p.sum(axis=-1, keepdims=True)


def attend(q_rows, kk, vv, scale, return_probs=False):
    """softmax(q k^T * scale) v for some query rows against ALL keys kk / values vv
    of their segment (one head)."""
    p = softmax_rows((q_rows @ kk.T) * scale)
    return (p @ vv, p) if return_probs else p @ vv


def attention(q, k, v, cu_seqlens: Sequence[int], heads: int, q_block: int = 1024,
              return_probs: bool = False, rows=None, workers: int = 1):
    """q, k, v: [T, d].  Block-diagonal bidirectional attention: rows
    cu_seqlens[i]:cu_seqlens[i+1] form segment i.  With `rows` (sorted global
    row indices) only those query rows are evaluated and returned, in order.
    `workers` > 1 evaluates the (independent) heads on a thread pool; the
    arithmetic of every head is unchanged."""
    T, d = q.shape
    if workers > 1 and rows is None and not return_probs:
        from concurrent.futures import ThreadPoolExecutor
        dh = d // heads
        out = np.zeros_like(q)

        def one(h):
            c = slice(h * dh, (h + 1) * dh)
            out[:, c] = attention(q[:, c], k[:, c], v[:, c], cu_seqlens, 1, q_block)
        with ThreadPoolExecutor(workers) as ex:
            list(ex.map(one, range(heads)))
        return out
    dh = d // heads
    scale = 1.0 / np.sqrt(dh)
    if rows is not None:
        rows = np.asarray(rows, np.int64)
        out = np.zeros((len(rows), d), q.dtype)
        seg = np.searchsorted(np.asarray(cu_seqlens), rows, side="right") - 1
        for s in np.unique(seg):
            a, b = int(cu_seqlens[s]), int(cu_seqlens[s + 1])
            sel = np.nonzero(seg == s)[0]
            for h in range(heads):
                c = slice(h * dh, (h + 1) * dh)
                out[sel, c] = attend(q[rows[sel], c], k[a:b, c], v[a:b, c], scale)
        return out
    out = np.zeros_like(q)
    probs = []
    for s in range(len(cu_seqlens) - 1):
        a, b = int(cu_seqlens[s]), int(cu_seqlens[s + 1])
        if b == a:
            continue
        for h in range(heads):
            c = slice(h * dh, (h + 1) * dh)
            kk, vv = k[a:b, c], v[a:b, c]
            for r in range(a, b, q_block):
                r1 = min(b, r + q_block)
                if return_probs:
                    out[r:r1, c], p = attend(q[r:r1, c], kk, vv, scale, True)
                    probs.append(p)
                else:
                    out[r:r1, c] = attend(q[r:r1, c], kk, vv, scale)
    return (out, probs) if return_probs else out


def position_rows(desc, items_grids, weights, dtype):
    """Position term for every hidden row (incl. CLS rows), in row order."""
    chunks = []
    for (gt, gh, gw) in items_grids:
        n = gt * gh * gw
        if n == 0:
            continue
        rows = n + (1 if desc.use_cls else 0)
        if desc.pos == "learned1d":
            chunks.append(weights["pos0"][:rows].astype(dtype))
        elif desc.pos == "sep2d":
            co = token_coords(gt, gh, gw, desc.merge, getattr(desc, "window", 0))
            pr = weights["pos0"][co[:, 1]].astype(dtype) + weights["pos1"][co[:, 2]].astype(dtype)
            if desc.use_cls:
                pr = np.concatenate([np.zeros((1, desc.d), dtype), pr], 0)
            chunks.append(pr)
        else:
            chunks.append(np.zeros((rows, desc.d), dtype))
    if not chunks:
        return np.zeros((0, desc.d), dtype)
    return np.concatenate(chunks, 0)


def grids_of(items, desc):
    return [token_grid(it.modality, it.n_frames, it.dst_h, it.dst_w, desc.patch, desc.tpatch, desc.merge)
            for it in items]


def cu_seqlens_of(grids, use_cls) -> np.ndarray:
    cu = [0]
    for (gt, gh, gw) in grids:
        n = gt * gh * gw
        cu.append(cu[-1] + (n + (1 if (use_cls and n) else 0)))
    return np.asarray(cu, np.int64)


def coords_hw_of(grids, desc) -> np.ndarray:
    """(h, w) patch coordinate of every hidden row, in row order (models without CLS rows)."""
    chunks = [token_coords(gt, gh, gw, desc.merge, getattr(desc, "window", 0))[:, 1:3]
              for (gt, gh, gw) in grids if gt * gh * gw]
    return np.concatenate(chunks, 0) if chunks else np.zeros((0, 2), np.int64)


def window_cu_seqlens_of(grids, desc) -> np.ndarray:
    """Cumulative row counts of the attention windows of all requests, in row order."""
    from .preprocess import window_lengths
    cu = [0]
    for (gt, gh, gw) in grids:
        if gt * gh * gw:
            for n in window_lengths(gt, gh, gw, desc.window):
                cu.append(cu[-1] + n)
    return np.asarray(cu, np.int64)


def layer_is_windowed(desc, l) -> bool:
    if not getattr(desc, "window", 0):
        return False
    fe = getattr(desc, "full_every", 0)
    return not (fe and (l + 1) % fe == 0)


def embed(patches_per_item: List[np.ndarray], grids, desc, weights, dtype=np.float64):
    """Patch embedding + CLS + position term -> hidden rows [T, d]."""
    wpe = weights["w_pe"].astype(dtype)
    bpe = weights["b_pe"].astype(dtype)
    segs = []
    for p, (gt, gh, gw) in zip(patches_per_item, grids):
        if gt * gh * gw == 0:
            continue
        x = p.astype(dtype) @ wpe.T + bpe
        if desc.use_cls:
            x = np.concatenate([weights["cls"].astype(dtype)[None, :], x], 0)
        segs.append(x)
    if not segs:
        return np.zeros((0, desc.d), dtype)
    x = np.concatenate(segs, 0)
    return x + position_rows(desc, grids, weights, dtype)


def encoder_block(x, cu, desc, weights, l, dtype=np.float64, rows=None, workers=1, rope=None, cu_win=None):
    """One pre-norm block.  With `rows`, only those output rows are computed (the
    keys and values of every row are still needed and are computed).  `rope`: rotation
    angles [T, dh/2] for models with rotary positions; `cu_win`: window boundaries for
    models with windowed attention (used by the layers layer_is_windowed names)."""
    g = lambda n: weights[f"l{l}.{n}"].astype(dtype)
    d = desc.d
    h = norm(desc, x, g("ln1_g"), g("ln1_b"))
    qkv = h @ g("w_qkv").T + g("b_qkv")
    q, k, v = qkv[:, :d], qkv[:, d:2 * d], qkv[:, 2 * d:]
    if rope is not None:
        q, k = rope_rotate(q, rope, desc.heads), rope_rotate(k, rope, desc.heads)
    seg = cu_win if layer_is_windowed(desc, l) else cu
    o = attention(q, k, v, seg, desc.heads, rows=rows, workers=workers)
    if rows is not None:
        x = x[np.asarray(rows, np.int64)]
    x = x + (o @ g("w_o").T + g("b_o"))
    h = norm(desc, x, g("ln2_g"), g("ln2_b"))
    u = h @ g("w_1").T + g("b_1")
    if getattr(desc, "gated", 0):
        h = silu(u[:, :desc.mlp]) * u[:, desc.mlp:]
    else:
        h = gelu(u)
    x = x + (h @ g("w_2").T + g("b_2"))
    return x


def layout_of(grids, desc, dtype=np.float64):
    """Per-row quantities the blocks of a variant model need: (rope angles or None, window
    boundaries or None)."""
    rope = cu_win = None
    if desc.pos == "rope2d":
        if desc.use_cls:
            raise ValueError("rotary positions are defined for models without a CLS row")
        rope = rope_angles(coords_hw_of(grids, desc), desc.d // desc.heads, desc.rope_theta).astype(dtype)
    if getattr(desc, "window", 0):
        if desc.use_cls:
            raise ValueError("windowed attention is defined for models without a CLS row")
        cu_win = window_cu_seqlens_of(grids, desc)
    return rope, cu_win


def encode(patches_per_item, grids, desc, weights, dtype=np.float64, progress=None, workers=1):
    """Patches of every request -> encoder output [T, d] (segments concatenated
    in request order; requests without frames contribute no rows)."""
    cu = cu_seqlens_of(grids, desc.use_cls)
    rope, cu_win = layout_of(grids, desc, dtype)
    x = embed(patches_per_item, grids, desc, weights, dtype)
    for l in range(desc.layers):
        x = encoder_block(x, cu, desc, weights, l, dtype, workers=workers, rope=rope, cu_win=cu_win)
        if progress:
            progress(l)
    if desc.final_ln:
        x = norm(desc, x, weights["lnf_g"].astype(dtype), weights["lnf_b"].astype(dtype))
    return x


def merge_project(x, desc, weights, dtype=np.float64):
    """Encoder output [T, d] -> [T/merge^2, out_dim]."""
    g = lambda n: weights[n].astype(dtype)
    m2 = desc.merge * desc.merge
    y = norm(desc, x.astype(dtype), g("lnm_g"), g("lnm_b"))
    y = y.reshape(x.shape[0] // m2, m2 * desc.d)
    y = gelu(y @ g("w_m1").T + g("b_m1"))
    return y @ g("w_m2").T + g("b_m2")
