"""Seeded synthetic inputs for the vision preprocess + ViT-encode path.

This module only *generates data*: request lists (raw uint8 frames with the
shapes and size mixes of the paper's image / video / text workloads, Sec. 2.2
"Characterization in Isolation" and Sec. 4.1 "Workloads") and random model
parameters.  It contains none of the method's arithmetic and is the one module
shared by the CPU checker and the GPU library's tests and benchmark.

Conventions (fixed here, used by every consumer):
  * frames: uint8, RGB interleaved, shape [n_frames, src_h, src_w, 3].
  * linear weights: shape [out_features, in_features] (row-major, the
    contraction dimension is contiguous), y = x @ W.T + b.
  * "bf16" models: every parameter is drawn in fp32 and then snapped to the
    nearest bf16-representable value (ties to even), still stored as fp32, so
    a later conversion to bf16 storage is exact.
"""
from __future__ import annotations

from dataclasses import dataclass, field, asdict
from typing import Dict, List, Optional

import numpy as np

TEXT, IMAGE, VIDEO = 0, 1, 2


@dataclass
class ModelDesc:
    dtype: str = "bf16"          # "f32" | "bf16"
    layers: int = 2
    d: int = 128
    heads: int = 2
    mlp: int = 512
    patch: int = 14
    tpatch: int = 1
    merge: int = 1               # 1 or 2 (2x2 spatial merge)
    out_dim: int = 0             # 0 = no projector
    use_cls: int = 0
    pos: str = "none"            # "none" | "learned1d" | "sep2d" | "rope2d"
    max_pos: int = 0             # rows of the position table(s)
    final_ln: int = 0
    ln_eps: float = 1e-6
    mean: tuple = (0.5, 0.5, 0.5)
    std: tuple = (0.5, 0.5, 0.5)
    norm: str = "layer"          # "layer" | "rms"
    gated: int = 0               # 1: MLP is silu(x W_gate) * (x W_up), then W_down
    window: int = 0              # attention window side in patches (0 = none); tokens are then ordered window by window
    full_every: int = 0          # with windows: layers l with (l+1) % full_every == 0 attend over the whole segment
    rope_theta: float = 10000.0  # base of the rotary angles (pos == "rope2d")

    @property
    def k(self) -> int:
        return 3 * self.tpatch * self.patch * self.patch

    @property
    def dh(self) -> int:
        return self.d // self.heads

    def asdict(self):
        return asdict(self)


@dataclass
class Item:
    modality: int
    n_frames: int
    src_h: int
    src_w: int
    dst_h: int
    dst_w: int
    frames: Optional[np.ndarray] = None   # uint8 [n_frames, src_h, src_w, 3]


@dataclass
class Workload:
    name: str
    desc: ModelDesc
    items: List[Item]
    weights: Dict[str, np.ndarray] = field(default_factory=dict)


# ----------------------------------------------------------------------------
# value helpers (data generation only)
# ----------------------------------------------------------------------------
def snap_to_bf16_grid(x: np.ndarray) -> np.ndarray:
    """Nearest bf16-representable fp32 value, ties to even (no NaN handling)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def random_frames(rng: np.random.Generator, n: int, h: int, w: int) -> np.ndarray:
    return rng.integers(0, 256, size=(n, h, w, 3), dtype=np.uint8)


LAYER_FIELDS = ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o",
                "ln2_g", "ln2_b", "w_1", "b_1", "w_2", "b_2")


def make_weights(desc: ModelDesc, seed: int, *, std: float = 0.02,
                 random_affine: bool = False) -> Dict[str, np.ndarray]:
    """Random parameters.  Default: matrices / CLS / position tables N(0, std),
    biases 0, LayerNorm gamma 1 and beta 0.  With random_affine=True the biases
    are N(0, 0.1) and gamma / beta are drawn around 1 / 0 so that every bias and
    affine term is exercised by tests."""
    rng = np.random.default_rng(seed)
    d, f, k = desc.d, desc.mlp, desc.k

    def mat(o, i):
        return rng.normal(0.0, std, size=(o, i)).astype(np.float32)

    def bias(n):
        if random_affine:
            return rng.normal(0.0, 0.1, size=n).astype(np.float32)
        return np.zeros(n, np.float32)

    def gamma(n):
        if random_affine:
            return (1.0 + rng.normal(0.0, 0.2, size=n)).astype(np.float32)
        return np.ones(n, np.float32)

    w: Dict[str, np.ndarray] = {}
    w["w_pe"] = mat(d, k)
    w["b_pe"] = bias(d)
    if desc.use_cls:
        w["cls"] = rng.normal(0.0, std, size=d).astype(np.float32)
    if desc.pos == "learned1d":
        w["pos0"] = mat(desc.max_pos, d)
    elif desc.pos == "sep2d":
        w["pos0"] = mat(desc.max_pos, d)
        w["pos1"] = mat(desc.max_pos, d)
    for l in range(desc.layers):
        p = f"l{l}."
        w[p + "ln1_g"] = gamma(d); w[p + "ln1_b"] = bias(d)
        w[p + "w_qkv"] = mat(3 * d, d); w[p + "b_qkv"] = bias(3 * d)
        w[p + "w_o"] = mat(d, d); w[p + "b_o"] = bias(d)
        w[p + "ln2_g"] = gamma(d); w[p + "ln2_b"] = bias(d)
        f1 = 2 * f if desc.gated else f            # gated MLP: rows [0, f) gate, rows [f, 2f) up
        w[p + "w_1"] = mat(f1, d); w[p + "b_1"] = bias(f1)
        w[p + "w_2"] = mat(d, f); w[p + "b_2"] = bias(d)
    if desc.final_ln:
        w["lnf_g"] = gamma(d); w["lnf_b"] = bias(d)
    if desc.out_dim:
        dm = d * desc.merge * desc.merge
        w["lnm_g"] = gamma(d); w["lnm_b"] = bias(d)
        w["w_m1"] = mat(dm, dm); w["b_m1"] = bias(dm)
        w["w_m2"] = mat(desc.out_dim, dm); w["b_m2"] = bias(desc.out_dim)
    if desc.dtype == "bf16":
        for key in w:
            w[key] = snap_to_bf16_grid(w[key])
    return w


# ----------------------------------------------------------------------------
# the five workloads (full size) and reduced versions of the same structure
# ----------------------------------------------------------------------------
def _dyn_sizes(rng, n, lo, hi, step):
    """H then W, each uniform over multiples of `step` in [lo, hi]."""
    h = rng.integers(lo // step, hi // step + 1, size=n) * step
    w = rng.integers(lo // step, hi // step + 1, size=n) * step
    return [int(v) for v in h], [int(v) for v in w]


def _source_size(rng, lo=240, hi=1080):
    """One 16:9 source size per item, height uniform in [lo, hi], even width."""
    hs = int(rng.integers(lo, hi + 1))
    ws = 2 * int(round(hs * 8 / 9))
    return hs, ws


def qwen_like_desc(layers=32, d=1280, heads=16, mlp=5120, out_dim=3584, max_grid=96,
                   dtype="bf16") -> ModelDesc:
    return ModelDesc(dtype=dtype, layers=layers, d=d, heads=heads, mlp=mlp, patch=14, tpatch=2,
                     merge=2, out_dim=out_dim, use_cls=0, pos="sep2d", max_pos=max_grid,
                     final_ln=0)


def config1(with_frames=True) -> Workload:
    """One 224x224 image, patch 16, CLS token, 4-layer d=256 fp32 ViT."""
    desc = ModelDesc(dtype="f32", layers=4, d=256, heads=4, mlp=1024, patch=16, tpatch=1, merge=1,
                     out_dim=0, use_cls=1, pos="learned1d", max_pos=197, final_ln=1)
    rng = np.random.default_rng(0)
    it = Item(IMAGE, 1, 224, 224, 224, 224, random_frames(rng, 1, 224, 224) if with_frames else None)
    return Workload("cfg1_image224_vit4x256_f32", desc, [it])


def config2(n_images=32, layers=24, with_frames=True) -> Workload:
    """Batch of fixed-resolution 336x336 images, patch 14, 24-layer d=1024 bf16 ViT."""
    desc = ModelDesc(dtype="bf16", layers=layers, d=1024, heads=16, mlp=4096, patch=14, tpatch=1,
                     merge=1, out_dim=0, use_cls=0, pos="learned1d", max_pos=576, final_ln=1)
    rng = np.random.default_rng(1)
    items = [Item(IMAGE, 1, 336, 336, 336, 336, random_frames(rng, 1, 336, 336) if with_frames else None)
             for _ in range(n_images)]
    return Workload("cfg2_batch32_image336_vit24x1024", desc, items)


def config3(n_images=64, layers=32, lo=224, hi=1344, with_frames=True, desc=None) -> Workload:
    """Dynamic-resolution image batch; H, W multiples of 28; 2x2 merge + projector."""
    desc = desc or qwen_like_desc(layers=layers)
    hs, ws = _dyn_sizes(np.random.default_rng(0), n_images, lo, hi, 28)
    rng = np.random.default_rng(2)
    items = [Item(IMAGE, 1, h, w, h, w, random_frames(rng, 1, h, w) if with_frames else None)
             for h, w in zip(hs, ws)]
    return Workload("cfg3_dynres64_vit32x1280_proj3584", desc, items)


def config4(n_frames=64, side=448, layers=32, with_frames=True, desc=None) -> Workload:
    """One video; temporal patch 2, full attention over all its tokens."""
    desc = desc or qwen_like_desc(layers=layers)
    rng = np.random.default_rng(3)
    it = Item(VIDEO, n_frames, side, side, side, side,
              random_frames(rng, n_frames, side, side) if with_frames else None)
    return Workload("cfg4_video64x448_vit32x1280_proj3584", desc, [it])


def config5(n_videos=2, n_images=24, n_text=200, video_frames=32, video_side=448, layers=32,
            lo=224, hi=1344, src_lo=240, src_hi=1080, with_frames=True, desc=None) -> Workload:
    """Mixed-modality batch (videos, images, text) whose raw frames arrive at
    random 16:9 sizes and are resized to the target before patchify."""
    desc = desc or qwen_like_desc(layers=layers)
    rng_sz = np.random.default_rng(5)
    hs, ws = _dyn_sizes(rng_sz, n_images, lo, hi, 28)
    rng = np.random.default_rng(4)
    items: List[Item] = []
    for _ in range(n_videos):
        sh, sw = _source_size(rng_sz, src_lo, src_hi)
        items.append(Item(VIDEO, video_frames, sh, sw, video_side, video_side,
                          random_frames(rng, video_frames, sh, sw) if with_frames else None))
    for h, w in zip(hs, ws):
        sh, sw = _source_size(rng_sz, src_lo, src_hi)
        items.append(Item(IMAGE, 1, sh, sw, h, w, random_frames(rng, 1, sh, sw) if with_frames else None))
    for _ in range(n_text):
        items.append(Item(TEXT, 0, 0, 0, 0, 0, None))
    return Workload("cfg5_mixed_2video_24image_200text", desc, items)


def config6(n_frames=64, side=448, layers=32, with_frames=True, desc=None) -> Workload:
    """The frames of the config-4 video submitted as a sequence of still images
    (Sec. 4.1, "Models", notes that some models treat a video that way): one request and one
    attention segment per frame, each frame repeated to fill the temporal patch.
    Same pixels and same encoder as config 4, twice the tokens, attention confined
    to 1024-token segments."""
    desc = desc or qwen_like_desc(layers=layers)
    rng = np.random.default_rng(3)
    frames = random_frames(rng, n_frames, side, side) if with_frames else None
    items = [Item(IMAGE, 1, side, side, side, side, frames[i:i + 1] if with_frames else None)
             for i in range(n_frames)]
    return Workload("cfg6_video64x448_as_frames_vit32x1280_proj3584", desc, items)


def windowed_desc(layers=32, d=1280, heads=16, mlp=3456, out_dim=3584, window=8, full_every=8) -> ModelDesc:
    """The encoder family that Table 1 lists as "Custom ViT": RMSNorm, gated MLP, rotary 2-D
    positions, attention inside windows of window x window patches except every
    full_every-th layer.  Same patching and merge as the other image/video workloads."""
    return ModelDesc(dtype="bf16", layers=layers, d=d, heads=heads, mlp=mlp, patch=14, tpatch=2, merge=2,
                     out_dim=out_dim, use_cls=0, pos="rope2d", max_pos=0, final_ln=0, norm="rms", gated=1,
                     window=window, full_every=full_every)


def config7(n_frames=64, side=448, layers=32, with_frames=True, desc=None) -> Workload:
    """The config-4 video through the windowed encoder family: 28 of 32 layers attend inside
    8x8-patch windows (64 tokens), 4 layers over the whole 32768-token video."""
    desc = desc or windowed_desc(layers=layers)
    wl = config4(n_frames=n_frames, side=side, with_frames=with_frames, desc=desc)
    wl.name = "cfg7_video64x448_windowed_vit32x1280_proj3584"
    return wl


def plain_rotary_desc(layers=24, d=1024, heads=16, mlp=4096, out_dim=5120) -> ModelDesc:
    """The third encoder family of Table 1: images of any size cut into 16x16 patches, no
    temporal patch and no spatial merge, rotary 2-D positions, RMSNorm, gated MLP, full
    attention in every layer; a two-layer adapter maps every token to the LLM width."""
    return ModelDesc(dtype="bf16", layers=layers, d=d, heads=heads, mlp=mlp, patch=16, tpatch=1, merge=1,
                     out_dim=out_dim, use_cls=0, pos="rope2d", max_pos=0, final_ln=0, norm="rms", gated=1)


def config8(n_images=16, layers=24, lo=256, hi=1024, with_frames=True, desc=None) -> Workload:
    """A batch of variable-size images (sides multiples of 16) through the merge-free rotary encoder."""
    desc = desc or plain_rotary_desc(layers=layers)
    hs, ws = _dyn_sizes(np.random.default_rng(8), n_images, lo, hi, 16)
    rng = np.random.default_rng(7)
    items = [Item(IMAGE, 1, h, w, h, w, random_frames(rng, 1, h, w) if with_frames else None)
             for h, w in zip(hs, ws)]
    return Workload("cfg8_varsize16_patch16_nomerge_vit24x1024_proj5120", desc, items)


def config9(n_images=32, layers=27, side=384, d=1152, heads=16, mlp=4304, with_frames=True) -> Workload:
    """Fixed-resolution crops through an encoder with the shape of the 400M-parameter fixed-resolution
    encoder that four of the seven models of Table 1 use: patch 14, 27 x 27 = 729 tokens per 384 x 384
    crop, d = 1152, 16 heads of 72, mlp 4304, learned positions, final LayerNorm.  Head size and mlp
    width are not sizes the kernels have: the runtime reaches them by zero padding."""
    g = side // 14
    desc = ModelDesc(dtype="bf16", layers=layers, d=d, heads=heads, mlp=mlp, patch=14, tpatch=1, merge=1,
                     out_dim=0, use_cls=0, pos="learned1d", max_pos=g * g, final_ln=1)
    rng = np.random.default_rng(9)
    px = g * 14
    items = [Item(IMAGE, 1, px, px, px, px, random_frames(rng, 1, px, px) if with_frames else None)
             for _ in range(n_images)]
    return Workload(f"cfg9_batch{n_images}_crop{px}_vit{layers}x{d}_head72", desc, items)


# config 6 runs the config-4 encoder (same weights): only the request structure differs
WEIGHT_SEEDS = {1: 1001, 2: 1002, 3: 1003, 4: 1004, 5: 1005, 6: 1004, 7: 1007, 8: 1008, 9: 1009}


def full_config(idx: int, with_frames=True, with_weights=True, layers=None) -> Workload:
    """The full-size workloads.  `layers` overrides the depth only."""
    kw = {} if layers is None else {"layers": layers}
    if idx == 1:
        wl = config1(with_frames)
        if layers is not None:
            wl.desc.layers = layers
    else:
        wl = {2: config2, 3: config3, 4: config4, 5: config5, 6: config6, 7: config7, 8: config8, 9: config9}[idx](with_frames=with_frames, **kw)
    if with_weights:
        wl.weights = make_weights(wl.desc, WEIGHT_SEEDS[idx])
    return wl


def small_config(idx: int, random_affine=True) -> Workload:
    """Reduced versions with the structure of each full workload (same patching,
    merge, position scheme, CLS / final-LN choices, ragged segment lengths) at a
    size a CPU reference finishes in seconds."""
    if idx == 1:
        wl = config1()
    elif idx == 2:
        desc = ModelDesc(dtype="bf16", layers=2, d=128, heads=2, mlp=512, patch=14, tpatch=1, merge=1,
                         pos="learned1d", max_pos=144, final_ln=1)
        rng = np.random.default_rng(11)
        wl = Workload("small2", desc, [Item(IMAGE, 1, 168, 168, 168, 168, random_frames(rng, 1, 168, 168))
                                       for _ in range(3)])
    elif idx == 3:
        desc = qwen_like_desc(layers=2, d=320, heads=4, mlp=640, out_dim=192, max_grid=16)
        wl = config3(n_images=5, lo=56, hi=224, desc=desc)
    elif idx == 4:
        desc = qwen_like_desc(layers=2, d=320, heads=4, mlp=640, out_dim=192, max_grid=16)
        wl = config4(n_frames=6, side=168, desc=desc)
    elif idx == 5:
        desc = qwen_like_desc(layers=2, d=320, heads=4, mlp=640, out_dim=192, max_grid=16)
        wl = config5(n_videos=1, n_images=3, n_text=4, video_frames=4, video_side=112, lo=56, hi=196,
                     src_lo=60, src_hi=200, desc=desc)
    elif idx == 6:
        desc = qwen_like_desc(layers=2, d=320, heads=4, mlp=640, out_dim=192, max_grid=16)
        wl = config6(n_frames=6, side=168, desc=desc)
    elif idx == 7:
        # the mixed batch (video, images with ragged window edges, text) through the windowed family
        desc = windowed_desc(layers=4, d=320, heads=4, mlp=640, out_dim=192, window=4, full_every=2)
        wl = config5(n_videos=1, n_images=3, n_text=2, video_frames=4, video_side=112, lo=56, hi=196,
                     src_lo=60, src_hi=200, desc=desc)
    elif idx == 8:
        desc = plain_rotary_desc(layers=2, d=256, heads=4, mlp=512, out_dim=192)
        wl = config8(n_images=4, lo=48, hi=240, desc=desc)
    elif idx == 9:
        wl = config9(n_images=3, layers=2, side=84, d=576, heads=8, mlp=296)
    else:
        raise ValueError(idx)
    wl.name = f"small{idx}"
    wl.weights = make_weights(wl.desc, 2000 + idx, random_affine=random_affine)
    return wl
