"""Host-side layout steps of the Python runtime (no GPU): zero padding of head sizes and MLP widths the
kernels do not have, interleaving of gated MLP weights."""
import numpy as np
import pytest

import workloads
from paper_2603_26498_amd.runtime import VisionEncoder


def test_head_and_mlp_padding_keeps_every_entry_and_adds_only_zeros():
    wl = workloads.small_config(9)                       # d=576, 8 heads of 72, mlp 296
    d = wl.desc
    enc = VisionEncoder(d)                               # host only: no weights uploaded
    assert (enc.dh, enc.dh_lib, enc.mlp_lib) == (72, 80, 320)
    assert enc.cdesc.head_dim == 80 and enc.cdesc.mlp == 320
    assert abs(enc.cdesc.attn_scale - 1.0 / np.sqrt(72)) < 1e-7
    w = wl.weights
    qkv = enc._lib_layout("w_qkv", w["l0.w_qkv"])
    assert qkv.shape == (3 * 8 * 80, 576)
    q4 = qkv.reshape(3, 8, 80, 576)
    assert np.array_equal(q4[:, :, :72], w["l0.w_qkv"].reshape(3, 8, 72, 576)) and not q4[:, :, 72:].any()
    b = enc._lib_layout("b_qkv", w["l0.b_qkv"]).reshape(3, 8, 80)
    assert np.array_equal(b[:, :, :72], w["l0.b_qkv"].reshape(3, 8, 72)) and not b[:, :, 72:].any()
    wo = enc._lib_layout("w_o", w["l0.w_o"]).reshape(576, 8, 80)
    assert np.array_equal(wo[:, :, :72], w["l0.w_o"].reshape(576, 8, 72)) and not wo[:, :, 72:].any()
    w1 = enc._lib_layout("w_1", w["l0.w_1"])
    assert w1.shape == (320, 576) and np.array_equal(w1[:296], w["l0.w_1"]) and not w1[296:].any()
    w2 = enc._lib_layout("w_2", w["l0.w_2"])
    assert w2.shape == (576, 320) and np.array_equal(w2[:, :296], w["l0.w_2"]) and not w2[:, 296:].any()
    # the padded model computes the same function: scores and the MLP sum only gain zero terms
    rng = np.random.default_rng(0)
    x = rng.normal(size=(5, 576))
    q_true = (x @ w["l0.w_qkv"][:576].T).reshape(5, 8, 72)
    q_pad = (x @ qkv[:640].T).reshape(5, 8, 80)
    assert np.allclose(np.einsum("thd,shd->hts", q_true, q_true), np.einsum("thd,shd->hts", q_pad, q_pad))
    h_true, h_pad = x @ w["l0.w_1"].T, x @ w1.T
    assert np.allclose(h_true @ w["l0.w_2"].T, h_pad @ w2.T)


def test_gated_weights_are_interleaved_and_padded_in_pairs():
    desc = workloads.windowed_desc(layers=1, d=128, heads=2, mlp=96, out_dim=64, window=4, full_every=0)
    enc = VisionEncoder(desc)
    assert enc.mlp_lib == 128 and enc.dh_lib == 0
    w = workloads.make_weights(desc, 5)
    w1 = enc._lib_layout("w_1", w["l0.w_1"])             # caller: gate rows, then up rows
    assert w1.shape == (256, 128)
    assert np.array_equal(w1[0:192:2], w["l0.w_1"][:96]) and np.array_equal(w1[1:192:2], w["l0.w_1"][96:])
    assert not w1[192:].any()
    assert enc._lib_layout("w_2", w["l0.w_2"]).shape == (128, 128)


def test_head_sizes_without_a_kernel_and_without_padding_room_are_refused():
    desc = workloads.ModelDesc(dtype="bf16", layers=1, d=1024, heads=8, mlp=256)      # heads of 128
    with pytest.raises(ValueError):
        VisionEncoder(desc)
