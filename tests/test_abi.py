"""CPU-only checks of the C-ABI library: it loads, exports every symbol the
header declares, validates descriptions and shapes, and its host-side plan
(token order, cumulative lengths, index maps) agrees with the CPU reference."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import workloads
from oracle import encoder as oe
from oracle import preprocess as op
from paper_2603_26498_amd import binding as B
from paper_2603_26498_amd.runtime import VisionEncoder

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "tcmv.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(tcmv_[a-z0-9_]+)\s*\(", hdr))
    assert declared, "no declarations found"
    assert declared == set(B.SIGNATURES), declared ^ set(B.SIGNATURES)
    lib = C.CDLL(B.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name
    assert B.tcmv_version() >= 100
    assert B.error_name(-2) == "TCMV_E_BAD_SHAPE"


def test_library_exports_every_scheduler_symbol():
    from paper_2603_26498_amd import sched_binding as SB
    hdr = open(os.path.join(ROOT, "include", "tcms.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(tcms_[a-z0-9_]+)\s*\(", hdr))
    assert declared == set(SB.SIGNATURES), declared ^ set(SB.SIGNATURES)
    lib = C.CDLL(B.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name
    assert C.sizeof(SB.tcms_cluster_model) == 10 * 8 and C.sizeof(SB.tcms_regulator) == 9 * 8


def test_struct_sizes_match_header_layout():
    assert C.sizeof(B.tcmv_model_desc) == 13 * 4 + 4 + 24 + 4 * 4 + 4 + 4 + 4
    assert C.sizeof(B.tcmv_item) == 6 * 4 + 8
    assert C.sizeof(B.tcmv_weights) == 14 * 8


def test_description_validation():
    with pytest.raises(B.TcmvError) as e:
        B.tcmv_create(B.make_desc(dtype="bf16", layers=1, d=100, heads=3, mlp=64))
    assert e.value.code == B.TCMV_E_INVALID_ARG
    with pytest.raises(B.TcmvError) as e:
        B.tcmv_create(B.make_desc(dtype="bf16", layers=1, d=192, heads=4, mlp=256))      # head size 48
    assert e.value.code == B.TCMV_E_UNSUPPORTED and "head size" in str(e.value)
    with pytest.raises(B.TcmvError):
        B.tcmv_create(B.make_desc(dtype="f32", layers=1, d=64, heads=1, mlp=64, merge=3))
    ctx = B.tcmv_create(B.make_desc(dtype="f32", layers=1, d=64, heads=1, mlp=64, patch=7))
    assert B.tcmv_k_pad(B.make_desc(dtype="f32", layers=1, d=64, heads=1, mlp=64, patch=7)) == 148
    B.tcmv_destroy(ctx)
    assert B.tcmv_k_pad(B.make_desc(dtype="bf16", layers=1, d=64, heads=1, mlp=64, patch=14)) == 640
    assert B.tcmv_k_pad(B.make_desc(dtype="bf16", layers=1, d=64, heads=1, mlp=64, patch=14, tpatch=2)) == 1216


def _plan(desc, items):
    enc = VisionEncoder(desc)
    return enc, enc.plan(items, upload=False)


@pytest.mark.parametrize("idx", [1, 2, 3, 4, 5, 6, 7])
def test_plan_matches_reference_token_order(idx):
    wl = workloads.small_config(idx)
    enc, pl = _plan(wl.desc, wl.items)
    grids = oe.grids_of(wl.items, wl.desc)
    cu = oe.cu_seqlens_of(grids, wl.desc.use_cls)
    assert pl.cu_seqlens == cu.tolist()
    assert pl.info.n_tokens == cu[-1]
    assert pl.info.n_patch_rows == sum(g[0] * g[1] * g[2] for g in grids)
    assert pl.info.k == wl.desc.k and pl.info.k_pad % 2 == 0 and pl.info.k_pad >= wl.desc.k
    thw = pl.row_map(0)
    dst = pl.row_map(1)
    ref = np.concatenate([op.token_coords(*g, wl.desc.merge, wl.desc.window) for g in grids if g[0]] or [np.zeros((0, 3), int)])
    assert np.array_equal(thw >> 16, ref[:, 0]) and np.array_equal((thw >> 8) & 255, ref[:, 1])
    assert np.array_equal(thw & 255, ref[:, 2])
    # destination rows: patch rows in order, skipping one CLS row at the start of each segment
    exp, r = [], 0
    for g in grids:
        n = g[0] * g[1] * g[2]
        if n:
            r += 1 if wl.desc.use_cls else 0
            exp += list(range(r, r + n))
            r += n
    assert dst.tolist() == exp
    pos = pl.row_map(2)
    if wl.desc.pos == "sep2d":
        assert np.array_equal(pos & 0xFFFF, ref[:, 1]) and np.array_equal(pos >> 16, ref[:, 2])
    elif wl.desc.pos == "learned1d":
        seg0 = np.searchsorted(cu, dst, side="right") - 1
        assert np.array_equal(pos, dst - cu[seg0])
    m2 = wl.desc.merge ** 2
    assert pl.info.n_out_tokens == (cu[-1] // m2 if wl.desc.out_dim else 0)
    assert pl.info.hidden_bytes == cu[-1] * wl.desc.d * 4


def test_full_size_token_counts():
    """Plan sizes of the full workloads (no frames needed on the host)."""
    expect = {1: 197, 2: 18432, 4: 32768, 6: 65536, 7: 32768}
    for idx in (1, 2, 3, 4, 5, 6, 7):
        wl = workloads.full_config(idx, with_frames=False, with_weights=False)
        enc, pl = _plan(wl.desc, wl.items)
        cu = oe.cu_seqlens_of(oe.grids_of(wl.items, wl.desc), wl.desc.use_cls)
        assert pl.cu_seqlens == cu.tolist()
        if idx in expect:
            assert pl.info.n_tokens == expect[idx]
        if idx == 5:
            assert pl.info.n_segments == 26 and pl.info.n_items == 226
            assert all(a == b for a, b in zip(pl.cu_seqlens[26:], pl.cu_seqlens[27:]))   # text: no tokens


def test_bad_shapes_are_rejected():
    desc = workloads.qwen_like_desc(layers=1, d=320, heads=4, mlp=640, out_dim=192, max_grid=16)
    enc = VisionEncoder(desc)
    I = workloads.Item
    for bad in ([I(1, 1, 30, 28, 30, 28)],            # not a multiple of patch*merge
                [I(1, 1, 28, 28, 0, 28)],             # empty target
                [I(2, 3, 28, 28, 28, 28)],            # odd video length with temporal patch 2
                [I(1, 1, 28, 28, 28 * 17, 28)],       # grid side above the position table
                [I(1, 1, 0, 28, 28, 28)]):            # empty source
        with pytest.raises(B.TcmvError) as e:
            enc.plan(bad, upload=False)
        assert e.value.code == B.TCMV_E_BAD_SHAPE, bad
    with pytest.raises(B.TcmvError) as e:
        enc.plan([I(7, 1, 28, 28, 28, 28)], upload=False)
    assert e.value.code == B.TCMV_E_INVALID_ARG
    # empty and text-only plans are valid and empty
    for items in ([], [I(0, 0, 0, 0, 0, 0)] * 3):
        pl = enc.plan(items, upload=False)
        assert pl.info.n_tokens == 0 and pl.info.n_patch_rows == 0 and pl.cu_seqlens == [0] * (len(items) + 1)
    # more tokens than the kernels' 32-bit element offsets allow (tokens x widest row below 2^32): 14 images of
    # 254 x 254 patches with rows up to 5120 wide; one fewer image fits
    big = workloads.qwen_like_desc(layers=1, max_grid=254)
    side = 254 * 14
    with pytest.raises(B.TcmvError) as e:
        VisionEncoder(big).plan([I(1, 1, side, side, side, side)] * 14, upload=False)
    assert e.value.code == B.TCMV_E_BAD_SHAPE and "2^32" in str(e.value)
    assert VisionEncoder(big).plan([I(1, 1, side, side, side, side)] * 12, upload=False).info.n_tokens == 12 * 254 * 254
    # learned 1-D table too short
    d2 = workloads.ModelDesc(dtype="bf16", layers=1, d=128, heads=2, mlp=128, patch=14, pos="learned1d", max_pos=3)
    with pytest.raises(B.TcmvError) as e:
        VisionEncoder(d2).plan([I(1, 1, 28, 28, 28, 28)], upload=False)
    assert e.value.code == B.TCMV_E_BAD_SHAPE


def test_device_calls_fail_cleanly_without_weights_or_gpu():
    desc = workloads.qwen_like_desc(layers=1, d=320, heads=4, mlp=640, out_dim=192, max_grid=16)
    enc = VisionEncoder(desc)
    pl = enc.plan([workloads.Item(1, 1, 28, 28, 28, 28)], upload=False)
    rc = B.lib().tcmv_encode(enc.ctx, pl.handle, 256, 256, 256, 256, 1 << 30, None)
    assert rc == B.TCMV_E_NO_WEIGHTS
    rc = B.lib().tcmv_preprocess(enc.ctx, pl.handle, 256, 256, None)     # item has a null frame pointer
    assert rc == B.TCMV_E_INVALID_ARG
    assert "frame pointer" in B.tcmv_last_error(enc.ctx)
    assert B.tcmv_op_attention_workspace(B.TCMV_BF16, [0, 100, 100, 164], 128, 2) > 0


def test_plan_metadata_belongs_to_the_caller():
    """The library hands out the plan's index metadata as host bytes and never allocates device memory itself: the
    stage calls take the caller's device copy, and refuse a missing, misaligned or short one."""
    desc = workloads.qwen_like_desc(layers=1, d=320, heads=4, mlp=640, out_dim=192, max_grid=16)
    enc = VisionEncoder(desc)
    item = workloads.Item(1, 1, 28, 28, 28, 28)
    pl = enc.plan([item], upload=False)
    assert pl.meta is None and pl.info.meta_bytes > 0 and pl.info.meta_bytes % 256 == 0
    blob = B.tcmv_plan_meta(pl.handle)
    assert len(blob) == pl.info.meta_bytes
    # the normalisation table (3 x 256 values, bf16-representable for a bf16 model) is part of it
    tab = np.array([((v / 255.0) - 0.5) / 0.5 for v in range(256)], np.float32)
    tab = (tab.view(np.uint32) + 0x7FFF + ((tab.view(np.uint32) >> 16) & 1) & 0xFFFF0000).astype(np.uint32).view(np.float32)
    assert blob.find(tab.tobytes()) >= 0
    # an empty plan needs no metadata
    empty = enc.plan([workloads.Item(0, 0, 0, 0, 0, 0)], upload=False)
    assert empty.info.meta_bytes == 0 and B.tcmv_plan_meta(empty.handle) == b""
    assert B.lib().tcmv_plan_upload(empty.handle, None, 0, None) == B.TCMV_OK
    # argument checks come before any device work
    assert B.lib().tcmv_plan_upload(pl.handle, None, pl.info.meta_bytes, None) == B.TCMV_E_INVALID_ARG
    assert B.lib().tcmv_plan_upload(pl.handle, 256 + 16, pl.info.meta_bytes, None) == B.TCMV_E_INVALID_ARG
    assert B.lib().tcmv_plan_upload(pl.handle, 256, pl.info.meta_bytes - 1, None) == B.TCMV_E_WORKSPACE_TOO_SMALL
    assert B.lib().tcmv_plan_upload(None, 256, 0, None) == B.TCMV_E_INVALID_ARG
    rc = B.lib().tcmv_preprocess(enc.ctx, pl.handle, None, 256, None)
    assert rc == B.TCMV_E_INVALID_ARG


def test_attention_index_is_host_data():
    cu = [0, 100, 100, 164]
    n = B.lib().tcmv_op_attention_index_bytes(B.TCMV_BF16, (C.c_int64 * 4)(*cu), 3, 128, 2)
    assert n > 0 and n % 256 == 0
    idx = B.tcmv_op_attention_index(B.TCMV_BF16, cu, 128, 2)
    assert len(idx) == n
    vcol = np.frombuffer(idx[:164 * 4], np.int32)
    # every row has its own column in the transposed-V buffer; the second non-empty segment starts at a multiple of 64
    assert len(set(vcol.tolist())) == 164 and vcol[:100].max() < 128 and vcol[100:].min() == 128
    buf = C.create_string_buffer(16)
    assert B.lib().tcmv_op_attention_index(B.TCMV_BF16, (C.c_int64 * 4)(*cu), 3, 128, 2, buf, 16) == B.TCMV_E_WORKSPACE_TOO_SMALL
    assert B.lib().tcmv_op_attention_index_bytes(B.TCMV_BF16, (C.c_int64 * 4)(0, 5, 3, 9), 3, 128, 2) == 0


def test_windowed_plan_whose_transposed_values_do_not_fit_32_bit_offsets_is_refused():
    """Every window is padded to 64 columns of the transposed values, so a plan with small windows needs far more
    columns than it has tokens; the offset guard must count them."""
    desc = workloads.ModelDesc(dtype="bf16", layers=1, d=2048, heads=32, mlp=2048, patch=14, tpatch=1, merge=1,
                               pos="none", window=2, full_every=0)
    enc = VisionEncoder(desc)
    # 8 x 8 grids: 16 windows of 4 tokens -> 1024 columns for 64 tokens
    items = [workloads.Item(1, 1, 112, 112, 112, 112)] * 3000
    with pytest.raises(B.TcmvError) as e:
        enc.plan(items, upload=False)
    assert e.value.code == B.TCMV_E_BAD_SHAPE and "transposed" in str(e.value)
    assert enc.plan(items[:1000], upload=False).info.n_tokens == 1000 * 64
