"""ctypes binding of libtcmv.so: same names as include/tcmv.h, argument
marshalling only.  Every step of the path runs in the library's HIP kernels;
there is no fallback: if the library is missing, loading raises."""
from __future__ import annotations

import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libtcmv.so")

TCMV_F32, TCMV_BF16 = 0, 1
TCMV_POS_NONE, TCMV_POS_LEARNED_1D, TCMV_POS_SEPARABLE_2D, TCMV_POS_ROTARY_2D = 0, 1, 2, 3
TCMV_NORM_LAYER, TCMV_NORM_RMS = 0, 1
TCMV_TEXT, TCMV_IMAGE, TCMV_VIDEO = 0, 1, 2
TCMV_OK = 0
TCMV_E_INVALID_ARG, TCMV_E_BAD_SHAPE, TCMV_E_WORKSPACE_TOO_SMALL = -1, -2, -3
TCMV_E_NO_WEIGHTS, TCMV_E_HIP, TCMV_E_UNSUPPORTED = -4, -5, -6
EPI_STORE, EPI_GELU, EPI_RESID, EPI_GATED = 0, 1, 2, 5

LAYER_FIELDS = ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o", "ln2_g", "ln2_b", "w_1", "b_1", "w_2", "b_2")


class tcmv_model_desc(C.Structure):
    _fields_ = [("dtype", C.c_int), ("layers", C.c_int), ("d", C.c_int), ("heads", C.c_int), ("mlp", C.c_int),
                ("patch", C.c_int), ("tpatch", C.c_int), ("merge", C.c_int), ("out_dim", C.c_int),
                ("use_cls", C.c_int), ("pos", C.c_int), ("max_pos", C.c_int), ("final_ln", C.c_int),
                ("ln_eps", C.c_float), ("mean", C.c_float * 3), ("std", C.c_float * 3),
                ("norm", C.c_int), ("mlp_gated", C.c_int), ("window", C.c_int), ("full_every", C.c_int),
                ("rope_theta", C.c_float), ("head_dim", C.c_int), ("attn_scale", C.c_float)]


class tcmv_item(C.Structure):
    _fields_ = [("modality", C.c_int), ("n_frames", C.c_int), ("src_h", C.c_int), ("src_w", C.c_int),
                ("dst_h", C.c_int), ("dst_w", C.c_int), ("d_frames", C.c_void_p)]


class tcmv_weights(C.Structure):
    _fields_ = [("w_pe", C.c_void_p), ("b_pe", C.c_void_p), ("cls", C.c_void_p), ("pos0", C.c_void_p),
                ("pos1", C.c_void_p), ("layer", C.POINTER(C.c_void_p)),
                ("lnf_g", C.c_void_p), ("lnf_b", C.c_void_p), ("lnm_g", C.c_void_p), ("lnm_b", C.c_void_p),
                ("w_m1", C.c_void_p), ("b_m1", C.c_void_p), ("w_m2", C.c_void_p), ("b_m2", C.c_void_p)]


class tcmv_plan_info(C.Structure):
    _fields_ = [("n_patch_rows", C.c_int64), ("n_tokens", C.c_int64), ("n_out_tokens", C.c_int64),
                ("k", C.c_int64), ("k_pad", C.c_int64),
                ("patches_bytes", C.c_size_t), ("hidden_bytes", C.c_size_t), ("out_bytes", C.c_size_t),
                ("encode_workspace_bytes", C.c_size_t), ("merge_workspace_bytes", C.c_size_t),
                ("n_items", C.c_int), ("n_segments", C.c_int), ("meta_bytes", C.c_size_t)]


class TcmvError(RuntimeError):
    def __init__(self, code, where, detail=""):
        self.code = code
        super().__init__(f"{where}: {error_name(code)} ({code}) {detail}")


# name -> (restype, argtypes); the list of symbols include/tcmv.h declares
SIGNATURES = {
    "tcmv_version": (C.c_int, []),
    "tcmv_error_name": (C.c_char_p, [C.c_int]),
    "tcmv_k_pad": (C.c_int64, [C.POINTER(tcmv_model_desc)]),
    "tcmv_create": (C.c_int, [C.POINTER(tcmv_model_desc), C.POINTER(C.c_void_p)]),
    "tcmv_destroy": (None, [C.c_void_p]),
    "tcmv_last_error": (C.c_char_p, [C.c_void_p]),
    "tcmv_set_weights": (C.c_int, [C.c_void_p, C.POINTER(tcmv_weights)]),
    "tcmv_plan_create": (C.c_int, [C.c_void_p, C.POINTER(tcmv_item), C.c_int, C.POINTER(C.c_void_p)]),
    "tcmv_plan_destroy": (None, [C.c_void_p]),
    "tcmv_plan_query": (C.c_int, [C.c_void_p, C.POINTER(tcmv_plan_info)]),
    "tcmv_plan_cu_seqlens": (C.POINTER(C.c_int64), [C.c_void_p]),
    "tcmv_plan_row_map": (C.c_int64, [C.c_void_p, C.c_int, C.POINTER(C.POINTER(C.c_int32))]),
    "tcmv_plan_meta": (C.c_void_p, [C.c_void_p, C.POINTER(C.c_size_t)]),
    "tcmv_plan_upload": (C.c_int, [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
    "tcmv_preprocess": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "tcmv_encode": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t,
                              C.c_void_p]),
    "tcmv_merge_project": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t,
                                     C.c_void_p]),
    "tcmv_profile_enable": (C.c_int, [C.c_void_p, C.c_int]),
    "tcmv_profile_read": (C.c_int, [C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_int64)]),
    "tcmv_op_layernorm": (C.c_int, [C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int,
                                    C.c_float, C.c_void_p]),
    "tcmv_op_stream": (C.c_int, [C.c_void_p, C.c_size_t, C.c_void_p, C.c_size_t, C.c_void_p]),
    "tcmv_op_gemm": (C.c_int, [C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int,
                               C.c_int, C.c_void_p]),
    "tcmv_op_attention_workspace": (C.c_size_t, [C.c_int, C.POINTER(C.c_int64), C.c_int, C.c_int, C.c_int]),
    "tcmv_op_attention_index_bytes": (C.c_size_t, [C.c_int, C.POINTER(C.c_int64), C.c_int, C.c_int, C.c_int]),
    "tcmv_op_attention_index": (C.c_int, [C.c_int, C.POINTER(C.c_int64), C.c_int, C.c_int, C.c_int, C.c_void_p,
                                          C.c_size_t]),
    "tcmv_op_attention": (C.c_int, [C.c_int, C.c_void_p, C.POINTER(C.c_int64), C.c_int, C.c_int, C.c_int, C.c_void_p,
                                    C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
    "tcmv_op_attention_noalloc": (C.c_int, [C.c_int, C.c_void_p, C.POINTER(C.c_int64), C.c_int, C.c_int, C.c_int,
                                            C.c_void_p, C.c_void_p, C.c_void_p]),
}
TCMV_NOALLOC_SCRATCH_BYTES = 16 << 20

_lib = None


def lib():
    """The loaded library.  Raises if libtcmv.so has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2603_26498_amd.build` "
                               "(there is no fallback path)")
        l = C.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(l, name)
            fn.restype = res
            fn.argtypes = args
        _lib = l
    return _lib


def error_name(code: int) -> str:
    return lib().tcmv_error_name(code).decode()


def make_desc(dtype="bf16", layers=0, d=0, heads=1, mlp=0, patch=14, tpatch=1, merge=1, out_dim=0, use_cls=0,
              pos="none", max_pos=0, final_ln=0, ln_eps=1e-6, mean=(0.5, 0.5, 0.5), std=(0.5, 0.5, 0.5),
              norm="layer", gated=0, window=0, full_every=0, rope_theta=10000.0, head_dim=0, attn_scale=0.0):
    m = tcmv_model_desc()
    m.dtype = {"f32": TCMV_F32, "bf16": TCMV_BF16}[dtype] if isinstance(dtype, str) else int(dtype)
    m.layers, m.d, m.heads, m.mlp = layers, d, heads, mlp
    m.patch, m.tpatch, m.merge, m.out_dim = patch, tpatch, merge, out_dim
    m.use_cls = use_cls
    m.pos = {"none": 0, "learned1d": 1, "sep2d": 2, "rope2d": 3}[pos] if isinstance(pos, str) else int(pos)
    m.norm = {"layer": 0, "rms": 1}[norm] if isinstance(norm, str) else int(norm)
    m.mlp_gated, m.window, m.full_every, m.rope_theta = int(gated), int(window), int(full_every), float(rope_theta)
    m.max_pos, m.final_ln, m.ln_eps = max_pos, final_ln, ln_eps
    m.head_dim, m.attn_scale = int(head_dim), float(attn_scale)
    for i in range(3):
        m.mean[i] = mean[i]
        m.std[i] = std[i]
    return m


def _ptr(t):
    """Device (or host) address of a torch tensor / int / None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


# ---- thin wrappers with the C names ------------------------------------------------------------
def tcmv_version():
    return lib().tcmv_version()


def tcmv_k_pad(desc):
    return lib().tcmv_k_pad(C.byref(desc))


def tcmv_create(desc):
    out = C.c_void_p()
    rc = lib().tcmv_create(C.byref(desc), C.byref(out))
    if rc != TCMV_OK:
        raise TcmvError(rc, "tcmv_create", lib().tcmv_last_error(None).decode())
    return out


def tcmv_destroy(ctx):
    lib().tcmv_destroy(ctx)


def tcmv_last_error(ctx):
    return lib().tcmv_last_error(ctx).decode()


def _check(ctx, rc, where):
    if rc != TCMV_OK:
        raise TcmvError(rc, where, tcmv_last_error(ctx) if ctx else "")


def tcmv_set_weights(ctx, w: tcmv_weights):
    _check(ctx, lib().tcmv_set_weights(ctx, C.byref(w)), "tcmv_set_weights")


def tcmv_plan_create(ctx, items):
    """items: sequence of (modality, n_frames, src_h, src_w, dst_h, dst_w, device_ptr_or_None)."""
    n = len(items)
    arr = (tcmv_item * max(n, 1))()
    for i, it in enumerate(items):
        arr[i].modality, arr[i].n_frames, arr[i].src_h, arr[i].src_w, arr[i].dst_h, arr[i].dst_w = it[:6]
        arr[i].d_frames = _ptr(it[6])
    out = C.c_void_p()
    _check(ctx, lib().tcmv_plan_create(ctx, arr, n, C.byref(out)), "tcmv_plan_create")
    return out


def tcmv_plan_destroy(plan):
    lib().tcmv_plan_destroy(plan)


def tcmv_plan_query(plan) -> tcmv_plan_info:
    info = tcmv_plan_info()
    rc = lib().tcmv_plan_query(plan, C.byref(info))
    if rc != TCMV_OK:
        raise TcmvError(rc, "tcmv_plan_query")
    return info


def tcmv_plan_cu_seqlens(plan, n_items):
    p = lib().tcmv_plan_cu_seqlens(plan)
    return [p[i] for i in range(n_items + 1)]


def tcmv_plan_row_map(plan, which):
    import numpy as np
    p = C.POINTER(C.c_int32)()
    n = lib().tcmv_plan_row_map(plan, which, C.byref(p))
    if n < 0:
        raise TcmvError(int(n), "tcmv_plan_row_map")
    if n == 0:
        return np.zeros(0, np.int32)
    return np.ctypeslib.as_array(p, shape=(n,)).copy()


def tcmv_plan_meta(plan) -> bytes:
    """Host copy of the plan's index metadata (what tcmv_plan_upload copies)."""
    n = C.c_size_t()
    p = lib().tcmv_plan_meta(plan, C.byref(n))
    return C.string_at(p, n.value) if p and n.value else b""


def tcmv_plan_upload(ctx, plan, d_meta, meta_bytes, stream=None):
    _check(ctx, lib().tcmv_plan_upload(plan, _ptr(d_meta), meta_bytes, stream), "tcmv_plan_upload")


def tcmv_preprocess(ctx, plan, d_meta, d_patches, stream=None):
    _check(ctx, lib().tcmv_preprocess(ctx, plan, _ptr(d_meta), _ptr(d_patches), stream), "tcmv_preprocess")


def tcmv_encode(ctx, plan, d_meta, d_patches, d_hidden, d_workspace, workspace_bytes, stream=None):
    _check(ctx, lib().tcmv_encode(ctx, plan, _ptr(d_meta), _ptr(d_patches), _ptr(d_hidden), _ptr(d_workspace),
                                  workspace_bytes, stream), "tcmv_encode")


def tcmv_merge_project(ctx, plan, d_hidden, d_out, d_workspace, workspace_bytes, stream=None):
    _check(ctx, lib().tcmv_merge_project(ctx, plan, _ptr(d_hidden), _ptr(d_out), _ptr(d_workspace), workspace_bytes,
                                         stream), "tcmv_merge_project")


KERNEL_CLASSES = ("preprocess", "embed_gemm", "layernorm", "qkv_gemm", "attention", "out_gemm", "fc1_gemm",
                  "fc2_gemm", "merge_gemm", "other")


def tcmv_profile_enable(ctx, classes):
    """classes: bit mask over KERNEL_CLASSES (bit i = class i), -1 or True for all, 0 / False for off."""
    classes = -1 if classes is True else int(classes)
    _check(ctx, lib().tcmv_profile_enable(ctx, classes), "tcmv_profile_enable")


def tcmv_profile_read(ctx):
    """-> {kernel class: (milliseconds, launches)} since the last read."""
    n = len(KERNEL_CLASSES)
    ms = (C.c_double * n)()
    cnt = (C.c_int64 * n)()
    _check(ctx, lib().tcmv_profile_read(ctx, ms, cnt), "tcmv_profile_read")
    return {KERNEL_CLASSES[i]: (ms[i], cnt[i]) for i in range(n)}


def tcmv_op_layernorm(dtype, d_x, d_gamma, d_beta, d_y, rows, d, eps, stream=None):
    rc = lib().tcmv_op_layernorm(dtype, _ptr(d_x), _ptr(d_gamma), _ptr(d_beta), _ptr(d_y), rows, d, eps, stream)
    if rc != TCMV_OK:
        raise TcmvError(rc, "tcmv_op_layernorm")


def tcmv_op_stream(d_in, in_bytes, d_out, out_bytes, stream=None):
    rc = lib().tcmv_op_stream(_ptr(d_in), in_bytes, _ptr(d_out), out_bytes, stream)
    if rc != TCMV_OK:
        raise TcmvError(rc, "tcmv_op_stream")


def tcmv_op_gemm(dtype, epilogue, d_a, d_w, d_bias, d_c, m, n, k, stream=None):
    rc = lib().tcmv_op_gemm(dtype, epilogue, _ptr(d_a), _ptr(d_w), _ptr(d_bias), _ptr(d_c), m, n, k, stream)
    if rc != TCMV_OK:
        raise TcmvError(rc, "tcmv_op_gemm")


def tcmv_op_attention_workspace(dtype, cu_seqlens, d, heads):
    n = len(cu_seqlens) - 1
    arr = (C.c_int64 * (n + 1))(*cu_seqlens)
    return lib().tcmv_op_attention_workspace(dtype, arr, n, d, heads)


def tcmv_op_attention_index(dtype, cu_seqlens, d, heads) -> bytes:
    """The index data of tcmv_op_attention for these segment lengths, as host bytes (the caller uploads them)."""
    n = len(cu_seqlens) - 1
    arr = (C.c_int64 * (n + 1))(*cu_seqlens)
    nbytes = lib().tcmv_op_attention_index_bytes(dtype, arr, n, d, heads)
    if nbytes == 0:
        raise TcmvError(TCMV_E_INVALID_ARG, "tcmv_op_attention_index_bytes")
    buf = C.create_string_buffer(nbytes)
    rc = lib().tcmv_op_attention_index(dtype, arr, n, d, heads, buf, nbytes)
    if rc != TCMV_OK:
        raise TcmvError(rc, "tcmv_op_attention_index")
    return buf.raw


def tcmv_op_attention(dtype, d_qkv, cu_seqlens, d, heads, d_index, d_out, d_workspace, workspace_bytes, stream=None):
    n = len(cu_seqlens) - 1
    arr = (C.c_int64 * (n + 1))(*cu_seqlens)
    rc = lib().tcmv_op_attention(dtype, _ptr(d_qkv), arr, n, d, heads, _ptr(d_index), _ptr(d_out), _ptr(d_workspace),
                                 workspace_bytes, stream)
    if rc != TCMV_OK:
        raise TcmvError(rc, "tcmv_op_attention")


def tcmv_op_attention_noalloc(dtype, d_qkv, cu_seqlens, d, heads, d_index, d_out, stream=None):
    n = len(cu_seqlens) - 1
    arr = (C.c_int64 * (n + 1))(*cu_seqlens)
    rc = lib().tcmv_op_attention_noalloc(dtype, _ptr(d_qkv), arr, n, d, heads, _ptr(d_index), _ptr(d_out), stream)
    if rc != TCMV_OK:
        raise TcmvError(rc, "tcmv_op_attention_noalloc")
