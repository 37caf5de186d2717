"""GPU parity of the single operators (called through the C ABI) against the
CPU reference, with adversarial inputs that the end-to-end configurations
cannot see: non-zero biases, ragged shapes, peaked softmax, segment leaks."""
import numpy as np
import pytest
import torch

from oracle import encoder as oe
from paper_2603_26498_amd import binding as B
from util import assert_tokens_close, bf16_grid

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a)).to(DEV)
    return t.to(dtype) if dtype is not None else t


def sync():
    torch.cuda.synchronize()


# ---------------------------------------------------------------- LayerNorm
@pytest.mark.parametrize("rows,d", [(1, 256), (7, 160), (197, 256), (1030, 1280), (513, 1024), (33, 2048), (5, 64)])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_layernorm(rows, d, dtype):
    rng = np.random.default_rng(rows * 7 + d)
    x = (rng.normal(0, 3, (rows, d)) + rng.normal(0, 2, (rows, 1))).astype(np.float32)
    g = (1 + rng.normal(0, 0.3, d)).astype(np.float32)
    b = rng.normal(0, 0.2, d).astype(np.float32)
    ref = oe.layernorm(x.astype(np.float64), g.astype(np.float64), b.astype(np.float64), 1e-6)
    y = torch.empty((rows, d), dtype=torch.bfloat16 if dtype == "bf16" else torch.float32, device=DEV)
    B.tcmv_op_layernorm(B.TCMV_BF16 if dtype == "bf16" else B.TCMV_F32, dev(x), dev(g), dev(b), y, rows, d, 1e-6)
    sync()
    got = y.float().cpu().numpy()
    if dtype == "f32":
        assert np.abs(got - ref).max() <= 2e-5 * max(1.0, np.abs(ref).max())
    else:
        assert np.abs(got - ref).max() <= 2 ** -8 * np.abs(ref).max() + 1e-6
        assert_tokens_close(got, ref, 1e-2, 0.9999, "layernorm")


def test_layernorm_in_place_f32():
    rng = np.random.default_rng(3)
    x = rng.normal(0, 1, (37, 256)).astype(np.float32)
    ref = oe.layernorm(x.astype(np.float64), np.ones(256), np.zeros(256), 1e-6)
    t = dev(x)
    B.tcmv_op_layernorm(B.TCMV_F32, t, dev(np.ones(256, np.float32)), dev(np.zeros(256, np.float32)), t, 37, 256, 1e-6)
    sync()
    assert np.abs(t.cpu().numpy() - ref).max() <= 2e-5


# ---------------------------------------------------------------- GEMM
def _gemm_ref(a, w, bias, epi, c0):
    y = a.astype(np.float64) @ w.astype(np.float64).T + (bias.astype(np.float64) if bias is not None else 0)
    if epi == B.EPI_GELU:
        y = oe.gelu(y)
    if epi == B.EPI_RESID:
        y = c0.astype(np.float64) + y
    return y


@pytest.mark.parametrize("m,n,k", [(1, 64, 64), (127, 128, 64), (128, 128, 128), (300, 320, 640), (1000, 1280, 1216),
                                   (257, 136, 192), (129, 3840, 1280), (2050, 1280, 5120),
                                   # 200..511 tiles of 128x128: the mid-size tile kernel (smaller ones use 64x64 tiles)
                                   (2050, 1928, 320), (1500, 2560, 128), (3333, 1280, 192)])
@pytest.mark.parametrize("epi", [B.EPI_STORE, B.EPI_GELU, B.EPI_RESID])
def test_gemm_bf16(m, n, k, epi):
    rng = np.random.default_rng(m + 3 * n + 7 * k + epi)
    a = bf16_grid(rng.normal(0, 1, (m, k)))
    w = bf16_grid(rng.normal(0, 0.05, (n, k)))
    bias = rng.normal(0, 0.5, n).astype(np.float32)
    c0 = rng.normal(0, 1, (m, n)).astype(np.float32)
    ref = _gemm_ref(a, w, bias, epi, c0)
    if epi == B.EPI_RESID:
        c = dev(c0)
    else:
        c = torch.full((m, n), float("nan"), dtype=torch.bfloat16, device=DEV)
    B.tcmv_op_gemm(B.TCMV_BF16, epi, dev(a, torch.bfloat16), dev(w, torch.bfloat16), dev(bias), c, m, n, k)
    sync()
    got = c.float().cpu().numpy()
    if epi == B.EPI_RESID:      # fp32 output: only accumulation-order error
        assert np.abs(got - ref).max() <= 1e-4 * max(1.0, np.abs(ref).max())
    else:
        assert np.abs(got - ref).max() <= 2 ** -8 * np.abs(ref).max() + 1e-5
        assert_tokens_close(got, ref, 1e-2, 0.9999, "gemm")


@pytest.mark.parametrize("m,n,k", [(40000 + 37, 2560, 128), (100000, 1024, 64)])
def test_residual_epilogue_on_an_output_larger_than_the_cache(m, n, k):
    """fp32 outputs above 400 MB take the form of the residual epilogue that requests the old values one group of
    columns ahead (both large tile families, ragged rows); every row is checked."""
    rng = np.random.default_rng(m + n)
    a = bf16_grid(rng.normal(0, 1, (m, k)))
    w = bf16_grid(rng.normal(0, 0.05, (n, k)))
    bias = rng.normal(0, 0.5, n).astype(np.float32)
    c0 = rng.normal(0, 1, (m, n)).astype(np.float32)
    assert m * n * 4 > 400e6
    c = dev(c0)
    B.tcmv_op_gemm(B.TCMV_BF16, B.EPI_RESID, dev(a, torch.bfloat16), dev(w, torch.bfloat16), dev(bias), c, m, n, k)
    sync()
    got = c.cpu().numpy()
    for lo in range(0, m, 8192):                      # reference in slabs: float64 of the whole output would be 0.5 GB
        hi = min(m, lo + 8192)
        ref = _gemm_ref(a[lo:hi], w, bias, B.EPI_RESID, c0[lo:hi])
        assert np.abs(got[lo:hi] - ref).max() <= 1e-4 * max(1.0, np.abs(ref).max()), (lo, hi)


def test_gemm_bf16_no_bias_and_exact_small_integers():
    """Small integer inputs make every product and sum exact: bit-exact result expected."""
    rng = np.random.default_rng(0)
    m, n, k = 200, 192, 128
    a = rng.integers(-3, 4, (m, k)).astype(np.float32)
    w = rng.integers(-3, 4, (n, k)).astype(np.float32)
    c = dev(np.zeros((m, n), np.float32))
    B.tcmv_op_gemm(B.TCMV_BF16, B.EPI_RESID, dev(a, torch.bfloat16), dev(w, torch.bfloat16), None, c, m, n, k)
    sync()
    assert np.array_equal(c.cpu().numpy(), a @ w.T)


@pytest.mark.parametrize("m,n,k", [(1, 1, 1), (197, 256, 768), (70, 100, 50), (197, 1024, 256), (65, 64, 147)])
@pytest.mark.parametrize("epi", [B.EPI_STORE, B.EPI_GELU, B.EPI_RESID])
def test_gemm_f32(m, n, k, epi):
    rng = np.random.default_rng(m + n + k + epi)
    a = rng.normal(0, 1, (m, k)).astype(np.float32)
    w = rng.normal(0, 0.1, (n, k)).astype(np.float32)
    bias = rng.normal(0, 0.5, n).astype(np.float32)
    c0 = rng.normal(0, 1, (m, n)).astype(np.float32)
    ref = _gemm_ref(a, w, bias, epi, c0)
    c = dev(c0) if epi == B.EPI_RESID else torch.full((m, n), float("nan"), device=DEV)
    B.tcmv_op_gemm(B.TCMV_F32, epi, dev(a), dev(w), dev(bias), c, m, n, k)
    sync()
    assert np.abs(c.cpu().numpy() - ref).max() <= 2e-5 * max(1.0, np.abs(ref).max())


# ---------------------------------------------------------------- attention
def _attn(dtype, qkv, cu, d, heads):
    T = qkv.shape[0]
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    cd = B.TCMV_BF16 if dtype == "bf16" else B.TCMV_F32
    ws_bytes = B.tcmv_op_attention_workspace(cd, cu, d, heads)
    ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device=DEV)
    ws.fill_(0xFF)                                   # poison: padding must never be used
    index = torch.frombuffer(bytearray(B.tcmv_op_attention_index(cd, cu, d, heads)), dtype=torch.uint8).to(DEV)
    out = torch.full((T, d), float("nan"), dtype=tdt, device=DEV)
    B.tcmv_op_attention(cd, dev(qkv, tdt), cu, d, heads, index, out, ws, ws.numel())
    sync()
    return out.float().cpu().numpy()


def _qkv(rng, T, d, q_scale, dtype):
    q = rng.normal(0, q_scale, (T, d)); k = rng.normal(0, 1, (T, d)); v = rng.normal(0, 1, (T, d))
    x = np.concatenate([q, k, v], 1).astype(np.float32)
    return bf16_grid(x) if dtype == "bf16" else x


ATTN_CASES = [
    # (segment lengths, d, heads, std of q): scores have std ~ q_scale
    ([64], 64, 1, 1.0),
    ([1], 128, 2, 1.0),                                 # single key: output = V
    ([130, 0, 5, 257], 160, 2, 1.0),                    # ragged, empty segment, head size 80
    ([576, 576], 128, 2, 0.3),                          # near-uniform softmax
    ([300, 77, 1, 640], 160, 2, 6.0),                   # peaked softmax
    ([1000], 320, 4, 8.0),                              # peaked, several query tiles and heads
    ([63, 65, 127, 129], 64, 2, 4.0),
    ([200], 96, 1, 2.0),
    ([333], 32, 1, 2.0),
]


@pytest.mark.parametrize("lens,d,heads,qs", ATTN_CASES)
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_attention(lens, d, heads, qs, dtype):
    rng = np.random.default_rng(sum(lens) + d + heads)
    cu = [0] + list(np.cumsum(lens))
    T = cu[-1]
    qkv = _qkv(rng, T, d, qs, dtype)
    x = qkv.astype(np.float64)
    ref = oe.attention(x[:, :d], x[:, d:2 * d], x[:, 2 * d:], cu, heads)
    got = _attn(dtype, qkv, [int(c) for c in cu], d, heads)
    if dtype == "f32":
        assert np.abs(got - ref).max() <= 2e-5 * max(1.0, np.abs(ref).max())
    else:
        # probabilities and outputs are rounded to bf16 (2^-9 relative each)
        assert np.abs(got - ref).max() <= 1.2e-2 * np.abs(ref).max()
        assert_tokens_close(got, ref, 2e-2, 0.9995, "attention")
        assert np.sqrt(((got - ref) ** 2).mean()) <= 4e-3 * np.sqrt((ref ** 2).mean())


@pytest.mark.parametrize("lens,qs,big_head", [
    ([1000, 333, 1, 0, 640, 257, 129, 2048], 6.0, None),     # ragged: 256-row work items (4 waves x 2 query tiles), peaked
    ([2048, 2048, 1024], 6.0, None),                          # multiples of 512: 512-row work items (8 waves), peaked
    ([4096, 3072], 1.0, 3),                                   # long segments: key-norm bound holds except for one head
    ([1000, 333, 2085, 640, 1500, 64], 1.0, None),            # small scores, ragged: the reference-free loop with masked last tiles
    ([4096, 2560, 1536], 0.5, None),                          # small scores, full tiles, 512-row items: the reference-free loop without masks
])
def test_attention_large_work_items(lens, qs, big_head):
    """Enough work items for the kernels with two query tiles per wave to be chosen (a single small problem
    gets 128-row items): 16 heads of 80, ragged and aligned segments, peaked scores (rescaling path), and long
    segments on which the reference-free copy handles all heads but one."""
    rng = np.random.default_rng(sum(lens))
    d, heads, dh = 1280, 16, 80
    cu = [0] + list(np.cumsum(lens))
    T = cu[-1]
    q = rng.normal(0, qs, (T, d)); k = rng.normal(0, 1, (T, d)); v = rng.normal(0, 1, (T, d))
    if big_head is not None:
        q[:, big_head * dh:(big_head + 1) * dh] *= 8.0
    qkv = bf16_grid(np.concatenate([q, k, v], 1).astype(np.float32))
    x = qkv.astype(np.float64)
    ref = oe.attention(x[:, :d], x[:, d:2 * d], x[:, 2 * d:], cu, heads)
    got = _attn("bf16", qkv, [int(c) for c in cu], d, heads)
    assert np.abs(got - ref).max() <= 1.2e-2 * np.abs(ref).max()
    assert_tokens_close(got, ref, 2e-2, 0.9995, "attention, large work items")
    assert np.sqrt(((got - ref) ** 2).mean()) <= 4e-3 * np.sqrt((ref ** 2).mean())


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_attention_segments_do_not_leak(dtype):
    """Encode {A, B} together == A and B alone; huge values in B must not move A."""
    rng = np.random.default_rng(42)
    d, heads = 160, 2
    la, lb = 150, 90
    qkv = _qkv(rng, la + lb, d, 2.0, dtype)
    both = _attn(dtype, qkv, [0, la, la + lb], d, heads)
    a_alone = _attn(dtype, qkv[:la], [0, la], d, heads)
    b_alone = _attn(dtype, qkv[la:], [0, lb], d, heads)
    assert np.array_equal(both[:la], a_alone) and np.array_equal(both[la:], b_alone)
    poisoned = qkv.copy()
    poisoned[la:, 2 * d:] = 3e4            # V of segment B
    poisoned[la:, d:2 * d] *= 50           # K of segment B
    got = _attn(dtype, poisoned, [0, la, la + lb], d, heads)
    assert np.array_equal(got[:la], both[:la])


def test_attention_zero_queries_give_mean_of_values():
    rng = np.random.default_rng(9)
    d, heads, T = 160, 2, 200
    qkv = _qkv(rng, T, d, 1.0, "bf16")
    qkv[:, :d] = 0
    got = _attn("bf16", qkv, [0, T], d, heads)
    ref = qkv[:, 2 * d:].astype(np.float64).mean(0, keepdims=True)
    assert np.abs(got - ref).max() <= 1e-2 * np.abs(qkv[:, 2 * d:]).max()


def test_empty_inputs_are_no_ops():
    B.tcmv_op_layernorm(B.TCMV_BF16, None, None, None, None, 0, 256, 1e-6)
    B.tcmv_op_gemm(B.TCMV_BF16, 0, None, None, None, None, 0, 128, 64)
    B.tcmv_op_attention(B.TCMV_BF16, None, [0, 0, 0], 128, 2, None, None, None, 0)
    sync()


def _bf16_round(v):
    """fp64 -> nearest bf16 value (ties to even), as fp64; the fp32 step in between is harmless here because the
    values tested are never within 2^-24 relative of a bf16 tie."""
    u = np.asarray(v, np.float32).view(np.uint32).astype(np.uint64)
    u = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16) << 16
    return u.astype(np.uint32).view(np.float32).astype(np.float64)


@pytest.mark.parametrize("m,n,k", [(192, 64, 64), (16384 + 37, 2560, 128)])
@pytest.mark.parametrize("with_bias", [False, True])
def test_gelu_epilogue_on_an_exact_grid(m, n, k, with_bias):
    """The activation of the fc1 epilogue on known arguments.  Rows of A are one-hot, so the accumulator is exactly
    one weight (plus an fp32 bias chosen so that the sum is exact): the weights run over every bf16 value with
    2^-12 <= |x| <= 10, i.e. an exact grid that is dense near 0.  The bf16 output must be within one bf16 unit in
    the last place of the rounded exact erf-form GELU (or 2^-22 where that is larger) for every argument; a tanh-form
    or a sigmoid-form activation misses this by several units.  Both tile families are driven (small shape: 64-row
    tiles; large shape: persistent 256-row tiles)."""
    e, mant = np.meshgrid(np.arange(-12, 4), np.arange(128), indexing="ij")
    mag = (np.ldexp(1.0 + mant / 128.0, e)).reshape(-1)
    mag = mag[mag <= 10.0]
    grid = np.concatenate([mag, -mag, [0.0]]).astype(np.float32)
    assert np.array_equal(bf16_grid(grid), grid)
    rng = np.random.default_rng(11)
    w = grid[rng.integers(0, grid.size, (n, k))]
    w.reshape(-1)[:grid.size] = grid                                  # every grid value occurs at least once
    a = np.zeros((m, k), np.float32)
    a[np.arange(m), np.arange(m) % k] = 1.0
    # bias: multiples of 2^-13 below 2; |x| < 16 with a last place of 2^-19 fits the 24 bits of an fp32
    bias = (rng.integers(-16000, 16000, n) * 2.0 ** -13).astype(np.float32) if with_bias else np.zeros(n, np.float32)
    x = w.astype(np.float64).T[np.arange(m) % k] + bias.astype(np.float64)            # [m, n], exact
    assert np.array_equal(x.astype(np.float32).astype(np.float64), x)
    want = _bf16_round(oe.gelu(x))
    c = torch.full((m, n), float("nan"), dtype=torch.bfloat16, device=DEV)
    B.tcmv_op_gemm(B.TCMV_BF16, B.EPI_GELU, dev(a, torch.bfloat16), dev(w, torch.bfloat16), dev(bias), c, m, n, k)
    sync()
    got = c.float().cpu().numpy().astype(np.float64)
    ulp = np.ldexp(1.0, np.floor(np.log2(np.maximum(np.abs(want), 1e-300))).astype(np.int64) - 7)
    tol = np.maximum(ulp, 2.0 ** -22)
    bad = np.abs(got - want) > tol
    assert not bad.any(), (x[bad][:5], got[bad][:5], want[bad][:5])
    # the pin has teeth: the tanh form of the activation, rounded the same way, breaks the bound
    tanh_form = _bf16_round(0.5 * x * (1 + np.tanh(np.sqrt(2 / np.pi) * (x + 0.044715 * x ** 3))))
    assert (np.abs(tanh_form - want) > tol).any()


def test_gemm_bf16_large_tile_path_with_ragged_rows():
    """Enough 256x256 tiles to select the large-tile kernel, with a ragged last row tile."""
    rng = np.random.default_rng(77)
    m, n, k = 16384 + 37, 2560, 128
    a = bf16_grid(rng.normal(0, 1, (m, k)))
    w = bf16_grid(rng.normal(0, 0.05, (n, k)))
    bias = rng.normal(0, 0.5, n).astype(np.float32)
    for epi in (B.EPI_STORE, B.EPI_GELU, B.EPI_RESID):
        c0 = rng.normal(0, 1, (m, n)).astype(np.float32)
        ref = _gemm_ref(a, w, bias, epi, c0)
        c = dev(c0) if epi == B.EPI_RESID else torch.full((m, n), float("nan"), dtype=torch.bfloat16, device=DEV)
        B.tcmv_op_gemm(B.TCMV_BF16, epi, dev(a, torch.bfloat16), dev(w, torch.bfloat16), dev(bias), c, m, n, k)
        sync()
        got = c.float().cpu().numpy()
        tol = 1e-4 * max(1.0, np.abs(ref).max()) if epi == B.EPI_RESID else 2 ** -8 * np.abs(ref).max() + 1e-5
        assert np.abs(got - ref).max() <= tol, epi


def test_gemm_bf16_wide_tile_path_with_ragged_rows_and_columns():
    """A shape for which tiles 320 columns wide need fewer rounds over the CUs than 256x256 ones (640 -> 512
    tiles on 256 CUs): the wave tiles are 160 columns wide and leave the kernel in column groups of 64, 64
    and 32.  Last row tile and last column tile ragged; the gated epilogue goes the same way."""
    rng = np.random.default_rng(78)
    m, n, k = 8100, 5112, 128
    a = bf16_grid(rng.normal(0, 1, (m, k)))
    w = bf16_grid(rng.normal(0, 0.05, (n, k)))
    bias = rng.normal(0, 0.5, n).astype(np.float32)
    for epi in (B.EPI_STORE, B.EPI_GELU, B.EPI_RESID):
        c0 = rng.normal(0, 1, (m, n)).astype(np.float32)
        ref = _gemm_ref(a, w, bias, epi, c0)
        c = dev(c0) if epi == B.EPI_RESID else torch.full((m, n), float("nan"), dtype=torch.bfloat16, device=DEV)
        B.tcmv_op_gemm(B.TCMV_BF16, epi, dev(a, torch.bfloat16), dev(w, torch.bfloat16), dev(bias), c, m, n, k)
        sync()
        got = c.float().cpu().numpy()
        tol = 1e-4 * max(1.0, np.abs(ref).max()) if epi == B.EPI_RESID else 2 ** -8 * np.abs(ref).max() + 1e-5
        assert np.abs(got - ref).max() <= tol, epi
    u = a.astype(np.float64) @ w.astype(np.float64).T + bias
    ref = oe.silu(u[:, 0::2]) * u[:, 1::2]
    c = torch.full((m, n // 2), 7.0, dtype=torch.bfloat16, device=DEV)
    B.tcmv_op_gemm(B.TCMV_BF16, B.EPI_GATED, dev(a, torch.bfloat16), dev(w, torch.bfloat16), dev(bias), c, m, n, k)
    sync()
    assert np.abs(c.float().cpu().numpy() - ref).max() <= 2 ** -7 * np.abs(ref).max()


# ---------------------------------------------------------------- encoder-family variants
@pytest.mark.parametrize("rows,d", [(3, 320), (1030, 1280), (77, 64)])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_rmsnorm(rows, d, dtype):
    rng = np.random.default_rng(rows + d)
    x = (rng.normal(0.5, 3, (rows, d))).astype(np.float32)
    g = (1 + rng.normal(0, 0.3, d)).astype(np.float32)
    ref = oe.rmsnorm(x.astype(np.float64), g.astype(np.float64), 1e-6)
    y = torch.empty((rows, d), dtype=torch.bfloat16 if dtype == "bf16" else torch.float32, device=DEV)
    B.tcmv_op_layernorm(B.TCMV_BF16 if dtype == "bf16" else B.TCMV_F32, dev(x), dev(g), None, y, rows, d, 1e-6)
    sync()
    got = y.float().cpu().numpy()
    tol = 2e-5 if dtype == "f32" else 2 ** -8
    assert np.abs(got - ref).max() <= tol * max(1.0, np.abs(ref).max())


@pytest.mark.parametrize("m,n2,k", [(300, 256, 128), (1029, 1280, 320), (4100, 6912, 1280)])
def test_gated_epilogue(m, n2, k):
    """Columns arrive as (gate, up) pairs; the kernel writes silu(gate) * up."""
    rng = np.random.default_rng(m)
    a = bf16_grid(rng.normal(0, 1, (m, k)).astype(np.float32))
    w = bf16_grid(rng.normal(0, 0.08, (n2, k)).astype(np.float32))
    bias = rng.normal(0, 0.3, n2).astype(np.float32)
    u = a.astype(np.float64) @ w.astype(np.float64).T + bias
    ref = oe.silu(u[:, 0::2]) * u[:, 1::2]
    c = torch.full((m, n2 // 2), 7.0, dtype=torch.bfloat16, device=DEV)
    B.tcmv_op_gemm(B.TCMV_BF16, B.EPI_GATED, dev(a, torch.bfloat16), dev(w, torch.bfloat16), dev(bias), c, m, n2, k)
    sync()
    got = c.float().cpu().numpy()
    assert np.abs(got - ref).max() <= 2 ** -7 * np.abs(ref).max()
    assert_tokens_close(got, ref, 1e-2, 0.9999, "gated epilogue")


def test_attention_mixed_norm_bounds_in_one_launch():
    """Some (segment, head, query tile) combinations have provably small scores and are exponentiated without
    a softmax reference, others in the same launch are not: head 0 has large queries, one block of query rows
    of head 1 is large, one segment has large keys.  Every row must come out right whichever copy handled it."""
    rng = np.random.default_rng(123)
    d, heads, dh = 240, 3, 80
    lens = [700, 1300, 520]
    cu = [0] + list(np.cumsum(lens))
    T = cu[-1]
    q = rng.normal(0, 1.0, (T, d)); k = rng.normal(0, 1.0, (T, d)); v = rng.normal(0, 1.0, (T, d))
    q[:, :dh] *= 7.0                       # head 0: bound far above the limit everywhere
    q[300:556, dh:2 * dh] *= 7.0           # head 1: one tile of queries in segment 0
    k[cu[2]:, 2 * dh:] *= 6.0              # head 2: large keys in the last segment only
    qkv = bf16_grid(np.concatenate([q, k, v], 1).astype(np.float32))
    x = qkv.astype(np.float64)
    ref = oe.attention(x[:, :d], x[:, d:2 * d], x[:, 2 * d:], cu, heads)
    got = _attn("bf16", qkv, [int(c) for c in cu], d, heads)
    assert np.isfinite(got).all()
    assert np.abs(got - ref).max() <= 1.2e-2 * np.abs(ref).max()
    assert_tokens_close(got, ref, 2e-2, 0.9995, "attention, mixed bounds")
    # the same rows, recomputed with uniformly small inputs elsewhere, do not change (no interaction between copies)
    small = qkv.copy()
    small[:, :dh] = qkv[:, :dh] / 7.0
    got2 = _attn("bf16", bf16_grid(small), [int(c) for c in cu], d, heads)
    assert np.array_equal(got[:, dh:], got2[:, dh:])


# ---------------------------------------------------------------- bandwidth reference
def test_stream_reference_reads_and_writes_what_it_says():
    """Words written are the XOR of the words each thread read (threads stride over the input), so no read can be
    dropped; a size of zero on either side is allowed, misaligned sizes are refused."""
    nt = 2048 * 256
    n_in, n_out = nt + nt // 2 + 5, nt + 77
    rng = np.random.default_rng(0)
    src = rng.integers(0, 2 ** 32, (n_in, 4), dtype=np.uint64).astype(np.uint32)
    acc = np.zeros((nt, 4), np.uint32)
    for k in range(0, n_in, nt):
        blk = src[k:k + nt]
        acc[:len(blk)] ^= blk
    want = acc[np.arange(n_out) % nt]
    d_in = torch.from_numpy(src.view(np.int32)).to(DEV)
    d_out = torch.zeros((n_out, 4), dtype=torch.int32, device=DEV)
    B.tcmv_op_stream(d_in, n_in * 16, d_out, n_out * 16)
    sync()
    assert np.array_equal(d_out.cpu().numpy().view(np.uint32), want)
    B.tcmv_op_stream(None, 0, d_out, 16 * 10)             # nothing read: zeros written
    B.tcmv_op_stream(d_in, 16 * 10, None, 0)
    B.tcmv_op_stream(None, 0, None, 0)
    sync()
    assert not d_out[:10].any() and np.array_equal(d_out[10:].cpu().numpy().view(np.uint32), want[10:])
    with pytest.raises(B.TcmvError):
        B.tcmv_op_stream(d_in, 24, d_out, 16)
