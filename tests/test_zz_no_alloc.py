"""The attention operator without a workspace argument (for callers that cannot allocate device memory): two calls
in a row, the second on a smaller input, each against the entry point that takes a workspace."""
import numpy as np
import pytest
import torch

from paper_2603_26498_amd import binding as B

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _both(qkv, cu, d, heads):
    T = qkv.shape[0]
    index = torch.frombuffer(bytearray(B.tcmv_op_attention_index(B.TCMV_BF16, cu, d, heads)), dtype=torch.uint8).to(DEV)
    nbytes = B.tcmv_op_attention_workspace(B.TCMV_BF16, cu, d, heads)
    assert 0 < nbytes <= B.TCMV_NOALLOC_SCRATCH_BYTES
    ws = torch.empty(nbytes, dtype=torch.uint8, device=DEV)
    ws.fill_(0xFF)
    ref = torch.full((T, d), float("nan"), dtype=torch.bfloat16, device=DEV)
    B.tcmv_op_attention(B.TCMV_BF16, qkv, cu, d, heads, index, ref, ws, nbytes)
    got = torch.full((T, d), float("nan"), dtype=torch.bfloat16, device=DEV)
    B.tcmv_op_attention_noalloc(B.TCMV_BF16, qkv, cu, d, heads, index, got)
    torch.cuda.synchronize()
    return got, ref


def test_attention_without_workspace_argument_matches_the_one_with():
    g = torch.Generator(device=DEV).manual_seed(5)
    d, heads = 320, 4                                   # head size 80
    # first call: ragged segments (one empty), 1500 rows; second call: a smaller input, other segment lengths,
    # peaked scores (the running-maximum kernel) - whatever the first call left in the array must not matter
    for T, cu, qs in ((1500, [0, 700, 700, 1189, 1500], 0.7), (333, [0, 40, 333], 6.0)):
        qkv = torch.randn(T, 3 * d, device=DEV, generator=g)
        qkv[:, :d] *= qs
        qkv = qkv.to(torch.bfloat16)
        got, ref = _both(qkv, cu, d, heads)
        assert torch.isfinite(ref.float()).all()
        assert torch.equal(got.view(torch.int16), ref.view(torch.int16))      # same kernels, same order: bit-equal


def test_shapes_beyond_the_fixed_scratch_are_refused():
    d, heads, T = 1280, 16, 16384                        # transposed values alone: 1280 x 16384 x 2 bytes = 40 MiB
    cu = [0, T]
    assert B.tcmv_op_attention_workspace(B.TCMV_BF16, cu, d, heads) > B.TCMV_NOALLOC_SCRATCH_BYTES
    index = torch.frombuffer(bytearray(B.tcmv_op_attention_index(B.TCMV_BF16, cu, d, heads)), dtype=torch.uint8).to(DEV)
    qkv = torch.zeros(T, 3 * d, dtype=torch.bfloat16, device=DEV)
    out = torch.zeros(T, d, dtype=torch.bfloat16, device=DEV)
    with pytest.raises(B.TcmvError) as e:
        B.tcmv_op_attention_noalloc(B.TCMV_BF16, qkv, cu, d, heads, index, out)
    assert e.value.code == B.TCMV_E_WORKSPACE_TOO_SMALL
