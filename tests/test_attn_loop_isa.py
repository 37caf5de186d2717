"""The hand-scheduled attention loop issues its LDS fragment reads from inline assembly and waits for them with
explicit `s_waitcnt lgkmcnt(2)`.  That accounting is sound only while nothing else inside the loop uses the same
counter (LDS operations of the compiler's own, scalar memory loads) and while the reads and waits stay in the
written order.  This test compiles the kernel source to gfx950 assembly (no GPU needed) and checks, for every
instantiation that has the pipelined loop, the loop block as the hardware will see it."""
import collections
import os
import re
import subprocess

import pytest

from paper_2603_26498_amd import build as B

SRC = os.path.join(B.CSRC, "attn_bf16.hip")


def _blocks(body):
    blocks, cur = [], None
    for ln in body.split("\n"):
        if re.match(r"^\.LBB\d+_\d+:", ln):
            cur = []
            blocks.append(cur)
        elif cur is not None and ln.startswith("\t") and not ln.startswith(("\t.", "\t;")):
            cur.append(ln.strip().split(";")[0].strip())
    return blocks


def test_pipelined_loop_is_the_only_user_of_the_lds_counter(tmp_path):
    try:
        hipcc = B._hipcc()
    except RuntimeError:
        pytest.skip("hipcc not found")
    out = str(tmp_path / "attn.s")
    B._run([hipcc, *B.FLAGS, "-S", "--cuda-device-only", SRC, "-o", out])
    asm = open(out).read()
    seen = 0
    # head size 80, two query tiles per wave, 8 or 4 waves, queries pre-scaled or not, reference-free copy
    for m in re.finditer(r"^(_ZN4tcmv16attn_bf16_kernelILi80ELi2ELi[48]ELb[01]ELb1EEEvNS_8AttnArgsE):", asm, re.M):
        body = asm[m.end():asm.index(".Lfunc_end", m.end())]
        loops = [b for b in _blocks(body) if sum(i.startswith("v_mfma_f32_32x32x16_bf16") for i in b) == 44]
        assert len(loops) == 1, (m.group(1), len(loops))
        ins = loops[0]
        ops = collections.Counter(i.split()[0] for i in ins)
        assert ops["ds_read_b128"] == 22 and ops["v_exp_f32_e32"] == 64, ops
        assert not [i for i in ins if i.startswith(("s_load", "s_buffer_load", "ds_")) and not i.startswith("ds_read_b128")], \
            "something else in the loop uses the LDS / scalar-memory counter"
        waits = [i for i in ins if i.startswith("s_waitcnt")]
        assert waits == ["s_waitcnt lgkmcnt(2)"] * 8, waits
        # between two waits: the MFMAs of three fragments (two of the last group of a region) and as many reads as the
        # ring protocol says; every read comes after both MFMAs of its step
        seq = [("W" if i.startswith("s_waitcnt") else "M" if i.startswith("v_mfma") else "R")
               for i in ins if i.startswith(("s_waitcnt", "v_mfma", "ds_read_b128"))]
        region = "WMMRMMRMMR" + "WMMRMMRMMR" + "WMMMMRMMR" + "WMMRMMRR"
        assert "".join(seq) == region * 2, "".join(seq)
        seen += 1
    assert seen == 4
