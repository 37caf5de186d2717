#!/usr/bin/env python3
"""Launches the GEMM kernel alone at the four per-layer shapes of the video workload
(32768 rows, d=1280, mlp 5120, bf16: QKV store, out-projection + residual, fc1 + GELU,
fc2 + residual), three launches each.  Meant to be run under rocprofv3 --pmc, e.g.

    rocprofv3 --pmc SQ_BUSY_CU_CYCLES SQ_VALU_MFMA_BUSY_CYCLES SQ_LDS_BANK_CONFLICT SQ_INSTS_MFMA \\
              --output-format csv -d out/gemm -o a -- python3 paper_2603_26498_amd/profile_gemm.py
"""
import os
import sys

import torch

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
from paper_2603_26498_amd import binding as B  # noqa: E402


def main():
    m = 32768
    g = torch.Generator(device="cuda").manual_seed(0)
    for (n, k, epi) in [(3840, 1280, B.EPI_STORE), (1280, 1280, B.EPI_RESID), (5120, 1280, B.EPI_GELU),
                        (1280, 5120, B.EPI_RESID)]:
        a = torch.randn(m, k, device="cuda", generator=g).to(torch.bfloat16)
        w = (torch.randn(n, k, device="cuda", generator=g) * 0.02).to(torch.bfloat16)
        bias = torch.zeros(n, device="cuda")
        c = torch.zeros(m, n, device="cuda", dtype=torch.float32 if epi == B.EPI_RESID else torch.bfloat16)
        for _ in range(3):
            B.tcmv_op_gemm(B.TCMV_BF16, epi, a, w, bias, c, m, n, k)
        torch.cuda.synchronize()
    print("4 GEMM shapes x3 done")


if __name__ == "__main__":
    main()
