#!/usr/bin/env python3
"""Launches the attention kernel alone at the video workload's shape (one
32768-token segment, d=1280, 16 heads, bf16) and then a plain 1 GiB device copy.
Meant to be run under rocprofv3 --pmc (one counter per run), e.g.

    rocprofv3 --pmc FETCH_SIZE  --output-format csv -d out/fetch -o a -- python3 paper_2603_26498_amd/profile_attention.py
    rocprofv3 --pmc WRITE_SIZE  --output-format csv -d out/write -o a -- python3 paper_2603_26498_amd/profile_attention.py

The copy (1 GiB read + 1 GiB written, known exactly) calibrates the counter
units; the attention kernel's counters are scaled by the same factor."""
import os
import sys

import torch

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
from paper_2603_26498_amd import binding as B  # noqa: E402


def main():
    T, d, heads = 32768, 1280, 16
    g = torch.Generator(device="cuda").manual_seed(0)
    qkv = (torch.randn(T, 3 * d, device="cuda", generator=g) * 0.7).to(torch.bfloat16)
    cu = [0, T]
    nbytes = B.tcmv_op_attention_workspace(B.TCMV_BF16, cu, d, heads)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    out = torch.empty(T, d, dtype=torch.bfloat16, device="cuda")
    for _ in range(3):
        B.tcmv_op_attention(B.TCMV_BF16, qkv, cu, d, heads, out, ws, nbytes)
    torch.cuda.synchronize()
    src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
    dst = torch.empty_like(src)
    for _ in range(3):
        dst.copy_(src)
    torch.cuda.synchronize()
    print("attention x3 and 1 GiB copy x3 done")


if __name__ == "__main__":
    main()
