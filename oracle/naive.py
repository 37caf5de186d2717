"""Pure-Python (no numpy arithmetic) attention for tiny inputs
(TEST INFRASTRUCTURE ONLY).  Scaled dot-product attention with a softmax over
the keys of the query's own segment, written as explicit loops over scalars so
that it shares nothing with the vectorised reference except the definition."""
from __future__ import annotations

import math


def attention_loops(q, k, v, cu_seqlens, heads):
    """q, k, v: nested lists [T][d] of Python floats -> nested list [T][d]."""
    T = len(q)
    d = len(q[0]) if T else 0
    dh = d // heads
    out = [[0.0] * d for _ in range(T)]
    for s in range(len(cu_seqlens) - 1):
        a, b = cu_seqlens[s], cu_seqlens[s + 1]
        for h in range(heads):
            c0 = h * dh
            for i in range(a, b):
                scores = []
                for j in range(a, b):
                    acc = 0.0
                    for c in range(dh):
                        acc += q[i][c0 + c] * k[j][c0 + c]
                    scores.append(acc / math.sqrt(dh))
                mx = max(scores)
                ex = [math.exp(sc - mx) for sc in scores]
                z = math.fsum(ex)
                for c in range(dh):
                    acc = 0.0
                    for j in range(a, b):
                        acc += ex[j - a] / z * v[j][c0 + c]
                    out[i][c0 + c] = acc
    return out
