"""CPU oracle of the decode-side consumer: one new token's attention over the compressed prompt cache.

TEST INFRASTRUCTURE ONLY (tests, the smoke check, the benchmark's cpu_baseline leg); imports nothing from
the HIP package.

What is computed (paper Appendix A, "Complexity": compression only removes cached positions and leaves the
retained keys and values unchanged, so ordinary attention runs over what is left; Section 3.5 measures the
per-token decode latency over that retained cache).  The cache is the output of the compression operator
(Section 2.5): for unit u = (prompt p, layer l, KV head h) the retained rows are
``head_off[u] .. head_off[u+1]-1`` of ``packed_k`` / ``packed_v``.  With grouped-query attention, query head
j reads KV head j // G, G = n_q_heads / H.  For every (p, l, j):

    s_i   = scale * <q[p, l, j], k_i>            i over the retained rows of (p, l, j // G)
    w     = softmax(s)
    out   = sum_i w_i v_i
    lse   = log sum_i exp(s_i)                   (what a caller needs to merge with attention over other keys)

A unit without rows gives out = 0 and lse = -inf.  Everything in fp64, written out as the definition.
"""
from __future__ import annotations

import numpy as np


def decode_attention(q: np.ndarray, packed_k: np.ndarray, packed_v: np.ndarray, head_off: np.ndarray, H: int,
                     scale: float):
    """q [P, L, Hq, d]; packed_k [rows, d]; packed_v [rows, dv]; head_off [P*L*H + 1] (units ordered p, l, h).
    Returns (out [P, L, Hq, dv] float64, lse [P, L, Hq] float64)."""
    P, L, Hq, d = q.shape
    assert Hq % H == 0 and head_off.shape[0] == P * L * H + 1
    G = Hq // H
    dv = packed_v.shape[1]
    out = np.zeros((P, L, Hq, dv), dtype=np.float64)
    lse = np.full((P, L, Hq), -np.inf, dtype=np.float64)
    for p in range(P):
        for l in range(L):
            for j in range(Hq):
                u = (p * L + l) * H + j // G
                a, b = int(head_off[u]), int(head_off[u + 1])
                if b <= a:
                    continue
                K = packed_k[a:b].astype(np.float64)
                V = packed_v[a:b].astype(np.float64)
                s = float(scale) * (K @ q[p, l, j].astype(np.float64))
                top = s.max()
                e = np.exp(s - top)
                z = e.sum()
                out[p, l, j] = (e / z) @ V
                lse[p, l, j] = top + np.log(z)
    return out, lse
