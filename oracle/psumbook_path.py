"""A second, separate CPU implementation that follows the paper's three steps
(Section 3: reshape, build the Psumbook by Eq. 2, gather by code and
accumulate) in float64 numpy.  Test infrastructure only.

It exists to check the dequantize-then-multiply oracle against the identity the
method rests on:
    y[b][n] = s[n] * sum_c sum_j P[b][c][j][ code[c][n][j] ]
and, with one scale per run of g weights (g/v sub-vectors) of a row,
    y[b][n] = sum_G s[n][G] * sum_c sum_{j in G} P[b][c][j][ code[c][n][j] ].
It also counts the operations it performs, to compare with Eq. 3.
"""
from __future__ import annotations

import numpy as np


def psum_gemm(x, codes, codebooks, scales):
    """Returns (y float64 [B][N], counters dict)."""
    x64 = x.astype(np.float64)
    cb = codebooks.astype(np.float64)
    s = scales.astype(np.float64)
    m, N, J = codes.shape
    _, ncent, v = cb.shape
    B, K = x64.shape
    xr = x64.reshape(B, J, v)                       # Step 1: x^j_k = x_{v j + k}
    build_macs = 0
    gathers = 0
    if s.ndim == 1:
        s = s[:, None]                              # one group: the whole row
    G = s.shape[1]
    per_group = J // G                              # sub-vectors per normalisation group
    yg = np.zeros((B, G, N), np.float64)            # partial sums per group, scaled at the end
    for c in range(m):
        # Step 2 (Eq. 2): P[b][j][i] = sum_k C[c][i][k] x[b][j][k]
        P = np.einsum("bjk,ik->bji", xr, cb[c])
        build_macs += B * J * ncent * v
        # Step 3: look up one partial sum per (row, sub-vector) and accumulate
        idx = codes[c].astype(np.int64).T            # [J][N]
        for b in range(B):
            picked = np.take_along_axis(P[b], idx, axis=1)   # [J][N]
            yg[b] += picked.reshape(G, per_group, N).sum(axis=1)
            gathers += J * N
    y = np.einsum("bgn,ng->bn", yg, s)
    return y, {"build_macs": build_macs, "gathers": gathers}
