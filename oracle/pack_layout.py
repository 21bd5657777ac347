"""Independent numpy description of the packed code layout documented in
include/codegemm.h (test infrastructure only).  Written from the header's
prose: array [NGR][NKT][part][16][32][bytes]; inside a part, byte 8*(c-c0)+r of
entry (g, s) of unit (rg, kt) holds codes[c][128*rg + 8*g + r][32*kt + s], or 0
outside the matrix."""
from __future__ import annotations

import numpy as np


def pack_reference(codes: np.ndarray) -> np.ndarray:
    m, N, J = codes.shape
    NGR = -(-N // 128)
    NKT = -(-J // 32)
    padded = np.zeros((m, NGR * 128, NKT * 32), np.uint8)
    padded[:, :N, :J] = codes
    rg = np.arange(NGR, dtype=np.int64)[:, None, None, None, None]
    kt = np.arange(NKT, dtype=np.int64)[None, :, None, None, None]
    g = np.arange(16, dtype=np.int64)[None, None, :, None, None]
    s = np.arange(32, dtype=np.int64)[None, None, None, :, None]
    r = np.arange(8, dtype=np.int64)[None, None, None, None, :]
    n = 128 * rg + 8 * g + r
    j = 32 * kt + s
    unit_bytes = 128 * 32 * m
    out = np.zeros(NGR * NKT * unit_bytes, np.uint8)
    for c in range(m):
        part = c // 2
        part_bytes = 8 if 2 * part + 1 == m else 16
        off = (rg * NKT + kt) * unit_bytes + part * 16 * 512 + (g * 32 + s) * part_bytes + (c % 2) * 8 + r
        shape = np.broadcast_shapes(off.shape, n.shape, j.shape)
        vals = padded[c][np.broadcast_to(n, shape), np.broadcast_to(j, shape)]
        out[np.broadcast_to(off, shape).ravel()] = vals.ravel()
    return out
