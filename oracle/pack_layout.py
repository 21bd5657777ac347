"""Independent numpy description of the packed code layout documented in
include/codegemm.h (test infrastructure only).  Written from the header's
prose: array [NRB][NKT][S][part][64][bytes]; inside a part, byte 8*(c-c0)+r of
lane l at step t holds codes[c][512*rb + 64*r + l][S*kt + (t+l) mod S], or 0
outside the matrix."""
from __future__ import annotations

import numpy as np


def pack_reference(codes: np.ndarray, S: int) -> np.ndarray:
    m, N, J = codes.shape
    NRB = -(-N // 512)
    NKT = -(-J // S)
    padded = np.zeros((m, NRB * 512, NKT * S), np.uint8)
    padded[:, :N, :J] = codes
    rb = np.arange(NRB, dtype=np.int64)[:, None, None, None, None]
    kt = np.arange(NKT, dtype=np.int64)[None, :, None, None, None]
    t = np.arange(S, dtype=np.int64)[None, None, :, None, None]
    l = np.arange(64, dtype=np.int64)[None, None, None, :, None]
    r = np.arange(8, dtype=np.int64)[None, None, None, None, :]
    n = 512 * rb + 64 * r + l
    j = S * kt + (t + l) % S
    step_bytes = 64 * 8 * m
    out = np.zeros(NRB * NKT * S * step_bytes, np.uint8)
    for c in range(m):
        part = c // 2
        part_bytes = 8 if 2 * part + 1 == m else 16
        off = ((rb * NKT + kt) * S + t) * step_bytes + part * 16 * 64 + l * part_bytes + (c % 2) * 8 + r
        vals = padded[c][np.broadcast_to(n, off.shape), np.broadcast_to(j, off.shape)]
        out[off.ravel()] = vals.ravel()
    return out
