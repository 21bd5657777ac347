"""Average bits per weight (Section 2.2, Eq. 1) and compressed byte counts.

Test infrastructure: the closed form written out term by term, pinned by the
rows the paper prints in Table 1 and by the "bit" column of Table 8.
"""
from __future__ import annotations


def average_bits(v: int, m: int, b: int, g: int, N: int, K: int):
    """Returns (q_code, q_codebook, q_norm, q_bar) for an N x K weight matrix.
    g = -1 means one normalisation scale per output row, i.e. a group of K."""
    group = K if g == -1 else g
    s_codebook = 16 * m * (2 ** b) * v          # fp16 centroids
    s_code = b * m * N * (K // v)               # one b-bit code per vector per codebook
    s_norm = 16 * N * (K / group)               # one fp16 scale per group
    total = N * K
    return s_code / total, s_codebook / total, s_norm / total, (s_codebook + s_code + s_norm) / total
