"""Eq. 1 (average bits per weight) against the values the paper prints."""
import os

import pytest

from oracle.bits import average_bits

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def rows(name):
    for line in open(os.path.join(GOLD, name)):
        if line.strip() and not line.startswith("#"):
            yield line.split()


def test_table1_rows():
    for v, m, b, g, qc, qcb, qn, qbar in rows("table1_avg_bits.txt"):
        got = average_bits(int(v), int(m), int(b), int(g), 4096, 4096)
        for have, want in zip(got, (qc, qcb, qn, qbar)):
            assert abs(have - float(want)) <= 0.00051, (v, m, b, g, got)


def test_table8_bit_column():
    checked = 0
    for N, K, m, v, bit, *flag in rows("table8_bits.txt"):
        q = average_bits(int(v), int(m), 8, 128, int(N), int(K))[3]
        if flag:
            # printed value is the 8192 row's; Eq. 1 at 4096 differs in the codebook term only
            assert 0.004 < q - float(bit) < 0.007
            continue
        assert abs(q - float(bit)) <= 0.00051, (N, K, m, v, q)
        checked += 1
    assert checked == 10
