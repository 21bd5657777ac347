"""CPU pin of oracle/pack_layout.py::pack_reference, the expected value of the bit-exact
pack test.  The packed layout is decoded byte by byte in plain Python loops written from
the prose of include/codegemm.h (array [NGR][NKT][part][16][32][bytes]; a part holds two
codebooks x 8 rows = 16 bytes, the last part of an odd m one codebook = 8 bytes), never
from the numpy index arithmetic of pack_reference.  Checked: every byte of the packed
buffer decodes to exactly one (c, n, j); bytes whose (n, j) lies in the matrix hold that
code and every code appears exactly once; all other bytes are zero.  A planted mistake
(row-lane and slot swapped) in a copy of pack_reference must fail the same check."""
import numpy as np
import pytest

from oracle import pack_layout

SHAPES = [(1, 1, 1), (130, 33, 1), (129, 65, 2), (7, 32, 2), (257, 31, 3), (128, 64, 3), (200, 40, 4), (3, 5, 4)]


def decode(offset, m, NKT):
    """(c, n, j) of the packed byte at `offset`, from the header's description."""
    unit_bytes = 128 * 32 * m
    unit, rem = divmod(offset, unit_bytes)
    rg, kt = divmod(unit, NKT)
    full_part_bytes = 16 * 32 * 16                       # a part of two codebooks
    part = min(rem // full_part_bytes, (m - 1) // 2)
    rem -= part * full_part_bytes
    entry_bytes = 8 if 2 * part + 1 == m else 16         # the last part of an odd m holds one codebook
    entry, byte = divmod(rem, entry_bytes)
    g, s = divmod(entry, 32)
    assert 0 <= g < 16
    c = 2 * part + byte // 8
    r = byte % 8
    return c, 128 * rg + 8 * g + r, 32 * kt + s


def check_layout(pack_fn, N, J, m, seed=0):
    rng = np.random.default_rng(seed)
    codes = rng.integers(1, 256, size=(m, N, J), dtype=np.uint8)     # no zero code: pads are told apart
    packed = pack_fn(codes)
    NGR, NKT = -(-N // 128), -(-J // 32)
    assert packed.dtype == np.uint8 and packed.shape == (NGR * NKT * 128 * 32 * m,)
    seen = np.zeros((m, N, J), np.int32)
    for off in range(packed.size):
        c, n, j = decode(off, m, NKT)
        assert 0 <= c < m
        if n < N and j < J:
            assert packed[off] == codes[c, n, j], (off, c, n, j)
            seen[c, n, j] += 1
        else:
            assert packed[off] == 0, (off, c, n, j)
    assert np.all(seen == 1)


@pytest.mark.parametrize("N,J,m", SHAPES)
def test_pack_reference_is_the_documented_layout(N, J, m):
    check_layout(pack_layout.pack_reference, N, J, m, seed=N + J + m)


def swapped_copy():
    """pack_reference with the roles of the row-lane g and the slot s exchanged in the offset."""
    import inspect
    src = inspect.getsource(pack_layout.pack_reference)
    old = "(g * 32 + s) * part_bytes"
    assert src.count(old) == 1
    ns = {"np": np}
    exec(src.replace(old, "(s * 16 + g) * part_bytes"), ns)
    return ns["pack_reference"]


@pytest.mark.parametrize("N,J,m", [(130, 33, 1), (129, 65, 2), (257, 31, 3)])
def test_planted_swap_of_row_lane_and_slot_is_caught(N, J, m):
    with pytest.raises(AssertionError):
        check_layout(swapped_copy(), N, J, m)


def test_planted_codebook_parity_swap_is_caught():
    import inspect
    src = inspect.getsource(pack_layout.pack_reference)
    old = "(c % 2) * 8"
    assert src.count(old) == 1
    ns = {"np": np}
    exec(src.replace(old, "(1 - c % 2) * 8"), ns)
    with pytest.raises(AssertionError):
        check_layout(ns["pack_reference"], 129, 65, 2)
