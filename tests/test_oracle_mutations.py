"""Do the pins bite?  Each case plants one plausible mistake in a COPY of the CPU oracle's
source (a dropped term, a transposed index, a wrong stride, a missing scale, a conversion
slip), compiles the copy, swaps it in for the oracle's library, and requires that at least
one pin from tests/test_oracle_pins.py fails.  The unmodified source must pass the same
battery.  Everything here runs on the CPU; the mistakes live in the oracle copy only."""
import ctypes
import os
import subprocess

import pytest

import oracle
import test_oracle_pins as pins

SRC = os.path.join(os.path.dirname(os.path.abspath(oracle.__file__)), "codegemm_oracle.c")

# (name, text in the source, replacement).  Every pattern must occur exactly once.
MUTATIONS = [
    ("first codebook dropped when m > 1",
     "            for (int c = 0; c < m; ++c) {\n                int code = codes[",
     "            for (int c = (m > 1); c < m; ++c) {\n                int code = codes["),
    ("code array read as [m][K/v][N]",
     "codes[((size_t)c * N + n) * J + j];",
     "codes[((size_t)c * J + j) * N + n];"),
    ("centroid vector reversed",
     "sum += cb[((size_t)c * ORACLE_CENTROIDS + code) * v + k];",
     "sum += cb[((size_t)c * ORACLE_CENTROIDS + code) * v + (v - 1 - k)];"),
    ("codebook stride of 255 centroids",
     "sum += cb[((size_t)c * ORACLE_CENTROIDS + code) * v + k];",
     "sum += cb[((size_t)c * (ORACLE_CENTROIDS - 1) + code) * v + k];"),
    ("weights written sub-vector-major",
     "            w[kk] = scale * sum;",
     "            w[(size_t)k * J + j] = scale * sum;"),
    ("scale not applied",
     "            w[kk] = scale * sum;",
     "            w[kk] = sum;"),
    ("group scale of the next group",
     "scales[(size_t)n * (K / g) + (v * j) / g]",
     "scales[(size_t)n * (K / g) + ((v * j) / g + 1) % (K / g)]"),
    ("groups counted in vectors, not weights",
     "scales[(size_t)n * (K / g) + (v * j) / g]",
     "scales[(size_t)n * (K / g) + (j / g) % (K / g)]"),
    ("row scale of the neighbouring row",
     "(g == -1) ? half_bits_to_double(scales[n])",
     "(g == -1) ? half_bits_to_double(scales[(n + 1) % N])"),
    ("every batch row reads x[0]",
     "const double *xb = xd + (size_t)b * K;",
     "const double *xb = xd;"),
    ("sum of terms instead of sum of |terms|",
     "sum_abs += fabs(term);",
     "sum_abs += term;"),
    ("last element of the dot product skipped",
     "for (int kk = 0; kk < K; ++kk) {\n                        double term",
     "for (int kk = 0; kk < K - 1; ++kk) {\n                        double term"),
    ("half exponent bias off by one",
     "mag = ldexp((double)(frac | 0x400), expo - 25);",
     "mag = ldexp((double)(frac | 0x400), expo - 24);"),
    ("half subnormals flushed to zero",
     "mag = ldexp((double)frac, -24);               /* zero and subnormals */",
     "mag = 0.0;"),
    ("half sign ignored",
     "return sign ? -mag : mag;",
     "return mag;"),
    ("psumbook activations reversed inside a sub-vector",
     "half_bits_to_double(x[(size_t)b * K + (size_t)v * j + k]);",
     "half_bits_to_double(x[(size_t)b * K + (size_t)v * j + (v - 1 - k)]);"),
    ("psumbook stored as [B][K/v][m][256]",
     "P[(((size_t)b * m + c) * J + j) * ORACLE_CENTROIDS + i] = sum;",
     "P[(((size_t)b * J + j) * m + c) * ORACLE_CENTROIDS + i] = sum;"),
]


def battery():
    """A subset of the pins that runs in about a second: (callable, args)."""
    b = []
    for args in [(32, 4, 8, 1, 1), (16, 3, 8, 2, 3), (24, 7, 4, 3, 1), (32, 3, 16, 3, 2)]:
        b.append((pins.test_brute_force_exact_rational, args))
    b.append((pins.test_gather_identity_and_op_counts, (256, 65, 4, 1, 3)))
    b.append((pins.test_gather_identity_and_op_counts, (328, 33, 8, 3, 1)))
    for f in (pins.test_psumbook_eq2_brute_force, pins.test_psumbook_one_hot_centroids_copy_x_all_half_patterns,
              pins.test_psumbook_one_hot_x_reads_codebook, pins.test_zero_codebook_gives_zero_and_drops_out,
              pins.test_one_hot_centroids_gather_sum_of_x, pins.test_scale_linearity_power_of_two,
              pins.test_row_permutation_equivariance, pins.test_constant_codes_make_rows_proportional_to_scale,
              pins.test_sub_vector_position_matters, pins.test_dequantize_consistent_with_gemm,
              pins.test_one_group_per_row_is_the_row_scale, pins.test_equal_group_scales_reduce_to_row_scale,
              pins.test_group_scale_linearity_and_locality, pins.test_group_boundaries_sit_at_multiples_of_g):
        b.append((f, ()))
    b.append((pins.test_sign_codebook_equals_integer_matrix_product, (-1.0,)))
    for args in [(32, 3, 8, 2, 2, 16), (24, 5, 4, 1, 1, 12), (16, 2, 4, 3, 2, 4)]:
        b.append((pins.test_groups_brute_force_exact_rational, args))
    b.append((pins.test_groups_gather_identity, (512, 65, 8, 2, 2, 128)))
    return b


def compile_variant(tmp_path, name, text):
    src = tmp_path / f"{name}.c"
    lib = tmp_path / f"lib{name}.so"
    src.write_text(text)
    subprocess.run(["gcc", "-O1", "-fPIC", "-shared", "-std=c11", "-o", str(lib), str(src), "-lm"], check=True)
    h = ctypes.CDLL(str(lib))
    i, p = ctypes.c_int, ctypes.c_void_p
    h.oracle_num_threads.restype = i
    h.oracle_dequantize.argtypes = [i, i, i, i, i, p, p, p, p]
    h.oracle_dequantize.restype = i
    h.oracle_gemm.argtypes = [i, i, i, i, i, i, p, p, p, p, p, p]
    h.oracle_gemm.restype = i
    h.oracle_psumbook.argtypes = [i, i, i, i, p, p, p]
    h.oracle_psumbook.restype = i
    return h


def failures_with(lib):
    """Runs the battery with `lib` standing in for the oracle's library; names of the pins that failed."""
    oracle._load()
    saved = oracle._lib
    oracle._lib = lib
    failed = []
    try:
        for fn, args in battery():
            try:
                fn(*args)
            except Exception:          # an assertion, or an exception a broken oracle provokes
                failed.append(fn.__name__)
    finally:
        oracle._lib = saved
    return failed


def test_unmodified_source_passes_the_battery(tmp_path):
    lib = compile_variant(tmp_path, "clean", open(SRC).read())
    assert failures_with(lib) == []


@pytest.mark.parametrize("name,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_planted_mistake_is_caught(tmp_path, name, old, new):
    text = open(SRC).read()
    assert text.count(old) == 1, f"mutation site for '{name}' not found exactly once"
    lib = compile_variant(tmp_path, "mutant", text.replace(old, new))
    failed = failures_with(lib)
    assert failed, f"no pin noticed: {name}"
