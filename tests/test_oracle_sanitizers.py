"""The CPU oracle under AddressSanitizer + UndefinedBehaviorSanitizer (host code only).

Builds tests/sanitize/oracle_under_sanitizers.c, which includes the oracle's source, with
-fsanitize=address,undefined and runs it: every buffer has exactly its documented size and
the shapes are ragged, so an out-of-range index anywhere in the oracle aborts the run."""
import os
import shutil
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "sanitize", "oracle_under_sanitizers.c")


def build(tmp_path, extra):
    exe = str(tmp_path / "oracle_san")
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all", "-static-libasan", *extra, "-o", exe, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return exe


def run(exe):
    env = dict(os.environ)
    env.pop("LD_PRELOAD", None)                      # the sanitizer runtime must come first
    env["ASAN_OPTIONS"] = "detect_leaks=1:abort_on_error=0:verify_asan_link_order=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1"
    return subprocess.run([exe], env=env, capture_output=True, text=True, timeout=300)


@pytest.mark.skipif(shutil.which("gcc") is None, reason="no gcc")
def test_oracle_is_clean_under_asan_and_ubsan(tmp_path):
    r = run(build(tmp_path, []))
    assert r.returncode == 0, r.stdout + r.stderr
    assert "oracle clean under sanitizers" in r.stdout


@pytest.mark.skipif(shutil.which("gcc") is None, reason="no gcc")
def test_the_sanitizer_build_notices_an_overread(tmp_path):
    """The same program with a planted mistake in the included oracle source (the row scale read one
    past the end for the last row) must fail: shows the harness would catch such a thing."""
    text = open(os.path.join(HERE, "..", "oracle", "codegemm_oracle.c")).read()
    old = "(g == -1) ? half_bits_to_double(scales[n])"
    assert text.count(old) == 1
    bad_oracle = tmp_path / "codegemm_oracle.c"
    bad_oracle.write_text(text.replace(old, "(g == -1) ? half_bits_to_double(scales[n + 1])"))
    driver = open(SRC).read().replace('#include "../../oracle/codegemm_oracle.c"', f'#include "{bad_oracle}"')
    src2 = tmp_path / "driver.c"
    src2.write_text(driver)
    exe = str(tmp_path / "oracle_san_bad")
    subprocess.run(["gcc", "-O1", "-g", "-std=c11", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                    "-static-libasan", "-o", exe, str(src2), "-lm"], check=True)
    r = run(exe)
    assert r.returncode != 0
    assert "AddressSanitizer" in r.stderr
