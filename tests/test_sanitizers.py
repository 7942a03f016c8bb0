"""Memory-safety checks on the CPU: the oracle's C source under AddressSanitizer + UndefinedBehaviorSanitizer,
driven over small ragged inputs by tests/sanitize/oracle_driver.c (values are pinned elsewhere)."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan"]


def _build_and_run(tmp_path, driver_source, expect_ok):
    exe = str(tmp_path / "oracle_driver")
    subprocess.run(["gcc", "-O1", "-g", "-std=c11", "-fopenmp", *SAN, "-Wall", "-Wextra", "-Werror", "-o", exe,
                    driver_source, os.path.join(ROOT, "oracle", "npd_oracle.c"), "-lm"], check=True)
    env = dict(os.environ, OMP_NUM_THREADS="4", ASAN_OPTIONS="detect_leaks=1:abort_on_error=0")
    run = subprocess.run([exe], env=env, capture_output=True, text=True, timeout=300)
    if expect_ok:
        assert run.returncode == 0, run.stderr[-3000:]
        assert "oracle driver finished" in run.stdout
    return run


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_is_clean_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    _build_and_run(tmp_path, os.path.join(ROOT, "tests", "sanitize", "oracle_driver.c"), expect_ok=True)


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_the_sanitizer_build_reports_a_planted_overflow(tmp_path):
    """The same driver with its label array one element short: the run must fail, or the check above shows nothing."""
    text = open(os.path.join(ROOT, "tests", "sanitize", "oracle_driver.c")).read()
    short = text.replace("*labels = block(4 * T)", "*labels = block(4 * T - 4)")
    assert short != text
    src = tmp_path / "driver_short.c"
    src.write_text(short)
    run = _build_and_run(tmp_path, str(src), expect_ok=False)
    assert run.returncode != 0 and "heap-buffer-overflow" in run.stderr
