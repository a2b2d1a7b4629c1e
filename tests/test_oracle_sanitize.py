"""The oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only).

oracle/selftest.c calls every entry point of the oracle once on small, exactly sized buffers; it
is compiled here together with the oracle with -fsanitize=address,undefined and run as its own
process, so any out-of-bounds access, use after free, signed overflow or misaligned access in the
oracle aborts it."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_is_clean_under_sanitizers(tmp_path):
    exe = str(tmp_path / "orc_selftest")
    build = subprocess.run(["gcc", "-O1", "-g", "-fopenmp", "-std=gnu11", "-Wall", "-fsanitize=address,undefined",
                            "-fno-sanitize-recover=all", "-static-libasan", "-ffp-contract=off", "-o", exe,
                            os.path.join(ROOT, "oracle", "selftest.c"), "-lm"], capture_output=True, text=True)
    assert build.returncode == 0, build.stderr
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1", OMP_NUM_THREADS="2")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert run.returncode == 0, run.stdout + run.stderr
    assert "selftest: ok" in run.stdout
