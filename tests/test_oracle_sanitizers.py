"""The oracle's C code under AddressSanitizer and UndefinedBehaviorSanitizer (host compiler, CPU only): the driver in
tests/c/ runs the whole-step interface -- ragged batches, a model without samples, three steps in plain and in
bf16-storage-emulation mode, every query, sampling and the ANOVA -- and must finish without a report (leaks
included)."""
import os
import shutil
import subprocess
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_clean_under_asan_and_ubsan():
    if shutil.which("gcc") is None:
        pytest.skip("no host C compiler")
    with tempfile.TemporaryDirectory() as tmp:
        exe = os.path.join(tmp, "oracle_sanitized")
        cmd = ["gcc", "-O1", "-g", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
               "-fno-omit-frame-pointer", "-I" + os.path.join(ROOT, "oracle"),
               os.path.join(ROOT, "tests", "c", "oracle_sanitizer_driver.c"), os.path.join(ROOT, "oracle", "gan_oracle.c"),
               "-lm", "-o", exe]
        built = subprocess.run(cmd, capture_output=True, text=True)
        if built.returncode != 0 and "sanitize" in built.stderr:
            pytest.skip("the host compiler has no sanitizer runtime: " + built.stderr[-200:])
        assert built.returncode == 0, built.stderr[-2000:]
        env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0", UBSAN_OPTIONS="print_stacktrace=1",
                   OMP_NUM_THREADS="2")
        run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=600)
        assert run.returncode == 0 and run.stdout.strip() == "ok", (run.returncode, run.stdout[-500:], run.stderr[-3000:])
