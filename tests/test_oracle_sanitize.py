"""The C oracle under AddressSanitizer and UndefinedBehaviorSanitizer: oracle/sanitize_check.c runs every
function on small inputs (empty, ragged, ties, values beyond binary16) in a build of its own; any report ends
the run with a non-zero status.  Host only."""
import os
import shutil
import subprocess
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_is_clean_under_address_and_undefined_behaviour_sanitizers():
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    with tempfile.TemporaryDirectory() as tmp:
        exe = os.path.join(tmp, "sanitize_check")
        cmd = [gcc, "-O1", "-g", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-mfpmath=sse",
               "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-o", exe,
               os.path.join(ROOT, "oracle", "sanitize_check.c"), "-lm"]
        built = subprocess.run(cmd, capture_output=True, text=True, timeout=300)
        if built.returncode != 0 and ("asan" in built.stderr or "ubsan" in built.stderr or "sanitize" in built.stderr):
            pytest.skip("this gcc has no sanitizer runtime: " + built.stderr.strip().splitlines()[-1])
        assert built.returncode == 0, built.stderr
        env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
        run = subprocess.run([exe], capture_output=True, text=True, timeout=300, env=env)
        assert run.returncode == 0, run.stdout + run.stderr
        assert "sanitize_check ok" in run.stdout
        assert "runtime error" not in run.stderr and "AddressSanitizer" not in run.stderr, run.stderr
