"""The oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host only, CPU only): oracle/selftest.c drives
every oracle entry point on exactly-sized buffers, edge cases included; any out-of-bounds access, use after free,
signed overflow or misaligned access aborts the program."""
import os
import subprocess
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_selftest_under_asan_and_ubsan():
    src = [os.path.join(ROOT, "oracle", "selftest.c"), os.path.join(ROOT, "oracle", "aj_oracle.c")]
    with tempfile.TemporaryDirectory() as tmp:
        exe = os.path.join(tmp, "selftest")
        # sanitizer runtimes linked statically: the program must not depend on the order of preloaded libraries
        cmd = ["gcc", "-O1", "-g", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
               "-static-libasan", "-static-libubsan", *src, "-o", exe, "-lm"]
        b = subprocess.run(cmd, capture_output=True, text=True)
        if b.returncode != 0 and "cannot find" in b.stderr:
            pytest.skip("static sanitizer runtimes are not installed")
        assert b.returncode == 0, b.stderr[-2000:]
        r = subprocess.run([exe], capture_output=True, text=True, timeout=300,
                           env={**os.environ, "OMP_NUM_THREADS": "4", "ASAN_OPTIONS": "detect_leaks=1"})
        assert r.returncode == 0 and "selftest ok" in r.stdout, (r.stdout[-500:], r.stderr[-3000:])
