"""The CPU checker under AddressSanitizer and UndefinedBehaviorSanitizer (host code only).

tests/sanitize_driver.c includes oracle/podoracle.c and calls every entry point on small awkward shapes; built
with -fsanitize=address,undefined and -fno-sanitize-recover it exits non-zero on the first out-of-bounds access,
leak or undefined operation.  A second, unsanitized build must print the same checksum: the sanitized run took
the same paths as the code the other tests pin.
"""
import os
import shutil
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "sanitize_driver.c")


def _build(tmp_path, name, flags):
    exe = str(tmp_path / name)
    cmd = ["gcc", "-std=c11", "-g", "-O1", "-ffp-contract=off", *flags, SRC, "-o", exe, "-lm"]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    return exe


@pytest.mark.skipif(shutil.which("gcc") is None, reason="no gcc")
def test_checker_runs_clean_under_address_and_undefined_sanitizers(tmp_path):
    san = _build(tmp_path, "driver_san", ["-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                                           "-static-libasan", "-fno-omit-frame-pointer"])
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:halt_on_error=1",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    r = subprocess.run([san], capture_output=True, text=True, env=env, timeout=600)
    assert r.returncode == 0, (r.stdout[-2000:], r.stderr[-4000:])
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-4000:]
    plain = _build(tmp_path, "driver_plain", [])
    p = subprocess.run([plain], capture_output=True, text=True, timeout=600)
    assert p.returncode == 0, p.stderr[-2000:]
    assert r.stdout.strip() == p.stdout.strip() and "checksum" in r.stdout
