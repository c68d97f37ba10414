"""CPU-side code under AddressSanitizer + UndefinedBehaviorSanitizer (host code only; nothing here touches a GPU).

The oracle: tests/sanitize/oracle_driver.c is linked with oracle/hola_oracle.c under -fsanitize=address,undefined and
calls every entry point on small, ragged and degenerate inputs; any report ends the run with a non-zero status."""
import os
import shutil
import subprocess

import pytest

from conftest import ROOT


def _run(cmd, **kw):
    return subprocess.run(cmd, capture_output=True, text=True, **kw)


def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    exe = tmp_path / "oracle_san"
    build = _run([gcc, "-O1", "-g", "-std=c99", "-Wall", "-Wextra", "-fsanitize=address,undefined",
                  "-fno-sanitize-recover=undefined", "-static-libasan", "-fopenmp", "-o", str(exe),
                  os.path.join(ROOT, "tests", "sanitize", "oracle_driver.c"), os.path.join(ROOT, "oracle", "hola_oracle.c"), "-lm"])
    assert build.returncode == 0, build.stderr
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = _run([str(exe)], env=env, timeout=300)
    assert run.returncode == 0, run.stdout + run.stderr
    assert "runtime error" not in run.stderr and "AddressSanitizer" not in run.stderr, run.stderr
    assert "rc=0" in run.stdout
