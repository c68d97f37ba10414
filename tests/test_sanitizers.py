"""CPU-side code under AddressSanitizer + UndefinedBehaviorSanitizer (host code only; nothing here touches a GPU).

The oracle: tests/sanitize/oracle_driver.c is linked with oracle/hola_oracle.c under -fsanitize=address,undefined and
calls every entry point on small, ragged and degenerate inputs; any report ends the run with a non-zero status.

The library's host side: every source of libhola is compiled with the sanitizers on its host half (the device half is
built as usual and never runs) and linked with tests/sanitize/host_driver.c, which walks the argument checks, the
workspace sizing, the tuning and timing aids and, with fake device pointers, every launch sequence up to the HIP
runtime's refusal on a machine without a GPU."""
import os
import shutil
import subprocess
from concurrent.futures import ThreadPoolExecutor

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


def test_library_host_side_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    from paper_2506_18952_amd import build as hb_build
    hipcc = hb_build.hipcc()
    clang = os.path.join(os.path.dirname(os.path.realpath(hipcc)), "..", "lib", "llvm", "bin", "clang")
    if not os.path.exists(clang):
        clang = "/opt/rocm/lib/llvm/bin/clang"
    if not os.path.exists(hipcc) or not os.path.exists(clang):
        pytest.skip("no hipcc / clang")
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
           "-fno-sanitize-recover=undefined"]
    flags = [f for f in hb_build.FLAGS if f != "-O3"] + ["-O1", "-g"]

    def compile_one(src):
        obj = str(tmp_path / (os.path.splitext(src)[0] + ".o"))
        r = _run([hipcc, *flags, *san, "-c", os.path.join(hb_build.CSRC, src), "-o", obj])
        return obj, r

    with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as pool:
        results = list(pool.map(compile_one, hb_build.SOURCES))
    for obj, r in results:
        assert r.returncode == 0, r.stderr[-4000:]
    drv = str(tmp_path / "host_driver.o")
    r = _run([clang, "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-g", "-I", os.path.join(ROOT, "include"),
              "-c", os.path.join(ROOT, "tests", "sanitize", "host_driver.c"), "-o", drv])
    assert r.returncode == 0, r.stderr
    exe = str(tmp_path / "host_san")
    r = _run([hipcc, "-fsanitize=address,undefined", drv, *[o for o, _ in results], "-o", exe])
    assert r.returncode == 0, r.stderr[-4000:]
    # leaks are the HIP runtime's own start-up allocations, not the library's: not looked for here
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = _run([exe], env=env, timeout=300)
    assert run.returncode == 0, run.stdout[-4000:] + run.stderr[-4000:]
    assert "runtime error" not in run.stderr and "AddressSanitizer" not in run.stderr, run.stderr[-4000:]
    assert "failures=0 rc=0" in run.stdout
