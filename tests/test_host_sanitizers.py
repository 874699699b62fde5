"""AddressSanitizer + UndefinedBehaviorSanitizer over the host code (no GPU needed): the C oracle in full, and
the library's host side - api.hip (argument checks, helpers, context life cycle) and padg.hip (the
macro-instance model) - compiled with the sanitizers on the host pass only.  The instrumented code is linked
into two small driver programs (tests/sanitize/), so that the sanitizer runtime comes first in the process
without any preloading; a finding makes the driver exit non-zero with the report on stderr."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2504_18154_amd", "csrc")
SAN = ["-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=undefined"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")


def _run(cmd, **kw):
    r = subprocess.run(cmd, capture_output=True, text=True, **kw)
    assert r.returncode == 0, f"{' '.join(cmd)}\n{r.stdout}\n{r.stderr[-4000:]}"
    return r


def test_oracle_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_driver")
    _run(["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-fno-omit-frame-pointer", "-static-libasan", *SAN, "-Wall", "-Wextra",
          "-o", exe, os.path.join(ROOT, "tests", "sanitize", "oracle_driver.c"),
          os.path.join(ROOT, "oracle", "ecoserve_oracle.c"), "-lm"])
    r = _run([exe], env=ENV, timeout=300)
    assert "oracle driver ok" in r.stdout and "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr


def test_library_host_code_under_asan_and_ubsan(tmp_path):
    from paper_2504_18154_amd import build as b
    hipcc = b._hipcc()
    objs = []
    for src in b.SOURCES:
        obj = str(tmp_path / src.replace(".hip", ".o"))
        # the sanitizers go to the host pass only (GPU sanitizers are not available here); the device pass is as in the product
        host_san = [x for f in SAN for x in ("-Xarch_host", f)] if src in ("api.hip", "padg.hip") else []
        flags = [f for f in b.FLAGS if f != "-O3"] + ["-O1", "-g", "-Xarch_host", "-fno-omit-frame-pointer"]
        r = subprocess.run([hipcc, *flags, *host_san, "-I", b.INCLUDE, "-c", os.path.join(CSRC, src), "-o", obj],
                           capture_output=True, text=True)
        assert r.returncode == 0, r.stderr[-3000:]
        objs.append(obj)
    # the driver is plain C++: compiled on its own, then linked with the library's objects (objects only on the link line)
    drv = str(tmp_path / "host_driver.o")
    _run([hipcc, "-x", "c++", "-std=c++17", "-O1", "-g", "-fno-omit-frame-pointer", *SAN, "-I", b.INCLUDE, "-c",
          os.path.join(ROOT, "tests", "sanitize", "host_driver.cpp"), "-o", drv])
    exe = str(tmp_path / "host_driver")
    _run([hipcc, "--offload-arch=gfx950", *SAN, "-o", exe, drv, *objs])
    # the HIP runtime's own start-up allocations are not this library's: leaks are checked in the oracle's run
    env = dict(ENV, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0")
    r = _run([exe], env=env, timeout=300)
    assert "host driver ok" in r.stdout and "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr
