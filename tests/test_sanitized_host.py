"""CPU-only builds with AddressSanitizer and UndefinedBehaviorSanitizer.

1. The fp64 oracle: every routine once on heap blocks of exactly the documented sizes
   (tests/sanitize/oracle_driver.c); a planted one-element-short cache must be reported,
   which shows the build would catch such a slip.
2. The host layer of the HIP library (argument checks, sizes, stream-K plans: the entry
   points that touch no device), host code instrumented, over a sweep of shapes
   (tests/sanitize/host_driver.cpp).

The programs are built in a temporary directory; nothing is loaded into this process.
"""
import os
import shutil
import subprocess
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")


def run(cmd, **kw):
    return subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, **kw)


def build_oracle_driver(out, extra=()):
    cmd = ["gcc", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all", "-static-libasan", *extra, "-o", out,
           os.path.join(SAN, "oracle_driver.c"), "-lm"]
    r = run(cmd)
    assert r.returncode == 0, r.stdout[-2000:]


def test_oracle_runs_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_driver")
    build_oracle_driver(exe)
    r = run([exe], env=ENV, timeout=120)
    assert r.returncode == 0 and r.stdout.strip().endswith("ok"), r.stdout[-3000:]


def test_a_planted_short_buffer_is_reported(tmp_path):
    exe = str(tmp_path / "oracle_driver_short")
    build_oracle_driver(exe, extra=("-DPLANT_SHORT_CACHE",))
    r = run([exe], env=ENV, timeout=120)
    assert r.returncode != 0 and "heap-buffer-overflow" in r.stdout, r.stdout[-3000:]


def test_host_layer_runs_clean_under_asan_and_ubsan(tmp_path):
    from paper_2211_05102_amd import build as B
    clangxx = "/opt/rocm/lib/llvm/bin/clang++"
    if not (os.path.exists(B.HIPCC) and os.path.exists(clangxx)):
        pytest.skip("no ROCm toolchain")
    san_host = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                "-Xarch_host", "-fno-sanitize-recover=all"]
    flags = [f for f in B.FLAGS if f != "-O3"] + ["-O1", "-g", *san_host]

    def compile_one(src):
        obj = str(tmp_path / src.replace(".hip", ".o"))
        r = run([B.HIPCC, *flags, "-c", os.path.join(B.CSRC, src), "-o", obj])
        assert r.returncode == 0, r.stdout[-2000:]
        return obj

    with ThreadPoolExecutor(max_workers=6) as ex:
        objs = list(ex.map(compile_one, B.SOURCES))
    drv = str(tmp_path / "host_driver.o")
    r = run([clangxx, "-O1", "-g", "-std=c++17", "-fsanitize=address", "-fsanitize=undefined",
             "-fno-sanitize-recover=all", "-I" + os.path.join(ROOT, "include"), "-c",
             os.path.join(SAN, "host_driver.cpp"), "-o", drv])
    assert r.returncode == 0, r.stdout[-2000:]
    exe = str(tmp_path / "host_driver")
    r = run([B.HIPCC, "--offload-arch=gfx950", "-fsanitize=address", "-fsanitize=undefined", drv, *objs, "-o", exe])
    assert r.returncode == 0, r.stdout[-2000:]
    r = run([exe], env=ENV, timeout=300)
    assert r.returncode == 0 and r.stdout.strip().endswith("ok"), r.stdout[-3000:]
    shutil.rmtree(tmp_path, ignore_errors=True)
