"""Host code under AddressSanitizer + UndefinedBehaviorSanitizer (no GPU involved).

Two small programs are built and run here:
 * tests/sanitize/oracle_driver.c together with oracle/kvqp_oracle.c (the CPU checker): every entry
   point over caches of all bit widths, group sizes, both key axes, ragged token counts and outlier
   lists, with buffers of exactly the stated sizes;
 * tests/sanitize/abi_driver.cpp together with csrc/kvqp_api.cpp (the C ABI's argument checks and
   size arithmetic), the GPU side replaced by counting stand-ins: rejected calls enqueue nothing,
   host arrays are read over exactly the documented length.
A sanitizer report makes the program exit non-zero, which fails the test.
"""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")


def run(cmd, **kw):
    r = subprocess.run(cmd, capture_output=True, text=True, timeout=300, **kw)
    assert r.returncode == 0, f"{' '.join(cmd)}\n{r.stdout[-3000:]}\n{r.stderr[-6000:]}"
    return r.stdout


def test_cpu_checker_is_clean_under_asan_and_ubsan(tmp_path):
    if shutil.which("gcc") is None:
        pytest.skip("no C compiler")
    exe = str(tmp_path / "oracle_driver")
    run(["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
         "-static-libasan", "-static-libubsan", os.path.join(SAN, "oracle_driver.c"),
         os.path.join(ROOT, "oracle", "kvqp_oracle.c"), "-lm", "-o", exe])
    out = run([exe], env=ENV)
    assert "cases clean" in out


def test_c_abi_host_side_is_clean_under_asan_and_ubsan(tmp_path):
    clang = "/opt/rocm/lib/llvm/bin/clang++"
    if shutil.which("hipcc") is None or not os.path.exists(clang):
        pytest.skip("no hipcc")
    flags = ["-x", "hip", "--cuda-host-only", "-O1", "-g", "-std=c++17", "-Xarch_host", "-fsanitize=address", "-Xarch_host",
             "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=all", "-I" + os.path.join(ROOT, "include"),
             "-I" + os.path.join(ROOT, "paper_2412_12706_amd", "csrc")]
    objs = []
    for src in (os.path.join(ROOT, "paper_2412_12706_amd", "csrc", "kvqp_api.cpp"), os.path.join(SAN, "abi_driver.cpp")):
        obj = str(tmp_path / (os.path.basename(src) + ".o"))
        run(["hipcc"] + flags + ["-c", src, "-o", obj])
        objs.append(obj)
    exe = str(tmp_path / "abi_driver")
    run([clang, "-fsanitize=address", "-fsanitize=undefined"] + objs + ["-o", exe])
    out = run([exe], env=ENV)
    assert "abi_driver: clean" in out
