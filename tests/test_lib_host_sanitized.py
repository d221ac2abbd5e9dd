"""The library's host code under AddressSanitizer and UndefinedBehaviorSanitizer.

csrc/kangaroo.hip is compiled with the host side instrumented (the device code is compiled as usual
and never runs here) and linked with tests/native/lib_host_san_driver.c, which calls what the
library does without a device: configuration checks, size arithmetic, call-order errors, Eq. 1 /
Eq. 2, the tile order for every K, the argument checks of the stand-alone ops.  The run must end with
every check held and without a sanitizer report.  An executable of its own is used because an
instrumented shared library could only be loaded into the test process by preloading the sanitizer
runtime."""
import os
import shutil
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CLANG = "/opt/rocm/lib/llvm/bin/clang"


def test_library_host_paths_are_clean_under_sanitizers(tmp_path):
    if shutil.which("hipcc") is None or not os.path.exists(CLANG):
        pytest.skip("hipcc / clang not available")
    inc = ["-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_2404_18911_amd", "csrc")]
    obj, drv, exe = str(tmp_path / "kg.o"), str(tmp_path / "drv.o"), str(tmp_path / "drv")
    steps = [
        ["hipcc", "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-omit-frame-pointer",
         *inc, "-c", os.path.join(ROOT, "paper_2404_18911_amd", "csrc", "kangaroo.hip"), "-o", obj],
        [CLANG, "-O1", "-g", "-fsanitize=address,undefined", "-fno-omit-frame-pointer", *inc, "-c",
         os.path.join(HERE, "native", "lib_host_san_driver.c"), "-o", drv],
        ["hipcc", "--offload-arch=gfx950", "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize", obj, drv, "-o", exe],
    ]
    for cmd in steps:
        res = subprocess.run(cmd, capture_output=True, text=True)
        assert res.returncode == 0, (cmd[0], res.stderr[-2000:])
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:exitcode=66", UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    res = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert res.returncode == 0, res.stdout[-2000:] + res.stderr[-4000:]
    assert res.stdout.strip().endswith("OK (0 failed)")
    assert "runtime error" not in res.stderr and "AddressSanitizer" not in res.stderr
