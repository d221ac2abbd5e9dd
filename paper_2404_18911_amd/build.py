"""Build libkangaroo.so (HIP, gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_HERE)
LIB = os.path.join(_HERE, "libkangaroo.so")
SOURCES = [os.path.join(_HERE, "csrc", "kangaroo.hip")]
HEADERS = [os.path.join(_HERE, "csrc", "kernels.hip.h"), os.path.join(_HERE, "csrc", "train.hip.h"),
           os.path.join(_ROOT, "include", "kangaroo.h")]


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(p) > t for p in SOURCES + HEADERS)


_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17",
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
          # leading scalar kernel arguments arrive in SGPRs at wave start (no scalar load before the
          # first weight address can be formed)
          "-mllvm", "-amdgpu-kernarg-preload-count=16",
          "-I", os.path.join(_ROOT, "include"), "-I", os.path.join(_HERE, "csrc")]


def device_asm(out_path: str) -> str:
    """The device code of the library as gfx950 assembly, with the flags of build() (for checks of
    the generated code; nothing runs it)."""
    cmd = ["hipcc"] + _FLAGS + ["--cuda-device-only", "-S", "-o", out_path] + SOURCES
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout + res.stderr)
    return out_path


def build(force: bool = True, verbose: bool = False) -> str:
    """Compile the library for gfx950.  Packed-FP32 instruction selection is switched off."""
    if not force and not stale():
        return LIB
    cmd = ["hipcc"] + _FLAGS + ["-fPIC", "-shared", "-o", LIB] + SOURCES
    if verbose:
        print(" ".join(cmd))
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout + res.stderr)
    return LIB


MICROBENCH = [os.path.join(_HERE, "csrc", "microbench", n) for n in ("mfma_rate.hip", "prompt_gemm_loop_model.hip")]


def build_microbench(out_dir: str | None = None) -> list[str]:
    """Compile the stand-alone measurement programs of csrc/microbench (nothing in the library or the
    tests runs them; profiles/ holds what they printed on an MI355X)."""
    out_dir = out_dir or os.path.join(_HERE, "csrc", "microbench")
    outs = []
    for src in MICROBENCH:
        exe = os.path.join(out_dir, os.path.splitext(os.path.basename(src))[0])
        res = subprocess.run(["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                              "-o", exe, src], capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError("hipcc failed:\n" + res.stdout + res.stderr)
        outs.append(exe)
    return outs


if __name__ == "__main__":
    print(build(verbose=True))
