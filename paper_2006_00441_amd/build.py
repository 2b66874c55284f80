"""Compile the HIP library for gfx950 into paper_2006_00441_amd/libdasgd.so (in-tree)."""
from __future__ import annotations

import os
import shutil
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libdasgd.so")
SOURCES = [os.path.join(CSRC, "dasgd.hip")]
DEPENDS = SOURCES + [os.path.join(CSRC, h) for h in ("kernels.hpp", "context.hpp", "tuning.hpp", "launch.hpp")] + [
    os.path.join(ROOT, "include", "dasgd.h"), os.path.join(ROOT, "include", "dasgd_diag.h")]
STUDY = os.path.join(HERE, "shape_study")            # stand-alone launch-shape study (see csrc/shape_study.hip)
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",    # keep the compiler off packed-fp32 forms
    "-Wall", "-Wextra", "-Wno-unused-command-line-argument",
]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found: the HIP library cannot be built on this machine")
    return exe


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(p) > t for p in DEPENDS)


def build(force: bool = True, extra_flags=(), out: str = LIB) -> str:
    if not force and out == LIB and not stale():
        return out
    tmp = out + f".tmp{os.getpid()}"
    cmd = [hipcc(), *HIPCC_FLAGS, *extra_flags, "-I", os.path.join(ROOT, "include"), "-o", tmp, *SOURCES]
    subprocess.run(cmd, check=True)
    os.replace(tmp, out)
    return out


def build_study(out: str = STUDY) -> str:
    """The stand-alone launch-shape study program (an executable; it times kernel variants on the GPU)."""
    flags = [f for f in HIPCC_FLAGS if f not in ("-shared", "-fPIC")]
    tmp = out + f".tmp{os.getpid()}"
    subprocess.run([hipcc(), *flags, "-o", tmp, os.path.join(CSRC, "shape_study.hip")], check=True)
    os.replace(tmp, out)
    return out


if __name__ == "__main__":
    print(build())
