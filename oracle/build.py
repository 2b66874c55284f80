"""Compile the C oracle into oracle/libdasgd_oracle.so (gcc, host only)."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SOURCES = ("dasgd_oracle.c", "dasgd_oracle_impl.h")
LIB = os.path.join(HERE, "libdasgd_oracle.so")
FLAGS = ["-O2", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-shared", "-fPIC", "-std=c11",
         "-Wall", "-Wextra"]


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(os.path.join(HERE, s)) > t for s in SOURCES)


def build(force: bool = False, out: str = LIB, source: str | None = None) -> str:
    """Compile; `source` may name another .c file (the mutation tests compile altered copies)."""
    if not force and out == LIB and not stale():
        return out
    src = source or os.path.join(HERE, "dasgd_oracle.c")
    tmp = out + f".tmp{os.getpid()}"
    subprocess.run(["gcc", *FLAGS, "-I", HERE, "-o", tmp, src], check=True)
    os.replace(tmp, out)
    return out


if __name__ == "__main__":
    print(build(force=True))
