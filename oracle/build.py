"""Compile the C oracle into oracle/liboracle.so (gcc, OpenMP).

Flags follow the paper's experimental setup (-O3 -fstrict-aliasing -DNDEBUG, Sec. 4) minus
-march=native: the library is built on one machine and loaded on another, so it must not
contain instructions chosen for the build host.
"""
from __future__ import annotations

import pathlib
import subprocess

HERE = pathlib.Path(__file__).resolve().parent
SRCS = [HERE / "tstgemm_oracle.c", HERE / "variants_oracle.c"]
LIB = HERE / "liboracle.so"
CFLAGS = ["-O3", "-fstrict-aliasing", "-DNDEBUG", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra"]


def build(force: bool = True) -> pathlib.Path:
    if not force and LIB.exists() and all(LIB.stat().st_mtime >= s.stat().st_mtime for s in SRCS):
        return LIB
    cmd = ["gcc", *CFLAGS, *map(str, SRCS), "-o", str(LIB), "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build())
