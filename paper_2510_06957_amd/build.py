"""Build libtstgemm.so (HIP, gfx950 only) in-tree with hipcc.

    python -m paper_2510_06957_amd.build

Packed-fp32 instruction selection is switched off for the device code
(-Xclang -target-feature -Xclang -packed-fp32-ops); the host pass warns that it does not
know the feature, which is harmless.
"""
from __future__ import annotations

import os
import pathlib
import shutil
import subprocess

HERE = pathlib.Path(__file__).resolve().parent
ROOT = HERE.parent
CSRC = HERE / "csrc"
LIB = HERE / "libtstgemm.so"
SOURCES = ["tcsc_host.cpp", "reblock.hip", "tstgemm_side.hip", "tstgemm_large.hip", "tstgemm_small.hip",
           "tstgemm_decode.hip", "tstgemm_packed.hip", "probes.hip", "tstgemm_noalloc.hip"]
ARCH = "gfx950"


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found: libtstgemm needs the ROCm toolchain")
    return exe


def command(out: pathlib.Path = LIB, extra: list[str] | None = None) -> list[str]:
    cmd = [hipcc(), f"--offload-arch={ARCH}", "-O3", "-std=c++17", "-fPIC", "-shared", "-x", "hip",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wall", "-Wno-unused-command-line-argument",
           f"-I{ROOT / 'include'}", f"-I{CSRC}"]
    cmd += [str(CSRC / s) for s in SOURCES]
    cmd += extra or []
    cmd += ["-o", str(out)]
    return cmd


def build(verbose: bool = False) -> pathlib.Path:
    cmd = command()
    if verbose:
        print(" ".join(cmd))
    r = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in r.stderr.splitlines() if noise not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed ({r.returncode}):\n{err}")
    if verbose and err.strip():
        print(err)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
