"""Compile the HIP sources into paper_2002_03629_amd/libjacobi_made.so (gfx950 only).

hipcc cross-compiles without a GPU.  Run as `python -m paper_2002_03629_amd.build`.
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB_PATH = os.path.join(HERE, "libjacobi_made.so")
SOURCES = ["jacobi_made.hip"]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-pthread", "-Wall", "-Wno-unused-function",
    # keep the compiler from forming packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def build_library(verbose: bool = True, out_path: str = LIB_PATH, defines=(), extra_flags=()) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = ([hipcc] + FLAGS + list(extra_flags) + ["-D" + d for d in defines] + [os.path.join(CSRC, s) for s in SOURCES] +
           ["-o", out_path])
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in proc.stdout.splitlines() if "packed-fp32-ops" not in l)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)
    return out_path


PROBES = os.path.join(HERE, "probes")


def build_probes(verbose: bool = True) -> None:
    """The stand-alone measurement probes (probes/*.hip -> probes/bin/<name>): what plain loops of the kernels' shape
    reach on the chip.  The library does not use them; profiles/ quotes their output next to the kernels' figures."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(os.path.join(PROBES, "bin"), exist_ok=True)
    for name in sorted(f[:-4] for f in os.listdir(PROBES) if f.endswith(".hip")):
        cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               os.path.join(PROBES, name + ".hip"), "-o", os.path.join(PROBES, "bin", name)]
        if verbose:
            print(" ".join(cmd), flush=True)
        proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        if proc.returncode != 0:
            raise RuntimeError("hipcc failed:\n" + proc.stdout)


if __name__ == "__main__":
    build_library()
    build_probes()
    sys.exit(0)
