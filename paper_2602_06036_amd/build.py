"""Builds the HIP shared library (gfx950) in-tree: paper_2602_06036_amd/libdflash.so."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "csrc", "dflash.hip")
OUT = os.path.join(HERE, "libdflash.so")

FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-shared", "-fPIC", "-fno-gpu-rdc",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function"]


def build(verbose: bool = True) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + FLAGS + [SRC, "-o", OUT]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    # the host pass prints a harmless "not a recognized feature" note for -packed-fp32-ops
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if err.strip() and verbose:
        print(err, file=sys.stderr)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    return OUT


if __name__ == "__main__":
    build()
