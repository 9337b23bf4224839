"""Compiles libblink.so (HIP, gfx950) in-tree. Run as `python -m paper_2604_07609_amd.build`."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "libblink.so")
SRC = os.path.join(HERE, "csrc", "blink.hip")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def build(verbose=True):
    cmd = [HIPCC] + FLAGS + ["-o", LIB, SRC, "-lpthread"]
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + r.stdout + err)
    if verbose and err.strip():
        print(err)
    return LIB


if __name__ == "__main__":
    build()
    sys.exit(0)
