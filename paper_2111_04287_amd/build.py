"""Build libbf.so in-tree for gfx950 with hipcc (and the oracle's C sources, if any)."""

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OUT = os.path.join(HERE, "libbf.so")

COMMON = ["-O3", "-std=c++17", "-fPIC", "-I" + os.path.join(ROOT, "include"), "-I" + CSRC]
# packed fp32 instructions are kept off for every HIP translation unit
DEVICE = ["--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _run(cmd):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in r.stdout.splitlines() if "not a recognized feature" not in l)
    if r.returncode != 0:
        sys.stderr.write(out + "\n")
        raise RuntimeError("command failed: " + " ".join(cmd))
    return out


def build(verbose=False):
    bdir = os.path.join(HERE, "_build")
    os.makedirs(bdir, exist_ok=True)
    hipcc = os.environ.get("HIPCC", "hipcc")
    host_obj = os.path.join(bdir, "bf_topology.o")
    dev_obj = os.path.join(bdir, "bf_kernels.o")
    _run(["g++"] + COMMON + ["-c", os.path.join(CSRC, "bf_topology.cpp"), "-o", host_obj])
    _run([hipcc] + COMMON + DEVICE + ["-c", os.path.join(CSRC, "bf_kernels.hip"), "-o", dev_obj])
    _run([hipcc, "-shared", "-fPIC", "-o", OUT, host_obj, dev_obj])
    if verbose:
        print("built", OUT)
    return OUT


if __name__ == "__main__":
    build(verbose=True)
