"""Build libbf.so in-tree for gfx950 with hipcc (and the oracle's C sources, if any)."""

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OUT = os.path.join(HERE, "libbf.so")

HIP_SOURCES = ["bf_tile_f32.hip", "bf_tile_bf16.hip", "bf_pipe_f32.hip", "bf_pipe_bf16.hip", "bf_chain.hip", "bf_shift.hip", "bf_dense.hip", "bf_kernels.hip"]
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
    # one host translation unit and four device ones (the tile kernel per storage type, the chain
    # and gather kernels, everything else), compiled side by side
    jobs = [(["g++"] + COMMON, "bf_topology.cpp")]
    jobs += [([hipcc] + COMMON + DEVICE, src) for src in HIP_SOURCES]
    objs = [os.path.join(bdir, os.path.splitext(src)[0] + ".o") for _, src in jobs]
    with ThreadPoolExecutor(max_workers=min(len(jobs), max(1, (os.cpu_count() or 2) // 2))) as pool:
        list(pool.map(lambda jo: _run(jo[0][0] + ["-c", os.path.join(CSRC, jo[0][1]), "-o", jo[1]]), zip(jobs, objs)))
    _run([hipcc, "-shared", "-fPIC", "-o", OUT] + objs)
    if verbose:
        print("built", OUT)
    return OUT


if __name__ == "__main__":
    build(verbose=True)
