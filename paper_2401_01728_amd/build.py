"""Builds the HIP libraries in-tree for gfx950 (cross-compiles without a GPU).

    python -m paper_2401_01728_amd.build

librv.so      the product: C ABI of include/rv.h (csrc/*.hip)
librvgen.so   the seeded input generator's device twin (inputs/gen.hip)
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "librv.so")
GENLIB = os.path.join(HERE, "inputs", "librvgen.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         # MFMA results that feed vector arithmetic (attention scores) stay in VGPRs instead of
         # being parked in and copied back from the accumulator registers
         "-mllvm", "-amdgpu-mfma-vgpr-form",
         "-Wno-unused-command-line-argument"]


def _run(cmd):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError("build failed: %s\n%s" % (" ".join(cmd), out))
    return out


def sources():
    return sorted(f for f in os.listdir(CSRC) if f.endswith(".hip"))


def build(verbose=False, jobs=None):
    os.makedirs(OBJ, exist_ok=True)
    jobs = jobs or min(8, os.cpu_count() or 1)
    srcs = sources()

    def cc(f):
        o = os.path.join(OBJ, f[:-4] + ".o")
        out = _run([HIPCC] + FLAGS + ["-c", os.path.join(CSRC, f), "-o", o])
        if verbose and out.strip():
            print(out)
        return o

    with ThreadPoolExecutor(jobs) as ex:
        objs = list(ex.map(cc, srcs))
    _run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs)
    _run([HIPCC] + FLAGS + ["-shared", os.path.join(HERE, "inputs", "gen.hip"), "-o", GENLIB])
    return LIB, GENLIB


if __name__ == "__main__":
    print(build(verbose=True))
    sys.exit(0)
