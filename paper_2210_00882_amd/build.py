"""Builds libmsrl.so (HIP, gfx950) next to this file: `python -m paper_2210_00882_amd.build`."""
from __future__ import annotations

import glob
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libmsrl.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-fPIC", "-std=c++17",
    # packed fp32 instructions are kept out of the generated code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
] + os.environ.get("MSRL_EXTRA_FLAGS", "").split()


# Flags for single translation units (by file-name prefix).  The lin-Gauss kernel's tile loops (32 tiles of a
# 256-unit fp32 layer with the output layer's arithmetic between them) are longer than the compiler's limit for
# loops it unrolls on request; not unrolled, the register arrays they index end up in scratch memory.
PER_FILE = {
    "inst_l17_": ["-mllvm", "-pragma-unroll-threshold=200000"],
    "inst_family_h256_f32_": ["-mllvm", "-pragma-unroll-threshold=200000"],
}


def _compile(src: str) -> str:
    name = os.path.basename(src)
    obj = os.path.join(OBJ, name + ".o")
    extra = [f for prefix, fl in PER_FILE.items() if name.startswith(prefix) for f in fl]
    subprocess.check_call([HIPCC, *FLAGS, *extra, "-c", src, "-o", obj], stderr=subprocess.STDOUT)
    return obj


def build(jobs: int = 8) -> str:
    os.makedirs(OBJ, exist_ok=True)
    sources = sorted(glob.glob(os.path.join(CSRC, "*.hip")))
    with ThreadPoolExecutor(max_workers=jobs) as pool:
        objs = list(pool.map(_compile, sources))
    subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs])
    return LIB


if __name__ == "__main__":
    print(build(int(sys.argv[1]) if len(sys.argv) > 1 else 8))
