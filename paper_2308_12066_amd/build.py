"""Build libpgmoe.so (hand-written HIP for gfx950) in-tree with hipcc.

    python -m paper_2308_12066_amd.build

Objects go to paper_2308_12066_amd/_build/, the library to paper_2308_12066_amd/libpgmoe.so.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libpgmoe.so")
SOURCES = ["api.hip", "gate.hip", "permute.hip", "ffn.hip", "ffn_gemm.hip", "combine.hip", "fetch.hip", "engine.hip"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
    # do not let the compiler form packed-fp32 VALU instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # matrix-core accumulators in ordinary vector registers (the register file is unified on this
    # chip): with the accumulator-register form the register allocator copies accumulators
    # between registers inside the k loops, and every such copy waits for the product before it
    "-mllvm", "-amdgpu-mfma-vgpr-form=1",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def _compile(src: str, force: bool) -> str:
    obj = os.path.join(OBJ, src.replace(".hip", ".o"))
    path = os.path.join(CSRC, src)
    deps = [path, os.path.join(CSRC, "pgmoe_internal.h"), os.path.join(CSRC, "ffn_common.h"), os.path.join(CSRC, "gate_small.h"), os.path.join(ROOT, "include", "pgmoe.h")]
    if not force and os.path.exists(obj) and all(os.path.getmtime(obj) >= os.path.getmtime(d) for d in deps):
        return obj
    subprocess.run([HIPCC, *FLAGS, "-c", path, "-o", obj], check=True)
    return obj


def build(force: bool = True, jobs: int = 6) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=jobs) as pool:
        objs = list(pool.map(lambda s: _compile(s, force), SOURCES))
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs], check=True)
    return LIB


if __name__ == "__main__":
    print(build(force="--incremental" not in sys.argv))
