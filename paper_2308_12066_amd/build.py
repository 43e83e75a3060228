"""Build libpgmoe.so (hand-written HIP for gfx950) in-tree with hipcc.

    python -m paper_2308_12066_amd.build

Objects go to paper_2308_12066_amd/_build/, the library to paper_2308_12066_amd/libpgmoe.so.
"""
from __future__ import annotations

import os
import re
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
    # the one inline-assembly statement (direct-to-LDS load) names M0 as clobbered, which the
    # compiler accepts with a warning about reserved registers
    "-Wno-inline-asm",
    # per-kernel register / scratch figures as remarks: checked below, kept in _build/
    "-Rpass-analysis=kernel-resource-usage",
    # do not let the compiler form packed-fp32 VALU instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # matrix-core accumulators in ordinary vector registers (the register file is unified on this
    # chip): with the accumulator-register form the register allocator copies accumulators
    # between registers inside the k loops, and every such copy waits for the product before it
    "-mllvm", "-amdgpu-mfma-vgpr-form=1",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


# Kernels that count their own outstanding loads (s_waitcnt vmcnt(N) written by hand): a register
# spill or any other scratch access the compiler added would be one more vector-memory operation
# in that count and a stage could be read from LDS before it has landed.  The build fails if one
# of them uses scratch memory.
NO_SCRATCH_KERNELS = ("ffn_gemm_tile_kernel",)


def resource_usage(remarks: str) -> dict:
    """{mangled kernel name: {"ScratchSize [bytes/lane]": n, "VGPRs": n, ...}} from the compiler's
    kernel-resource-usage remarks."""
    out, cur = {}, None
    for line in remarks.splitlines():
        m = re.search(r"remark:\s+Function Name: (\S+)", line)
        if m:
            cur = out.setdefault(m.group(1), {})
            continue
        m = re.search(r"remark:\s+([A-Za-z][^:]*): (\S+) \[-Rpass-analysis", line)
        if m and cur is not None:
            cur[m.group(1).strip()] = m.group(2)
    return out


def _check_resources(src: str, usage: dict) -> None:
    for name, u in usage.items():
        if not any(k in name for k in NO_SCRATCH_KERNELS):
            continue
        bad = {k: u.get(k) for k in ("ScratchSize [bytes/lane]", "SGPRs Spill", "VGPRs Spill") if u.get(k) != "0"}
        if bad:
            raise RuntimeError(f"{src}: {name} must not use scratch memory (it counts its own loads), compiler reports {bad}")


def _compile(src: str, force: bool) -> str:
    obj = os.path.join(OBJ, src.replace(".hip", ".o"))
    path = os.path.join(CSRC, src)
    deps = [path, os.path.join(CSRC, "pgmoe_internal.h"), os.path.join(CSRC, "ffn_common.h"), os.path.join(CSRC, "gate_small.h"), os.path.join(ROOT, "include", "pgmoe.h")]
    if not force and os.path.exists(obj) and all(os.path.getmtime(obj) >= os.path.getmtime(d) for d in deps):
        return obj
    r = subprocess.run([HIPCC, *FLAGS, "-c", path, "-o", obj], stderr=subprocess.PIPE, text=True)
    usage = resource_usage(r.stderr)
    # everything but the remarks (errors, warnings) goes to the caller's stderr as usual
    shown, skip = [], 0
    for ln in r.stderr.splitlines():
        if "-Rpass-analysis=kernel-resource-usage" in ln:
            skip = 2 if "Function Name" in ln else 0    # the remark's source line and caret follow the first one
            continue
        if skip and (ln.lstrip()[:1].isdigit() or ln.strip().startswith("|")):
            skip -= 1
            continue
        skip = 0
        if "packed-fp32-ops" not in ln:
            shown.append(ln)
    if shown:
        print("\n".join(shown), file=sys.stderr)
    if r.returncode:
        raise subprocess.CalledProcessError(r.returncode, r.args)
    with open(obj.replace(".o", ".resources.txt"), "w") as fh:
        for name, u in sorted(usage.items()):
            fh.write(name + "  " + "  ".join(f"{k}={v}" for k, v in u.items()) + "\n")
    _check_resources(src, usage)
    return obj


def build(force: bool = True, jobs: int = 6) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=jobs) as pool:
        objs = list(pool.map(lambda s: _compile(s, force), SOURCES))
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs], check=True)
    return LIB


if __name__ == "__main__":
    print(build(force="--incremental" not in sys.argv))
