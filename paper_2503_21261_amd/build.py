"""Builds libhot.so (the C-ABI library of HIP kernels) in-tree for gfx950."""
from __future__ import annotations

import os
import shlex
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libhot.so")
SOURCES = ["api.hip", "row_quant.hip", "col_quant.hip", "gx_front.hip", "col_bf16.hip", "gy_fused.hip", "igemm.hip", "select.hip", "profile.hip", "probe.hip"]

# IEEE fp32 is part of the contract: the integer codes depend on every add, mul and
# div rounding exactly once, so no contraction, no fast-math, correctly rounded
# division.  Packed fp32 instructions are disabled for the test machines.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
         "-fno-fast-math", "-fhip-fp32-correctly-rounded-divide-sqrt",
         "-fno-gpu-flush-denormals-to-zero",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def _hipcc() -> str:
    for cand in ("hipcc", "/opt/rocm/bin/hipcc"):
        try:
            subprocess.run([cand, "--version"], check=True, capture_output=True)
            return cand
        except (OSError, subprocess.CalledProcessError):
            continue
    raise RuntimeError("hipcc not found")


def build(verbose: bool = False) -> str:
    """Compile every .hip source and link libhot.so.  Always recompiles.  For experiments,
    HOT_HIPCC_FLAGS adds compiler flags (e.g. -DNAME) and HOT_LIB_OUT names another output."""
    hipcc = _hipcc()
    extra = shlex.split(os.environ.get("HOT_HIPCC_FLAGS", ""))
    lib_out = os.environ.get("HOT_LIB_OUT", LIB)
    os.makedirs(OBJ, exist_ok=True)

    def compile_one(src: str) -> str:
        obj = os.path.join(OBJ, src.replace(".hip", ".o"))
        cmd = [hipcc, *FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
        res = subprocess.run(cmd, capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{res.stdout}\n{res.stderr}")
        if verbose:
            noise = "not a recognized feature"
            sys.stderr.write("".join(l + "\n" for l in res.stderr.splitlines() if noise not in l))
        return obj

    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(compile_one, SOURCES))
    res = subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib_out, *objs],
                         capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"link failed:\n{res.stdout}\n{res.stderr}")
    return lib_out


if __name__ == "__main__":
    print(build(verbose=True))
