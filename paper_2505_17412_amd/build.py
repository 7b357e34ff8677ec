"""Build the HIP library (``libssa_hip.so``) for gfx950 with hipcc; one object per source, linked in-tree."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "lib", "libssa_hip.so")

SOURCES = ["ssa_api.hip", "build_blocks.hip", "generic_kernels.hip", "mfma_path.hip", "mfma_fwd.hip", "mfma_bwd.hip", "mfma_slc.hip", "cmp_module.hip", "gate.hip", "linear.hip", "layer.hip", "sel_index.hip", "profile.hip"]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-result",
    "-fno-honor-nans", "-mno-amdgpu-ieee",  # no NaN is ever produced on purpose; saves the canonicalising v_max
    "-mllvm", "-amdgpu-mfma-vgpr-form",  # keep MFMA accumulators in VGPRs: the softmax rescales them every tile
]


# Per-file additions.  The block-centric selection kernels and their merges are long straight-line tile code with no
# barrier: the ILP-driven iterative scheduler orders them better than the default one (measured per kernel: partial merge
# -16 %, selection dQ -7 %, selection forward -3 %), while it makes the barrier-pipelined kernels much slower, so it is
# applied to that one file only.
EXTRA_FLAGS = {"mfma_slc.hip": ["-mllvm", "-amdgpu-sched-strategy=iterative-ilp"]}


def _hipcc() -> str:
    for c in ("/opt/rocm/bin/hipcc", "hipcc"):
        if os.path.sep not in c or os.path.exists(c):
            return c
    return "hipcc"


def build(force: bool = True, verbose: bool = False) -> str:
    os.makedirs(OBJ, exist_ok=True)
    os.makedirs(os.path.dirname(LIB), exist_ok=True)
    headers = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    headers.append(os.path.join(HERE, "..", "include", "ssa.h"))
    newest_h = max(os.path.getmtime(h) for h in headers)

    def compile_one(src: str) -> str:
        s = os.path.join(CSRC, src)
        o = os.path.join(OBJ, src.replace(".hip", ".o"))
        if force or not os.path.exists(o) or os.path.getmtime(o) < max(os.path.getmtime(s), newest_h):
            cmd = [_hipcc(), *FLAGS, *EXTRA_FLAGS.get(src, []), "-c", s, "-o", o]
            if verbose:
                print(" ".join(cmd), flush=True)
            subprocess.check_call(cmd)
        return o

    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(compile_one, SOURCES))
    tmp = LIB + f".tmp{os.getpid()}"
    subprocess.check_call([_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs])
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(force="--incremental" not in sys.argv, verbose=True))
