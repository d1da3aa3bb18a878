"""Build the gfx950 shared library in-tree with hipcc (cross-compiles without a GPU).

    python -m paper_2604_15408_amd.build            # build libragged_hip.so next to this file
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor
from pathlib import Path

PKG = Path(__file__).resolve().parent
ROOT = PKG.parent
CSRC = PKG / "csrc"
LIB = PKG / "libragged_hip.so"
BUILD_DIR = PKG / "_build"
SOURCES = ["ragged_api.hip", "pack_unpack.hip", "attn.hip", "linear.hip", "mask.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
    # never let the compiler form packed-fp32 VALU ops (unreliable on this target)
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    f"-I{ROOT / 'include'}", f"-I{CSRC}",
]


# linear.hip: keep MFMA results in plain VGPRs.  Where LDS use limits a CU to one work-group the
# compiler otherwise moves accumulators to AGPRs and copies them back and forth around every MFMA.
#
# The short kernels (attention, pack / unpack, mask producer): the first 14 dwords of a kernel's arguments arrive in scalar registers with the
# wavefront instead of being fetched by its first instructions (the attention kernel orders its parameters
# by first use).  Measured side by side: attention and the 36-kernel pipeline 2-3 % faster; the linear
# layers, whose launches last 8-90 us, 1-2 % slower with it, so they are built without.
PRELOAD = ["-mllvm", "-amdgpu-kernarg-preload-count=14"]
PER_FILE_FLAGS = {"linear.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"], "attn.hip": PRELOAD, "pack_unpack.hip": PRELOAD,
                  "mask.hip": PRELOAD}


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def build(verbose: bool = False, extra_flags=()) -> Path:
    """Compile every HIP source for gfx950 and link the C-ABI shared library.  Always recompiles."""
    BUILD_DIR.mkdir(exist_ok=True)
    hipcc = _hipcc()

    def compile_one(name: str) -> Path:
        obj = BUILD_DIR / (name + ".o")
        cmd = [hipcc, *HIPCC_FLAGS, *PER_FILE_FLAGS.get(name, []), *extra_flags, "-c", str(CSRC / name), "-o", str(obj)]
        res = subprocess.run(cmd, capture_output=True, text=True)
        noise = "is not a recognized feature for this target"
        err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
        if res.returncode != 0:
            raise RuntimeError(f"hipcc failed on {name}:\n{err}")
        if verbose and err.strip():
            print(err, file=sys.stderr)
        return obj

    with ThreadPoolExecutor(max_workers=len(SOURCES)) as pool:
        objs = list(pool.map(compile_one, SOURCES))
    tmp = LIB.with_suffix(f".tmp{os.getpid()}.so")
    res = subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", str(tmp),
                          *map(str, objs)], capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"link failed:\n{res.stderr}")
    os.replace(tmp, LIB)
    build_call_cost(hipcc)
    build_ceilings(hipcc)
    return LIB


CALL_COST = PKG / "ragged_call_cost"


def build_call_cost(hipcc: str) -> Path:
    """The small C++ program that times the C ABI without Python in the loop (native/call_cost.cpp)."""
    res = subprocess.run([hipcc, "--offload-arch=gfx950", "-O2", "-std=c++17", f"-I{ROOT / 'include'}",
                          "-o", str(CALL_COST), str(PKG / "native" / "call_cost.cpp"), f"-L{PKG}", "-lragged_hip",
                          "-Wl,-rpath,$ORIGIN"], capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"building ragged_call_cost failed:\n{res.stderr}")
    return CALL_COST


CEILINGS = PKG / "libragged_ceilings.so"


def build_ceilings(hipcc: str) -> Path:
    """The benchmark's own ceiling kernels (native/ceilings.hip: streaming read / copy, MFMA loop); not part
    of the C ABI, so they live in a shared library of their own."""
    tmp = CEILINGS.with_suffix(f".tmp{os.getpid()}.so")
    res = subprocess.run([hipcc, *HIPCC_FLAGS, "-shared", "-o", str(tmp), str(PKG / "native" / "ceilings.hip")],
                         capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"building libragged_ceilings.so failed:\n{res.stderr}")
    os.replace(tmp, CEILINGS)
    return CEILINGS


if __name__ == "__main__":
    print(build(verbose=True))
