"""Compile the HIP sources in csrc/ into paper_2207_05022_amd/libsti.so (gfx950)."""
from __future__ import annotations

import glob
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
OBJ_DIR = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libsti.so")
PROBES_SRC = os.path.join(CSRC, "probes", "ceilings.hip")
PROBES_LIB = os.path.join(HERE, "libsti_probes.so")   # ceiling probes for bench.py --ceilings, not part of libsti
# libsti with the many-token GEMM kernel compiled to record its phase time stamps (bench.py --phase-budget)
PHASES_SRC = os.path.join(CSRC, "gemm_wide.hip")
PHASES_LIB = os.path.join(HERE, "libsti_phases.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
    # keep the compiler from forming packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # leading scalar kernel arguments arrive preloaded in scalar registers (no fetch from the
    # argument buffer in front of a kernel's first loads)
    "-mllvm", "-amdgpu-kernarg-preload-count=16",
    "-I", INCLUDE, "-I", CSRC,
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def _compile(src: str) -> str:
    obj = os.path.join(OBJ_DIR, os.path.basename(src)[:-4] + ".o")
    subprocess.run([HIPCC, *FLAGS, "-c", src, "-o", obj], check=True,
                   stderr=subprocess.PIPE, text=True)
    return obj


def build(verbose: bool = False) -> str:
    os.makedirs(OBJ_DIR, exist_ok=True)
    srcs = sources()
    try:
        with ThreadPoolExecutor(max_workers=min(8, len(srcs))) as pool:
            objs = list(pool.map(_compile, srcs))
        subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs],
                       check=True, stderr=subprocess.PIPE, text=True)
        subprocess.run([HIPCC, *FLAGS, "-shared", PROBES_SRC, "-o", PROBES_LIB],
                       check=True, stderr=subprocess.PIPE, text=True)
        stamped = os.path.join(OBJ_DIR, "gemm_wide_phases.o")
        subprocess.run([HIPCC, *FLAGS, "-DSTI_PHASE_STAMPS", "-c", PHASES_SRC, "-o", stamped],
                       check=True, stderr=subprocess.PIPE, text=True)
        plain = os.path.join(OBJ_DIR, "gemm_wide.o")
        subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", PHASES_LIB,
                        *[stamped if o == plain else o for o in objs]],
                       check=True, stderr=subprocess.PIPE, text=True)
    except subprocess.CalledProcessError as err:
        raise RuntimeError(f"hipcc failed: {' '.join(err.cmd)}\n{err.stderr}") from None
    if verbose:
        print(f"built {LIB} from {len(srcs)} sources, {PROBES_LIB} and {PHASES_LIB}")
    return LIB


if __name__ == "__main__":
    build(verbose=True)
