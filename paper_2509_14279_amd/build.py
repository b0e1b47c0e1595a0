"""Builds libfdl.so (the C-ABI library) for gfx950 with hipcc, in-tree.

    python -m paper_2509_14279_amd.build

Each .hip file under csrc/ is compiled to an object file in parallel and the
objects are linked into paper_2509_14279_amd/libfdl.so.  The micro-benchmarks that
measure the machine's ceilings for the roofline report (csrc_ceilings/) go into
a shared object of their own, libfdl_ceilings.so, which only bench.py loads.
"""
from __future__ import annotations

import concurrent.futures
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libfdl.so")
CEIL_SRC = os.path.join(HERE, "csrc_ceilings", "ceilings.hip")
CEIL_LIB = os.path.join(HERE, "libfdl_ceilings.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # only the extern "C" entry points marked in include/fdl.h are exported
    "-fvisibility=hidden",
    # the normal-distribution table of the row kernels is evaluated by the compiler (common.hip.h)
    "-fconstexpr-steps=200000000",
    # keep the compiler from forming packed-fp32 VALU instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument", "-Wno-inline-asm",
]


def sources():
    return sorted(f for f in os.listdir(CSRC) if f.endswith(".hip"))


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, src.replace(".hip", ".o"))
    extra = os.environ.get("FDL_HIPCC_FLAGS", "").split()   # e.g. -DFDL_B4_BK=32 to try another pipeline shape
    cmd = [HIPCC, *FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(verbose: bool = True) -> str:
    os.makedirs(OBJ, exist_ok=True)
    srcs = sources()
    with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, len(srcs))) as ex:
        objs = list(ex.map(_compile, srcs))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    if verbose:
        print(f"built {LIB} from {len(srcs)} sources")
    cmd = [HIPCC, *FLAGS, "-shared", CEIL_SRC, "-o", CEIL_LIB]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for the ceilings micro-benchmarks:\n" + r.stderr)
    if verbose:
        print(f"built {CEIL_LIB}")
    return LIB


if __name__ == "__main__":
    build()
