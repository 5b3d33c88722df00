"""Builds liblpq.so (the HIP library) in-tree with hipcc for gfx950.

    python -m paper_2110_08919_amd.build [--force] [--ablation]

Each .hip file under csrc/ is compiled to an object (in parallel), then linked into
paper_2110_08919_amd/liblpq.so.  hipcc cross-compiles, so no GPU is needed to build.
--ablation builds a second library, liblpq_ablation.so, with -DLPQ_ABLATION: the timing
experiments of the matrix-core kernel (LPQ_TUNE_DRY_RUN) exist only there; select it for a
measurement with LPQ_LIBRARY=<path>.
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
LIB = os.path.join(HERE, "liblpq.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-unknown-warning-option", "-Wno-unused-command-line-argument",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def sources():
    return sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".hip"))


def _newest_header() -> float:
    hs = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    hs.append(os.path.join(ROOT, "include", "lpq.h"))
    return max(os.path.getmtime(h) for h in hs)


def device_asm(src: str) -> str:
    """Where the compile of a matrix-core kernel file leaves its gfx950 assembly (a by-product kept
    for tests/test_kernel_schedule.py, which checks the instruction order the compiler chose)."""
    return os.path.join(OBJ, os.path.basename(src)[:-4] + "-hip-amdgcn-amd-amdhsa-gfx950.s")


def keeps_asm(src: str) -> bool:
    return os.path.basename(src).startswith("search_mfma")


def _compile(src: str, force: bool, ablation: bool) -> str:
    obj = os.path.join(OBJ, os.path.basename(src)[:-4] + (".abl.o" if ablation else ".o"))
    want_asm = keeps_asm(src) and not ablation
    stale = (force or not os.path.exists(obj)
             or os.path.getmtime(obj) < max(os.path.getmtime(src), _newest_header())
             or (want_asm and not os.path.exists(device_asm(src))))
    if stale:
        extra = ["-DLPQ_ABLATION"] if ablation else []
        if want_asm:
            extra.append("-save-temps=obj")
        subprocess.run([HIPCC, *FLAGS, *extra, "-c", src, "-o", obj], check=True)
        if want_asm:   # of the intermediate files only the device assembly is kept
            stem = os.path.join(OBJ, os.path.basename(src)[:-4])
            for f in os.listdir(OBJ):
                full = os.path.join(OBJ, f)
                if full.startswith(stem + "-h") and full != device_asm(src) or full == stem + ".hip-hip-amdgcn-amd-amdhsa.hipfb":
                    os.remove(full)
    return obj


def build(force: bool = False, jobs: int = 8, ablation: bool = False) -> str:
    os.makedirs(OBJ, exist_ok=True)
    lib = os.path.join(HERE, "liblpq_ablation.so") if ablation else LIB
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(lambda s: _compile(s, force, ablation), sources()))
    if force or not os.path.exists(lib) or any(os.path.getmtime(o) > os.path.getmtime(lib) for o in objs):
        subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *objs], check=True)
    return lib


if __name__ == "__main__":
    print(build(force="--force" in sys.argv, ablation="--ablation" in sys.argv))
