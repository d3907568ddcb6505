"""Compile the HIP sources under ``csrc/`` into ``libdmr_qlinear.so`` for gfx950 (in-tree)."""
from __future__ import annotations

import glob
import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB = os.path.join(_HERE, "libdmr_qlinear.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # keep the compiler from forming packed-fp32 VALU instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]
OBJ_DIR = os.path.join(_HERE, "_build")
NOISE = "is not a recognized feature for this target"


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def _run(cmd):
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    log = "\n".join(l for l in res.stdout.splitlines() if NOISE not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + " ".join(cmd) + "\n" + log)
    return log


def build_library(verbose: bool = False, jobs: int = 8) -> str:
    """Always recompiles (one object per source, in parallel, then one link): callers that only need the
    library use ``ensure_library``."""
    from concurrent.futures import ThreadPoolExecutor

    os.makedirs(OBJ_DIR, exist_ok=True)
    srcs = sources()
    objs = [os.path.join(OBJ_DIR, os.path.basename(src)[:-4] + ".o") for src in srcs]
    with ThreadPoolExecutor(max_workers=jobs) as pool:
        logs = list(pool.map(lambda so: _run(["hipcc"] + HIPCC_FLAGS + ["-c", so[0], "-o", so[1]]), zip(srcs, objs)))
    logs.append(_run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", LIB]))
    log = "\n".join(l for l in logs if l.strip())
    if verbose and log.strip():
        print(log)
    return LIB


def ensure_library() -> str:
    if not os.path.exists(LIB):
        build_library()
    return LIB
