"""Builds ``libmfreduce.so`` for gfx950 with hipcc (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
import sys

_HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(_HERE)
CSRC = os.path.join(_HERE, "csrc")
SOURCES = [os.path.join(CSRC, f) for f in ("mfreduce.hip", "launch_f16.hip", "launch_bf16.hip", "launch_f32.hip", "recurrence.hip", "launch_wide.hip", "rows_tiled_f16.hip", "rows_tiled_bf16.hip", "rows_tiled_f32.hip")]
BUILD_DIR = os.path.join(_HERE, "_build")
INCLUDE = os.path.join(ROOT, "include")
LIB_PATH = os.path.join(_HERE, "libmfreduce.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Wall", "-Wextra",
    # no packed-fp32 VALU forms
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def _compile(src: str, obj: str, verbose: bool, extra_flags) -> None:
    cmd = [hipcc(), *HIPCC_FLAGS, *extra_flags, "-I", INCLUDE, "-I", CSRC, "-c", src, "-o", obj]
    if verbose:
        print(" ".join(cmd), file=sys.stderr)
    subprocess.run(cmd, check=True)


def build(verbose: bool = False, extra_flags=()) -> str:
    """Compile every translation unit (in parallel) and link libmfreduce.so."""
    from concurrent.futures import ThreadPoolExecutor
    os.makedirs(BUILD_DIR, exist_ok=True)
    objs = [os.path.join(BUILD_DIR, os.path.basename(s)[:-4] + ".o") for s in SOURCES]
    with ThreadPoolExecutor(max_workers=min(len(SOURCES), os.cpu_count() or 1)) as ex:
        list(ex.map(lambda so: _compile(so[0], so[1], verbose, extra_flags), zip(SOURCES, objs)))
    tmp = LIB_PATH + ".tmp%d" % os.getpid()
    cmd = [hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs]
    if verbose:
        print(" ".join(cmd), file=sys.stderr)
    subprocess.run(cmd, check=True)
    os.replace(tmp, LIB_PATH)
    return LIB_PATH


CONTEXT_SOURCE = os.path.join(CSRC, "context_hipcub.hip")
CONTEXT_LIB_PATH = os.path.join(_HERE, "libmfrcontext.so")


def build_context(verbose: bool = False) -> str:
    """The hipCUB comparison reduction (benchmark context only; the library never links it)."""
    tmp = CONTEXT_LIB_PATH + ".tmp%d" % os.getpid()
    cmd = [hipcc(), *HIPCC_FLAGS, "-shared", "-o", tmp, CONTEXT_SOURCE]
    if verbose:
        print(" ".join(cmd), file=sys.stderr)
    subprocess.run(cmd, check=True)
    os.replace(tmp, CONTEXT_LIB_PATH)
    return CONTEXT_LIB_PATH


if __name__ == "__main__":
    print(build(verbose=True))
    print(build_context(verbose=True))
