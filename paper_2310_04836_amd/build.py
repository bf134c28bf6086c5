"""Builds libdgq.so (hand-written HIP for gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OBJ = os.environ.get("DGQ_BUILD_DIR") or os.path.join(PKG, "_build")
# DGQ_LIBRARY: load (and build into) another file than the in-tree library
LIB = os.environ.get("DGQ_LIBRARY") or os.path.join(PKG, "libdgq.so")

SOURCES = ["api.hip", "quant_act.hip", "weights.hip", "quantize_grid.hip", "smooth.hip", "linear_decode.hip", "linear_stream.hip", "linear_tiled.hip", "bmm.hip", "probe.hip"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = os.environ.get("DGQ_EXTRA_FLAGS", "").split() + [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
    "-ffp-contract=off", "-fhip-fp32-correctly-rounded-divide-sqrt", "-fno-fast-math",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument", "-Wno-inline-asm",
    "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
]


def _newest_dep() -> float:
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC)] + [os.path.join(ROOT, "include", "dgq.h")]
    return max(os.path.getmtime(d) for d in deps)


def is_built() -> bool:
    return os.path.exists(LIB)


def is_stale() -> bool:
    return (not is_built()) or os.path.getmtime(LIB) < _newest_dep()


def build(verbose: bool = False, save_temps: bool = False) -> str:
    """Compile every source and link libdgq.so.  Always recompiles."""
    os.makedirs(OBJ, exist_ok=True)

    def compile_one(src: str) -> str:
        obj = os.path.join(OBJ, src.replace(".hip", ".o"))
        cmd = [HIPCC, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
        if save_temps:
            cmd.insert(1, "-save-temps=obj")
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.check_call(cmd, cwd=OBJ)
        return obj

    with ThreadPoolExecutor(max_workers=min(len(SOURCES), 8)) as ex:
        objs = list(ex.map(compile_one, SOURCES))
    tmp = LIB + ".tmp.%d" % os.getpid()
    # export only the extern "C" entry points marked default-visible
    subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs])
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    build(verbose=True, save_temps="--save-temps" in sys.argv)
    print(LIB)
