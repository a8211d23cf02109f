"""Builds libhmmscan.so (the C-ABI HIP library) in-tree for gfx950 with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ_DIR = os.path.join(HERE, "_build")
LIB_PATH = os.path.join(HERE, "libhmmscan.so")

# (source, extra defines, object name)
UNITS = [("api.hip", [], "api.o"), ("ktimer.hip", [], "ktimer.o"), ("small_d.hip", [], "small_d.o"),
         ("large_d_sp.hip", [], "large_d_sp.o"),
         ("large_d_mp.hip", [], "large_d_mp.o"), ("estep.hip", [], "estep.o"), ("blocks.hip", [], "blocks.o"),
         ("static_scratch.hip", [], "static_scratch.o")] + \
        [("small_d_kernels.hip", ["-DHMM_SMALL_D=%d" % d], "small_d_kernels_%d.o" % d) for d in range(1, 9)]

# A second, small library for the tests: the same code with D = 4 only and tiles half as long (8 steps per lane
# instead of 16), so that results can be shown not to depend on where the tile boundaries fall.
VARIANT_LIB_PATH = os.path.join(HERE, "libhmmscan_tile8.so")
VARIANT_UNITS = [("small_d_kernels.hip", ["-DHMM_SMALL_D=4", "-DHMM_ONLY_SMALL_D=4", "-DHMM_TILE_STEPS_PER_LANE=8"],
                  "small_d_kernels_4_tile8.o"),
                 ("small_d.hip", ["-DHMM_ONLY_SMALL_D=4"], "small_d_only4.o")]
VARIANT_SHARED = ["api.o", "ktimer.o", "large_d_sp.o", "large_d_mp.o", "estep.o", "blocks.o", "static_scratch.o"]

HIPCC_FLAGS = [
    "-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC",
    # packed-FP32 instructions are kept out of the generated code on purpose
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    return "hipcc"


def _compile(unit) -> str:
    src, defines, objname = unit
    obj = os.path.join(OBJ_DIR, objname)
    cmd = [_hipcc(), *HIPCC_FLAGS, *defines, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        sys.stderr.write(r.stdout + r.stderr)
        raise RuntimeError("hipcc failed on " + " ".join([src] + defines))
    return obj


def build_library(verbose: bool = True) -> str:
    os.makedirs(OBJ_DIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as ex:
        all_objs = list(ex.map(_compile, UNITS + VARIANT_UNITS))
    objs, variant_objs = all_objs[:len(UNITS)], all_objs[len(UNITS):]
    variant_objs += [os.path.join(OBJ_DIR, o) for o in VARIANT_SHARED]
    for path, members in ((LIB_PATH, objs), (VARIANT_LIB_PATH, variant_objs)):
        tmp = path + ".tmp.%d" % os.getpid()
        r = subprocess.run([_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *members],
                           capture_output=True, text=True)
        if r.returncode != 0:
            sys.stderr.write(r.stdout + r.stderr)
            raise RuntimeError("link failed")
        os.replace(tmp, path)
        if verbose:
            print("built", path)
    return LIB_PATH


if __name__ == "__main__":
    build_library()
