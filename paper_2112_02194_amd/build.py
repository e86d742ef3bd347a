"""Compile libals.so for gfx950 with hipcc (cross-compiles without a GPU).

Every translation unit is compiled on its own (in parallel) and the objects are linked into one
shared library.  Some sources are compiled several times with a different -D each: one object per
row class, so that the long unrolled solver kernels build side by side.
"""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
LIB = os.path.join(HERE, "libals.so")
OBJDIR = os.path.join(HERE, "_build")

# matrix-core results go to ordinary vector registers in these units: their kernels take the results apart with
# vector instructions right away, and a copy out of the accumulation registers per result register costs more
# than the registers do
VGPR_FORM = ["-mllvm", "-amdgpu-mfma-vgpr-form"]

# (source, object name, extra flags)
UNITS = [
    ("als_api.hip", "als_api", []),
    ("gramian.hip", "gramian", []),
    ("rows_primal.hip", "rows_primal", []),
    ("solve_rows.hip", "solve_rows", []),
    ("loss.hip", "loss", []),
    ("topk.hip", "topk", VGPR_FORM),
    ("cg_free.hip", "cg_free", []),
    ("dual_prepare.hip", "dual_prepare", []),
    ("dual_rows.hip", "dual_rows", VGPR_FORM),
    ("dual_small.hip", "dual_small_g8", ["-DSMALL_G=8"] + VGPR_FORM),
    ("dual_small.hip", "dual_small_g4", ["-DSMALL_G=4"] + VGPR_FORM),
    ("dual_multi.hip", "dual_multi", VGPR_FORM),
    ("dual_wide.hip", "dual_wide_3", ["-DWIDE_KT=3"] + VGPR_FORM),
    ("dual_wide.hip", "dual_wide_4", ["-DWIDE_KT=4"] + VGPR_FORM),
    ("dual_wide.hip", "dual_wide_5", ["-DWIDE_KT=5"] + VGPR_FORM),
    ("dual_wide.hip", "dual_wide_6", ["-DWIDE_KT=6"] + VGPR_FORM),
    ("dual_wide.hip", "dual_wide_7", ["-DWIDE_KT=7"] + VGPR_FORM),
    ("dual_wide.hip", "dual_wide_8", ["-DWIDE_KT=8"] + VGPR_FORM),
]

FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-I" + INCLUDE, "-I" + CSRC,
         # packed fp32 instructions are kept out of the generated code on purpose
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _run(cmd):
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "is not a recognized feature for this target" not in l)
    if res.returncode != 0:
        raise RuntimeError("command failed: " + " ".join(cmd) + "\n" + out)
    return out


def build_library(verbose: bool = False, jobs: int = 8) -> str:
    os.makedirs(OBJDIR, exist_ok=True)

    def compile_unit(unit):
        src, name, defs = unit
        obj = os.path.join(OBJDIR, name + ".o")
        return obj, _run(["hipcc"] + FLAGS + defs + ["-c", os.path.join(CSRC, src), "-o", obj])

    with ThreadPoolExecutor(max_workers=jobs) as pool:
        results = list(pool.map(compile_unit, UNITS))
    objs = [o for o, _ in results]
    out = _run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs)
    if verbose:
        for _, log in results:
            if log.strip():
                print(log)
        if out.strip():
            print(out)
    return LIB
