"""Build step of the HIP library: hipcc, gfx950 only, output in-tree.

    python -m paper_2510_23498_amd.build

The packed-fp32 target feature is switched off for all device code (the compiler
would otherwise form packed fp32 instructions from ordinary float arithmetic).
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_PATH = os.path.join(PKG_DIR, "librampde.so")


def hipcc_path() -> str:
    cand = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(cand):
        raise RuntimeError("hipcc not found (expected on PATH or at /opt/rocm/bin/hipcc)")
    return cand


FUSED_HIDDEN_WIDTHS = (0, 256, 512, 1024)  # translation units of fused_inst.hip: one per width and precision

COMPILE_FLAGS = ["-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-Wno-pass-failed",
                 "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _compile(args):
    src, obj, defs = args
    cmd = [hipcc_path()] + COMPILE_FLAGS + defs + ["-c", src, "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    return res.returncode, res.stdout + res.stderr, obj


# headers each translation unit includes (directly or not), for the incremental mode
_DEPS = {
    "rampde.hip": ("common.hpp", "elementwise.hpp", "fused.hpp", "fused_launch.hpp", "wide.hpp", "gemm.hpp", "wgrad_slab.hpp", "gemm_slab.hpp", "conv_wgrad_tr.hpp", "conv.hpp", "norm.hpp",
                   os.path.join("..", "..", "include", "rampde.h")),
    "fused_inst.hip": ("common.hpp", "fused.hpp", "fused_launch.hpp"),
    "wide_inst.hip": ("common.hpp", "fused.hpp", "fused_launch.hpp", "wide.hpp"),
}


def _up_to_date(src: str, obj: str) -> bool:
    if not os.path.exists(obj):
        return False
    t = os.path.getmtime(obj)
    deps = [src, os.path.abspath(__file__)] + [os.path.join(CSRC, d) for d in _DEPS[os.path.basename(src)]]
    return all(os.path.getmtime(d) < t for d in deps)


def build_library(verbose: bool = False, jobs: int = 0, incremental: bool = False) -> str:
    """Compile the translation units under csrc/ in parallel and link librampde.so next to this
    file; returns its path.  incremental: keep objects newer than their sources and headers (a
    developer convenience; the default compiles everything)."""
    from concurrent.futures import ThreadPoolExecutor
    objdir = os.path.join(PKG_DIR, "_build")
    os.makedirs(objdir, exist_ok=True)
    units = [(os.path.join(CSRC, "rampde.hip"), os.path.join(objdir, "rampde.o"), []),
             (os.path.join(CSRC, "wide_inst.hip"), os.path.join(objdir, "wide.o"), [])]
    for hp in FUSED_HIDDEN_WIDTHS:
        for bf16 in (0, 1):
            units.append((os.path.join(CSRC, "fused_inst.hip"), os.path.join(objdir, f"fused_hp{hp}_{bf16}.o"),
                          [f"-DRAMPDE_INST_HP={hp}", f"-DRAMPDE_INST_BF16={bf16}"]))
    # (longest first: the widest instantiations take the longest to compile)
    units.sort(key=lambda u: -int(u[2][0].split("=")[1]) if u[2] else 1)
    jobs = jobs or min(len(units), os.cpu_count() or 1, 16)
    todo = [u for u in units if not (incremental and _up_to_date(u[0], u[1]))]
    with ThreadPoolExecutor(max_workers=jobs) as pool:
        results = list(pool.map(_compile, todo))
    results += [(0, "", u[1]) for u in units if u not in todo]
    for rc, out, obj in results:
        if rc != 0:
            sys.stderr.write(out)
            raise RuntimeError(f"hipcc failed building {obj}")
        if verbose:
            sys.stderr.write(out)
    cmd = [hipcc_path(), "--offload-arch=gfx950", "-shared", "-fPIC"] + [r[2] for r in results] + \
          ["-o", LIB_PATH + ".tmp"]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        sys.stderr.write(res.stdout + res.stderr)
        raise RuntimeError("hipcc failed linking librampde.so")
    os.replace(LIB_PATH + ".tmp", LIB_PATH)
    return LIB_PATH


if __name__ == "__main__":
    print(build_library(verbose="--quiet" not in sys.argv, incremental="--incremental" in sys.argv))
