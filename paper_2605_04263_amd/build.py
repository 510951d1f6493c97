"""Compiles the HIP library for gfx950 in-tree (paper_2605_04263_amd/libpv.so).

Every source under csrc/ is one translation unit, except pv_attn_bf16_inst.hip, which is compiled
once per (head size, GQA group size): the main attention kernel has three dozen instantiations
and they build in parallel this way.  Objects go to paper_2605_04263_amd/_build/.
"""
from __future__ import annotations

import glob
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
OUT = os.path.join(HERE, "libpv.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC",
         # packed fp32 VALU ops are kept off on purpose for every kernel of this library
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I" + os.path.join(ROOT, "include"), "-I" + CSRC]
INST_SOURCE = "pv_attn_bf16_inst.hip"
INST_UNITS = [(d, s) for d in (128, 64) for s in range(1, 10)]      # group sizes 1..8, 9 = query tiles


def _inputs():
    return (glob.glob(os.path.join(CSRC, "*.hip")) + glob.glob(os.path.join(CSRC, "*.h")) +
            [os.path.join(ROOT, "include", "pv.h")])


def library_is_stale() -> bool:
    """True when libpv.so is missing or older than any of its sources."""
    if not os.path.exists(OUT):
        return True
    built = os.path.getmtime(OUT)
    return any(os.path.getmtime(f) > built for f in _inputs())


def _units():
    """(source, object, extra flags) of every translation unit."""
    units = []
    for d, s in INST_UNITS:
        units.append((os.path.join(CSRC, INST_SOURCE), os.path.join(OBJ, f"pv_attn_bf16_inst_d{d}_s{s}.o"),
                      [f"-DPV_INST_D={d}", f"-DPV_INST_SET={s}"]))
    for src in sorted(glob.glob(os.path.join(CSRC, "*.hip"))):
        if os.path.basename(src) != INST_SOURCE:
            units.append((src, os.path.join(OBJ, os.path.basename(src)[:-4] + ".o"), []))
    return units


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    return err


def build_library(verbose: bool = True, extra_flags=(), jobs: int | None = None,
                  incremental: bool = False) -> str:
    """Compiles every translation unit (in parallel) and links libpv.so.  `incremental` skips units
    whose object is newer than every source and header (a convenience while developing; the default
    compiles everything)."""
    os.makedirs(OBJ, exist_ok=True)
    newest = max(os.path.getmtime(f) for f in _inputs())
    todo = [u for u in _units()
            if not (incremental and os.path.exists(u[1]) and os.path.getmtime(u[1]) > newest)]
    jobs = jobs or min(len(todo) or 1, int(os.environ.get("MAX_JOBS", os.cpu_count() or 4)), 16)

    def compile_unit(u):
        src, obj, defs = u
        return _run([HIPCC, *FLAGS, *extra_flags, *defs, "-c", src, "-o", obj], verbose)

    with ThreadPoolExecutor(max_workers=jobs) as pool:
        warnings = [w for w in pool.map(compile_unit, todo) if w.strip()]
    warnings.append(_run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC",
                          *[u[1] for u in _units()], "-o", OUT], verbose))
    if verbose:
        for w in warnings:
            if w.strip():
                print(w, file=sys.stderr)
    return OUT


if __name__ == "__main__":
    build_library(incremental="--incremental" in sys.argv)
