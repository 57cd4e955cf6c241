"""Build the HIP shared library for gfx950 in-tree (paper_2306_16601_amd/libspmm4x1.so).

The kernel configurations are compiled as separate objects (spmm_launch_cfg.hip once per
configuration) in parallel and linked with the host sources.
"""
from __future__ import annotations

import os
import shutil
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libspmm4x1.so")
OBJDIR = os.path.join(HERE, "_build")

HOST_SOURCES = ["api.cpp", "pack.cpp", "spmm_plan.hip", "spmm_peak.hip"]
# (token tile, waves, step slots) of the pipelined kernel; row tiles per wave of the simple kernel
PIPELINED = [(128, 16, 4), (128, 16, 5), (128, 16, 6), (128, 8, 4), (128, 8, 6), (128, 8, 8),
             (96, 16, 4), (96, 16, 5), (96, 16, 6)]
# (token tile, compute waves, step slots) of the pipelined kernel with 4 loader waves
FED = [(128, 12, 4), (128, 12, 6), (128, 8, 4), (128, 8, 6), (128, 8, 8), (96, 12, 4), (96, 12, 6), (64, 12, 4), (64, 12, 6)]
SIMPLE = [1, 2]
SLAB = [16, 32]            # token tiles of the short-batch kernel
STREAM = [64, 32, 16]      # token tiles of the streamed kernel
SIMPLE_NARROW = [32, 16]   # token tiles of the simple kernel besides 64 (one row tile per wave)
HEADERS = [os.path.join(CSRC, "spmm_internal.h"), os.path.join(CSRC, "spmm_kernels.h"),
           os.path.join(ROOT, "include", "spmm.h")]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-ffp-contract=off",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def units():
    """(object name, source, extra defines) of every translation unit."""
    out = [(os.path.splitext(s)[0] + ".o", os.path.join(CSRC, s), []) for s in HOST_SOURCES]
    cfg = os.path.join(CSRC, "spmm_launch_cfg.hip")
    for tm, nw, maxs in PIPELINED:
        out.append((f"cfg_{tm}_{nw}_{maxs}.o", cfg, [f"-DSPMM_CFG_TM={tm}", f"-DSPMM_CFG_NW={nw}", f"-DSPMM_CFG_MAXS={maxs}"]))
    for tm, nw, maxs in FED:
        out.append((f"cfg_fed_{tm}_{nw}_{maxs}.o", cfg, [f"-DSPMM_CFG_FED_TM={tm}", f"-DSPMM_CFG_NW={nw}", f"-DSPMM_CFG_MAXS={maxs}"]))
    for r in SIMPLE:
        out.append((f"cfg_simple_{r}.o", cfg, [f"-DSPMM_CFG_SIMPLE={r}"]))
    for tm in SIMPLE_NARROW:
        out.append((f"cfg_simple{tm}_1.o", cfg, ["-DSPMM_CFG_SIMPLE=1", f"-DSPMM_CFG_SIMPLE_TM={tm}"]))
    for tm in SLAB:
        out.append((f"cfg_slab{tm}.o", cfg, [f"-DSPMM_CFG_SLAB={tm}"]))
    for tm in STREAM:
        out.append((f"cfg_stream{tm}.o", cfg, [f"-DSPMM_CFG_STREAM={tm}"]))
    return out


def sources():
    return sorted({u[1] for u in units()})


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed: " + " ".join(cmd) + "\n" + err)
    if verbose and err.strip():
        print(err)


def build(force: bool = True, verbose: bool = False, jobs: int | None = None) -> str:
    """Compile every source with hipcc (cross-compiles without a GPU) and link the library."""
    deps = sources() + HEADERS
    if not force and os.path.exists(LIB) and all(os.path.getmtime(LIB) >= os.path.getmtime(d) for d in deps):
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if jobs is None:
        jobs = max(1, min(8, os.cpu_count() or 1))
    objdir = OBJDIR + ".%d" % os.getpid()
    os.makedirs(objdir, exist_ok=True)
    try:
        us = units()
        # the heaviest objects (pipelined kernels) first
        us.sort(key=lambda u: 0 if u[0].startswith("cfg_1") or u[0].startswith("cfg_9") or u[0].startswith("cfg_fed") else 1)
        cmds = [[hipcc, *HIPCC_FLAGS, *defs, "-x", "hip", "-c", src, "-o", os.path.join(objdir, obj)]
                for obj, src, defs in us]
        with ThreadPoolExecutor(max_workers=jobs) as pool:
            list(pool.map(lambda c: _run(c, verbose), cmds))
        tmp = LIB + ".tmp.%d" % os.getpid()
        _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *[os.path.join(objdir, u[0]) for u in us], "-o", tmp],
             verbose)
        os.replace(tmp, LIB)
    finally:
        shutil.rmtree(objdir, ignore_errors=True)
    return LIB


if __name__ == "__main__":
    print(build(force=True, verbose=True))
