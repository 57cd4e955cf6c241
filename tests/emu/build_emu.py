"""Builds tests/emu/_build/libspmm4x1_emu.so: the library's own sources compiled for the host
against the emulation shim in include/hip/hip_runtime.h (see there), with two textual changes:
  * the empty inline-assembly statements that pin a value to a vector register become no-ops;
  * where the lanes of a wave exchange data through LDS without a barrier (the transpose of 1-byte
    outputs, which relies on a wave's LDS operations completing in order), the emulated wave is
    brought into step before and after the read, because its lanes run one after the other here.
Test infrastructure only; nothing in the product path imports or loads it."""
from __future__ import annotations

import os
import re
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
OUT = os.path.join(HERE, "_build")
LIB = os.path.join(OUT, "libspmm4x1_emu.so")
CXX = os.environ.get("EMU_CXX", "/opt/rocm/llvm/bin/clang++")


def available() -> bool:
    return os.path.exists(CXX)


def _sources():
    sys.path.insert(0, ROOT)
    from paper_2306_16601_amd import build as B
    return B


def up_to_date() -> bool:
    if not os.path.exists(LIB):
        return False
    B = _sources()
    deps = B.sources() + B.HEADERS + [os.path.join(HERE, "emu.cpp"), os.path.join(HERE, "include", "hip", "hip_runtime.h"),
                                      os.path.abspath(__file__)]
    return all(os.path.getmtime(LIB) >= os.path.getmtime(d) for d in deps)


def build(force: bool = False) -> str:
    if not force and up_to_date():
        return LIB
    B = _sources()
    src = os.path.join(OUT, "src")
    obj = os.path.join(OUT, "obj")
    shutil.rmtree(OUT, ignore_errors=True)
    os.makedirs(src)
    os.makedirs(obj)
    csrc = os.path.join(ROOT, "paper_2306_16601_amd", "csrc")
    for f in os.listdir(csrc):
        s = open(os.path.join(csrc, f)).read()
        s = re.sub(r'asm volatile\(""\s*:\s*"\+v"\((\w+)\)\);', r'(void)\1;', s)
        s = s.replace('const v4i v = *(const v4i*)(lds + raddr);',
                      'emu::wave_barrier(); const v4i v = *(const v4i*)(lds + raddr); emu::wave_barrier();')
        code = re.sub(r'//.*', '', s)
        if re.search(r'\basm\b', code):
            raise RuntimeError("inline assembly in %s that the emulation build does not know" % f)
        open(os.path.join(src, f), "w").write(s)
    flags = ["-std=c++17", "-O1", "-g", "-fPIC", "-ffp-contract=off", "-w",
             "-I", os.path.join(HERE, "include"), "-I", os.path.join(ROOT, "include"), "-I", src, "-x", "c++"]
    cmds, objs = [], []
    for name, path, defs in B.units():
        if os.path.basename(path) == "spmm_peak.hip":
            continue          # instruction-rate measurement: nothing to emulate (stubbed in emu.cpp)
        o = os.path.join(obj, name)
        objs.append(o)
        cmds.append([CXX, *flags, *defs, "-c", os.path.join(src, os.path.basename(path)), "-o", o])
    o = os.path.join(obj, "emu.o")
    objs.append(o)
    cmds.append([CXX, *flags, "-c", os.path.join(HERE, "emu.cpp"), "-o", o])

    def run(c):
        r = subprocess.run(c, capture_output=True, text=True)
        if r.returncode:
            raise RuntimeError("emulation build failed: %s\n%s" % (" ".join(c), r.stderr[-3000:]))

    with ThreadPoolExecutor(max(1, min(8, os.cpu_count() or 1))) as pool:
        list(pool.map(run, cmds))
    run([CXX, "-shared", "-fPIC", *objs, "-lpthread", "-o", LIB])
    shutil.rmtree(obj, ignore_errors=True)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
