"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer: the packer (pack.cpp) and the
oracle (spmm_oracle.c) are compiled with -fsanitize=address,undefined into one driver
(tests/sanitize/host_paths.cpp) and run over edge shapes.  GPU code is not involved."""
import os
import shutil
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CXX = shutil.which("clang++") or "/opt/rocm/llvm/bin/clang++"
CC = CXX.replace("clang++", "clang")


@pytest.mark.skipif(not os.path.exists(CXX), reason="no clang++ for a sanitizer build")
def test_packer_and_oracle_under_asan_ubsan(tmp_path):
    san = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]
    csrc = os.path.join(ROOT, "paper_2306_16601_amd", "csrc")
    objs = []
    for src, comp, extra in (
            (os.path.join(csrc, "pack.cpp"), CXX, ["-std=c++17"]),
            (os.path.join(HERE, "sanitize", "host_paths.cpp"), CXX, ["-std=c++17"]),
            (os.path.join(ROOT, "oracle", "spmm_oracle.c"), CC, ["-std=c11", "-ffp-contract=off"])):
        o = str(tmp_path / (os.path.basename(src) + ".o"))
        subprocess.run([comp, *san, *extra, "-I", os.path.join(ROOT, "include"), "-I", csrc, "-c", src, "-o", o], check=True)
        objs.append(o)
    exe = str(tmp_path / "host_paths")
    subprocess.run([CXX, *san, *objs, "-lm", "-o", exe], check=True)
    env = dict(os.environ, ASAN_OPTIONS="verify_asan_link_order=0:detect_leaks=1", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=600)
    assert r.returncode == 0 and r.stdout.strip() == "ok", (r.returncode, r.stdout[-500:], r.stderr[-3000:])
