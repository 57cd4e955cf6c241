"""The HIP kernels themselves, run on the CPU.

tests/emu compiles the library's own sources for the host against a stand-in for the HIP
runtime (fibers for threads, exchange for the cross-lane instructions, guard pages around every
device buffer) and each case below runs one kernel family through the C ABI that way, in a
subprocess, against the CPU oracle.  What this checks without a GPU:
  * every global access of the kernel stays inside its buffers (an access outside is a
    segmentation fault of the subprocess, reported with the faulting block and thread);
  * every barrier is reached by every wave of its workgroup (the streamed kernel's segment
    crossings sit at wave-dependent points: each wave must run exactly nseg - 1 of them; a wave
    that runs more or fewer leaves the others waiting, which the emulator reports as a deadlock);
  * the integer results equal the oracle's bit for bit (the emulated matrix instruction and
    transposing read follow the lane layout the kernels document).
The timing-dependent side of the device (scheduling, LDS banking) is of course not modelled.
"""
import json
import os
import subprocess
import sys

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.join(HERE, "emu"))
import build_emu  # noqa: E402

pytestmark = pytest.mark.skipif(not build_emu.available(), reason="no host clang++ for the emulation build")


@pytest.fixture(scope="module")
def emu_lib():
    return build_emu.build()


def run_case(N, K, M, sparsity, out_type, postop, tm, variant, ldx=0, ldo=0, cus=4, kind="uniform", xtiled=False):
    # xtiled: True = tile-major activations, "out" = tile-major activations and tile-major 1-byte output
    cmd = [sys.executable, os.path.join(HERE, "emu", "run_case.py"), str(N), str(K), str(M), str(sparsity), out_type,
           postop, str(tm), str(variant), str(ldx), str(ldo), str(cus), kind] + (["xotiled"] if xtiled == "out" else ["xtiled"] if xtiled else [])
    r = subprocess.run(cmd, capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, "emulated kernel run failed (rc %d):\n%s" % (r.returncode, r.stderr[-3000:])
    return json.loads(r.stdout.strip().splitlines()[-1])


# (N, K, M, sparsity, out, postop, token tile, variant, expected kernel family, extra)
CASES = [
    # pipelined kernel, 16 and 8 waves, both tile widths, several tiles per stream, both K segments
    (512, 1024, 768, 0.9, "s8", "gelu", 128, 16, "spmm_rowtile_mfma<128, 16", {}),
    (512, 1024, 768, 0.9, "s32", "none", 96, 16, "spmm_rowtile_mfma<96, 16", {}),
    (256, 768, 512, 0.8, "f32", "none", 128, 8, "spmm_rowtile_mfma<128, 8", {}),
    (256, 2048, 384, 0.9, "u8", "gelu", 128, 16, "spmm_rowtile_mfma<128, 16", {}),            # weights reloaded per phase
    (300, 1000, 333, 0.85, "s8", "none", 128, 0, "spmm_rowtile_mfma<", {"cus": 2}),            # ragged everything
    (128, 512, 200, 0.7, "s8", "gelu", 128, 8, "spmm_rowtile_mfma<128, 8", {"ldx": 211, "ldo": 203}),   # unaligned pitches
    # pipelined kernel with loader waves: 12 + 4 and 8 + 4 waves, both tile widths, weights reloaded, ragged, unaligned
    (400, 1024, 384, 0.9, "f32", "none", 128, 112, "spmm_rowtile_mfma_fed<128, 12", {"cus": 2}),
    (272, 1536, 300, 0.8, "s32", "none", 128, 108, "spmm_rowtile_mfma_fed<128, 8", {"cus": 2}),
    (400, 600, 333, 0.9, "s8", "gelu", 96, 112, "spmm_rowtile_mfma_fed<96, 12", {"cus": 2}),
    (272, 700, 250, 0.8, "f32", "gelu", 128, 112, "spmm_rowtile_mfma_fed<128, 8", {"cus": 2, "ldx": 251, "ldo": 253, "kind": "ragged"}),
    (272, 700, 250, 0.8, "s8", "gelu", 64, 112, "spmm_rowtile_mfma_fed<128, 8", {"cus": 2, "kind": "ragged"}),   # dense tile: falls back to 8 + 4
    (200, 600, 203, 0.9, "u8", "none", 64, 112, "spmm_rowtile_mfma_fed<64, 12", {"cus": 2, "ldx": 211, "ldo": 209}),
    # token-tile-major activations ([M / 32][K][32], exactly sized allocation): one case per kernel family
    (300, 1000, 333, 0.85, "s8", "gelu", 96, 16, "spmm_rowtile_mfma<96, 16", {"cus": 2, "xtiled": True}),
    (256, 1536, 200, 0.9, "s32", "none", 128, 112, "spmm_rowtile_mfma_fed<128, 12", {"cus": 2, "xtiled": True}),
    (128, 700, 150, 0.8, "s8", "none", 64, 101, "spmm_rowtile_mfma_simple<64", {"xtiled": True}),
    (128, 2560, 40, 0.9, "s32", "none", 16, 103, "spmm_rowtile_mfma_slab<16", {"xtiled": True}),
    (128, 3584, 70, 0.9, "s8", "gelu", 32, 104, "spmm_rowtile_mfma_stream<32", {"xtiled": True}),
    (300, 1000, 333, 0.85, "s8", "gelu", 128, 16, "spmm_rowtile_mfma<128, 16", {"cus": 2, "xtiled": "out"}),
    (272, 1536, 200, 0.9, "u8", "none", 96, 112, "spmm_rowtile_mfma_fed<96, 12", {"cus": 2, "xtiled": "out"}),
    (128, 700, 150, 0.8, "s8", "none", 32, 101, "spmm_rowtile_mfma_simple<32", {"xtiled": "out"}),
    # simple kernel at its three tile widths
    (256, 1024, 192, 0.9, "s8", "gelu", 64, 101, "spmm_rowtile_mfma_simple<64", {}),
    (512, 768, 128, 0.8, "s32", "none", 64, 102, "spmm_rowtile_mfma_simple<64", {}),
    (256, 1536, 96, 0.9, "f32", "none", 32, 101, "spmm_rowtile_mfma_simple<32", {}),
    (128, 1024, 50, 0.9, "s8", "none", 16, 101, "spmm_rowtile_mfma_simple<16", {"ldx": 50, "ldo": 50}),
    # short-batch kernel (whole K slab in LDS)
    (256, 3072, 48, 0.9, "s8", "gelu", 16, 103, "spmm_rowtile_mfma_slab<16", {}),
    (128, 2560, 64, 0.8, "s32", "none", 32, 103, "spmm_rowtile_mfma_slab<32", {}),
    # streamed kernel: uniform and very uneven step lists (empty segments, a dense tile, a late tile)
    (256, 4096, 128, 0.9, "s8", "gelu", 64, 104, "spmm_rowtile_mfma_stream<64", {}),
    (256, 3584, 64, 0.9, "s32", "none", 32, 104, "spmm_rowtile_mfma_stream<32", {"kind": "ragged"}),
    (192, 4096, 40, 0.8, "s8", "none", 16, 104, "spmm_rowtile_mfma_stream<16", {"kind": "ragged"}),
    (144, 5000, 70, 0.95, "s32", "none", 64, 104, "spmm_rowtile_mfma_stream<64", {"kind": "ragged"}),
]


@pytest.mark.parametrize("case", CASES, ids=lambda c: "%dx%d_m%d_%s_%s_tm%d_v%d" % (c[0], c[1], c[2], c[4], c[5], c[6], c[7]))
def test_kernel_on_the_cpu_matches_oracle_and_stays_in_bounds(emu_lib, case):
    N, K, M, s, ot, po, tm, var, family, extra = case
    res = run_case(N, K, M, s, ot, po, tm, var, **extra)
    assert family in res["kernel"], res["kernel"]
    assert res["match"], "%d outputs differ from the oracle" % res["mismatches"]
    assert res["padding_untouched"]


def test_a_missing_barrier_would_be_reported():
    """The deadlock report itself: a tiny program in which one wave skips a barrier."""
    src = r'''
#include <hip/hip_runtime.h>
static void kernel() { if (threadIdx.x < 64) __syncthreads(); }
int main() { hipLaunchKernelGGL((kernel), dim3(1), dim3(128), 0, nullptr); return 0; }
'''
    build_emu.build()
    work = os.path.join(build_emu.OUT, "selftest")
    os.makedirs(work, exist_ok=True)
    open(os.path.join(work, "t.cpp"), "w").write(src)
    exe = os.path.join(work, "t")
    subprocess.run([build_emu.CXX, "-std=c++17", "-O1", "-w", "-I", os.path.join(HERE, "emu", "include"), os.path.join(work, "t.cpp"),
                    os.path.join(HERE, "emu", "emu.cpp"), "-lpthread", "-o", exe], check=True)
    r = subprocess.run([exe], capture_output=True, text=True, timeout=60)
    assert r.returncode == 86 and "DEADLOCK" in r.stderr, (r.returncode, r.stderr[-500:])
