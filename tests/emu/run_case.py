"""Runs ONE SpMM case through the host-emulated library and compares it with the CPU oracle.
Called as a subprocess by tests/test_emulated_kernels.py (a kernel that reads or writes outside
its buffers ends this process with a segmentation fault, a barrier that not every wave reaches
ends it with the emulator's deadlock report): prints one JSON line.
usage: python run_case.py N K M sparsity out_type postop token_tile variant ldx ldo cus [weight kind [xtiled]]"""
import ctypes
import json
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
sys.path.insert(0, ROOT)
sys.path.insert(0, HERE)


def main():
    N, K, M = int(sys.argv[1]), int(sys.argv[2]), int(sys.argv[3])
    sparsity, ot, po = float(sys.argv[4]), sys.argv[5], sys.argv[6]
    tm, var, ldx, ldo, cus = (int(v) for v in sys.argv[7:12])
    kind = sys.argv[12] if len(sys.argv) > 12 else "uniform"
    x_tiled = len(sys.argv) > 13 and sys.argv[13] in ("xtiled", "xotiled")
    o_tiled = len(sys.argv) > 13 and sys.argv[13] == "xotiled"
    os.environ["EMU_CUS"] = str(cus)
    import build_emu
    import paper_2306_16601_amd.binding as b
    b.LIB_PATH = build_emu.LIB                      # the host-emulated build instead of the HIP one
    import paper_2306_16601_amd as sp
    import oracle
    import workloads as wl
    L = b.lib()
    L.emu_alloc.restype = ctypes.c_void_p
    L.emu_alloc.argtypes = [ctypes.c_size_t]

    def dev(a):
        a = np.ascontiguousarray(a)
        p = L.emu_alloc(a.nbytes)
        ctypes.memmove(p, a.ctypes.data, a.nbytes)
        return p

    case = wl.Case("emu", N, K, M, sparsity, wl.N4K1, ot, po, keys=(77, N, K, M))
    d = wl.make(case)
    W, X = d["W"].copy(), d["X"]
    if kind == "ragged":
        # step lists of very different lengths: block-rows without any block (empty segments),
        # one dense row tile, one row tile that only has blocks in the last K segment
        W[: min(N, 64)] = 0
        if N > 96:
            W[80:96] = wl.rng_for(5, N, K).integers(1, 127, size=(16, K), dtype=np.int8)
        if N > 128:
            W[112:128, : max(0, K - 500)] = 0
    ldx = ldx or M
    ldo = ldo or M
    Xp = np.full((K, ldx), 0xEE, dtype=np.uint8)
    Xp[:, :M] = X
    h = sp.spmm_pack(W, case.orientation)
    sp.spmm_set_tuning(h, tm, var)
    lut = None
    if po == "gelu" and ot in ("s8", "u8"):
        lut = dev(sp.spmm_make_gelu_lut(d["mid_scale"], d["out_scale"], d["out_zero_point"], ot))
    ep = sp.make_epilogue(dev(d["w_scale"]), d["x_scale"], d["x_zero_point"], dev(d["bias"]), po, ot,
                          d["out_scale"], d["out_zero_point"], d["mid_scale"], lut)
    dt = {"s32": np.int32, "f32": np.float32, "s8": np.int8, "u8": np.uint8}[ot]
    tiles = (M + 31) // 32
    nbytes = tiles * N * 32 if o_tiled else N * ldo * np.dtype(dt).itemsize
    od = L.emu_alloc(nbytes)
    ctypes.memset(od, 0x5A, nbytes)
    if x_tiled:
        # token-tile-major activations in an allocation of exactly their size (guard pages behind it);
        # the padding of the last tile is poisoned
        Xt = sp.tile_major(X)
        Xt[-1, :, M - 32 * (Xt.shape[0] - 1):] = 0xEE
        sp.spmm_run_tiled(h, dev(Xt), M, 0, ep, od, ldo, 3 if o_tiled else 1, None)
    else:
        sp.spmm_run(h, dev(Xp), M, ldx, ep, od, ldo, None)
    if o_tiled:
        raw = np.empty(nbytes, dtype=dt)
        ctypes.memmove(raw.ctypes.data, od, nbytes)
        T = raw.reshape(tiles, N, 32)
        full = np.full((N, tiles * 32 + 1), 0x5A, dtype=dt)      # (one extra column: the padding check below)
        full[:, :tiles * 32] = T.transpose(1, 0, 2).reshape(N, tiles * 32)
    else:
        full = np.empty((N, ldo), dtype=dt)
        ctypes.memmove(full.ctypes.data, od, nbytes)
    got = full[:, :M]
    ref = oracle.spmm(W, X, d["w_scale"], d["x_scale"], d["bias"], po, ot, d["out_scale"], d["out_zero_point"],
                      d["mid_scale"], d["x_zero_point"])
    if ot == "f32" and po == "gelu":
        err = np.abs(got.astype(np.float64) - ref.astype(np.float64))
        ok = bool((err <= 1e-4 * np.abs(ref.astype(np.float64)) + 1e-6).all())   # (host exp2 / reciprocal stand-ins)
    elif ot == "f32":
        ok = bool(np.array_equal(got.view(np.uint32), ref.view(np.uint32)))
    else:
        ok = bool(np.array_equal(got, ref))
    pad_ok = bool((full[:, M:].view(np.uint8) == 0x5A).all())
    print(json.dumps({"match": ok, "padding_untouched": pad_ok, "kernel": sp.spmm_kernel_variant(h, M, ot, po),
                      "mismatches": int((got != ref).sum())}))


main()
