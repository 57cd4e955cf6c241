"""Host logic of the library (no GPU): the C ABI loads and exports what the header
declares, pack/unpack round-trips, block counts match the generator, and the compressed
device layout -- decoded here in numpy exactly as the kernel's lanes read it -- reproduces
the oracle's accumulator."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
import paper_2306_16601_amd as sp
import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "spmm.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(spmm_[a-z_0-9]+)\s*\(", hdr))
    assert {"spmm_pack", "spmm_unpack", "spmm_info", "spmm_run", "spmm_make_gelu_lut",
            "spmm_destroy", "spmm_status_string"} <= declared
    L = ctypes.CDLL(sp.LIB_PATH)
    for name in declared:
        assert hasattr(L, name), name
    assert declared == set(sp.EXPORTS)


def test_status_strings():
    assert sp.spmm_status_string(0) == "ok"
    assert len({sp.spmm_status_string(i) for i in range(5)}) == 5


def decode_layout_acc(handle, X):
    """Replay the device layout on the CPU: per step, 64 list slots, 16 rows; activations
    as (x - 128) with 128 * rowsum added back, exactly what the kernel accumulates."""
    N, K, _, _, _ = sp.spmm_info(handle)
    tile_rows, step_k, kc, n_tiles, n_seg, n_steps = sp.spmm_layout_dims(handle)
    vals, idx, seg_ptr, rowsum = sp.spmm_layout_export(handle)
    assert (tile_rows, step_k) == (16, 64)
    M = X.shape[1]
    Xs = X.astype(np.int64) - 128
    acc = np.zeros((n_tiles * 16, M), dtype=np.int64)
    for tile in range(n_tiles):
        for seg in range(n_seg):
            for s in range(seg_ptr[tile * n_seg + seg], seg_ptr[tile * n_seg + seg + 1]):
                for g in range(4):
                    for t in range(16):
                        e = int(idx[s, 8 * g + (t % 8)])
                        kl = (e & 0xFFFF) if t < 8 else (e >> 16)
                        k = seg * kc + kl
                        w = vals[s, 16 * g:16 * g + 16, t].view(np.int8).astype(np.int64)   # 16 rows
                        if not w.any():
                            assert k < K          # padding must still name a resident row
                            continue
                        assert k < K
                        acc[tile * 16:tile * 16 + 16] += w[:, None] * Xs[k][None, :]
    acc += 128 * rowsum.astype(np.int64)[:, None]
    return acc[:N]


CASES = [
    ("n4k1", 256, 256, 0.9), ("n1k4", 256, 256, 0.9), ("n4k1", 64, 1100, 0.8), ("n4k1", 50, 70, 0.5),
    ("n1k4", 37, 131, 0.7), ("n4k1", 16, 2100, 0.95), ("n4k1", 3, 5, 0.0),
]


@pytest.mark.parametrize("orient,N,K,s", CASES)
def test_roundtrip_counts_and_layout(orient, N, K, s):
    W = wl.sparse_weight(N, K, s, orient, keys=(77, N, K))
    h = sp.spmm_pack_host(W, orient)
    try:
        n, k, nnzb, padded, dev_bytes = sp.spmm_info(h)
        assert (n, k) == (N, K) and dev_bytes == 0
        assert np.array_equal(sp.spmm_unpack(h), W)
        assert nnzb == wl.realised_block_sparsity(W, orient)[0]          # sparsity preserved
        assert padded >= nnzb
        X = wl.activations(K, 24, keys=(77, N, K))
        ref = oracle.acc_s32(W, X).astype(np.int64)
        assert np.array_equal(decode_layout_acc(h, X), ref)
    finally:
        sp.spmm_destroy(h)


def test_layout_structure_tiny():
    W = wl.make(wl.tiny_cases()[0])["W"]
    h = sp.spmm_pack_host(W)
    try:
        tile_rows, step_k, kc, n_tiles, n_seg, n_steps = sp.spmm_layout_dims(h)
        assert (n_tiles, n_seg) == (16, 1)
        vals, idx, seg_ptr, rowsum = sp.spmm_layout_export(h)
        assert seg_ptr[0] == 0 and seg_ptr[-1] == n_steps and np.all(np.diff(seg_ptr) >= 0)
        assert np.array_equal(rowsum, W.astype(np.int32).sum(axis=1))
        # the k list of tile 0 is the union of its four block-rows (any order), zero padded
        union = np.flatnonzero((W[:16] != 0).any(axis=0))
        real, pad_rows = [], []
        for s in range(seg_ptr[0], seg_ptr[1]):
            for g in range(4):
                for t in range(16):
                    e = int(idx[s, 8 * g + (t % 8)])
                    kl = (e & 0xFFFF) if t < 8 else (e >> 16)
                    if vals[s, 16 * g:16 * g + 16, t].any():
                        real.append(kl)
                    else:
                        pad_rows.append(kl)
        assert sorted(real) == union.tolist()
        assert all(0 <= v < 256 for v in pad_rows)
        assert len(real) + len(pad_rows) == 64 * int(np.ceil(len(union) / 64))
    finally:
        sp.spmm_destroy(h)


def test_unstructured_and_extreme_weights_pack_losslessly():
    rng = np.random.default_rng(5)
    W = rng.integers(-128, 128, size=(21, 45), dtype=np.int8)
    W[rng.random(W.shape) < 0.6] = 0
    for orient in ("n4k1", "n1k4"):
        h = sp.spmm_pack_host(W, orient)
        assert np.array_equal(sp.spmm_unpack(h), W)
        X = wl.activations(45, 7, keys=(78,))
        assert np.array_equal(decode_layout_acc(h, X), oracle.acc_s32(W, X).astype(np.int64))
        sp.spmm_destroy(h)
    Z = np.zeros((8, 8), np.int8)
    h = sp.spmm_pack_host(Z)
    assert sp.spmm_info(h)[2] == 0 and sp.spmm_layout_dims(h)[5] == 0
    assert np.array_equal(sp.spmm_unpack(h), Z)
    sp.spmm_destroy(h)


def test_strided_weight_input():
    big = wl.sparse_weight(32, 64, 0.75, keys=(79,))
    W = big[:, :40]                                  # ldw = 64 > K = 40
    h = sp.spmm_pack_host(W)
    assert np.array_equal(sp.spmm_unpack(h), W)
    sp.spmm_destroy(h)


def test_pack_argument_errors():
    L = sp.lib()
    W = np.zeros((4, 4), np.int8)
    h = ctypes.c_void_p()
    p = W.ctypes.data_as(ctypes.c_void_p)
    assert L.spmm_pack_host(None, 4, 4, 4, 0, ctypes.byref(h)) == sp.SPMM_E_ARG
    assert L.spmm_pack_host(p, 4, 4, 4, 0, None) == sp.SPMM_E_ARG
    assert L.spmm_pack_host(p, 0, 4, 4, 0, ctypes.byref(h)) == sp.SPMM_E_ARG
    assert L.spmm_pack_host(p, 4, -1, 4, 0, ctypes.byref(h)) == sp.SPMM_E_ARG
    assert L.spmm_pack_host(p, 4, 4, 3, 0, ctypes.byref(h)) == sp.SPMM_E_ARG
    assert L.spmm_pack_host(p, 4, 4, 4, 7, ctypes.byref(h)) == sp.SPMM_E_ARG
    assert L.spmm_pack_host(p, 4, 70000, 70000, 0, ctypes.byref(h)) == sp.SPMM_E_UNSUPPORTED
    assert h.value is None
    assert L.spmm_unpack(None, p, 4) == sp.SPMM_E_ARG
    assert L.spmm_info(None, None, None, None, None, None) == sp.SPMM_E_ARG
    L.spmm_destroy(None)                             # allowed
    hh = sp.spmm_pack_host(W)
    assert L.spmm_unpack(hh, p, 3) == sp.SPMM_E_ARG
    ep = sp.make_epilogue()
    assert sp.spmm_run_status(hh, 16, 4, 4, ep, 16, 4) == sp.SPMM_E_ARG      # host-only handle
    assert L.spmm_set_tuning(hh, 48, 0) == sp.SPMM_E_UNSUPPORTED
    assert L.spmm_set_tuning(hh, 128, 101) == sp.SPMM_E_UNSUPPORTED
    assert L.spmm_set_tuning(hh, 0, 8) == sp.SPMM_E_ARG
    assert L.spmm_set_tuning(hh, 64, 0) == sp.SPMM_E_UNSUPPORTED
    assert L.spmm_set_tuning(hh, 64, 102) == sp.SPMM_OK
    assert L.spmm_set_tuning(hh, 32, 101) == sp.SPMM_OK
    assert L.spmm_set_tuning(hh, 16, 101) == sp.SPMM_OK
    assert L.spmm_set_tuning(hh, 32, 102) == sp.SPMM_E_UNSUPPORTED
    assert L.spmm_set_tuning(hh, 16, 0) == sp.SPMM_E_UNSUPPORTED
    assert L.spmm_set_tuning(hh, 16, 103) == sp.SPMM_OK
    assert L.spmm_set_tuning(hh, 32, 103) == sp.SPMM_OK
    assert L.spmm_set_tuning(hh, 64, 103) == sp.SPMM_E_UNSUPPORTED
    assert L.spmm_set_tuning(hh, 64, 104) == sp.SPMM_OK
    assert L.spmm_set_tuning(hh, 128, 104) == sp.SPMM_E_UNSUPPORTED
    assert L.spmm_set_tuning(hh, 96, 16) == sp.SPMM_OK
    assert L.spmm_set_tuning(hh, 96, 8) == sp.SPMM_E_UNSUPPORTED
    assert L.spmm_set_tuning(hh, 0, 0) == sp.SPMM_OK
    sp.spmm_destroy(hh)


def test_gelu_lut_matches_oracle_table_entry_by_entry():
    for mid, outs, zp, ot in [(0.1, 0.1, 0, "s8"), (0.42, 0.42, 0, "s8"), (0.05, 0.02, -100, "s8"),
                              (0.3, 0.15, 4, "u8")]:
        assert np.array_equal(sp.spmm_make_gelu_lut(mid, outs, zp, ot), oracle.gelu_lut(mid, outs, zp, ot))
    L = sp.lib()
    buf = np.zeros(256, np.int8).ctypes.data_as(ctypes.c_void_p)
    assert L.spmm_make_gelu_lut(0.0, 1.0, 0, sp.SPMM_OUT_S8, buf) == sp.SPMM_E_ARG
    assert L.spmm_make_gelu_lut(1.0, 1.0, 0, sp.SPMM_OUT_F32, buf) == sp.SPMM_E_ARG
    assert L.spmm_make_gelu_lut(1.0, 1.0, 300, sp.SPMM_OUT_S8, buf) == sp.SPMM_E_ARG
    assert L.spmm_make_gelu_lut(1.0, 1.0, 0, sp.SPMM_OUT_S8, None) == sp.SPMM_E_ARG


def _half_read_conflicts(idx, seg_ptr, n_tiles, n_seg):
    """Extra LDS passes of the layout: for every half-read (16 rows read together by half a
    wave in one transposing read) the largest number of rows sharing a residue mod 16, minus 1."""
    extra = total = 0
    for s in range(int(seg_ptr[-1])):
        for instr in range(2):
            for pair in range(2):
                rows = []
                for g in (2 * pair, 2 * pair + 1):
                    for t in range(8):
                        e = int(idx[s, 8 * g + t])
                        rows.append((e & 0xFFFF) if instr == 0 else (e >> 16))
                counts = np.bincount(np.array(rows) % 16, minlength=16)
                extra += int(counts.max()) - 1
                total += 1
    return extra / max(1, total)


@pytest.mark.parametrize("sparsity", [0.9, 0.8, 0.7])
def test_step_order_avoids_lds_bank_conflicts(sparsity):
    W = wl.sparse_weight(256, 1024, sparsity, keys=(80, int(sparsity * 100)))
    h = sp.spmm_pack_host(W)
    try:
        _, _, _, n_tiles, n_seg, _ = sp.spmm_layout_dims(h)
        _, idx, seg_ptr, _ = sp.spmm_layout_export(h)
        # ascending order would give about 1.9 extra passes per half-read (16 random residues)
        # (a residue class with more entries than half-reads must double up, so not 0)
        assert _half_read_conflicts(idx, seg_ptr, n_tiles, n_seg) < 1.0
    finally:
        sp.spmm_destroy(h)


def test_plan_picks_token_tile_and_waves_per_shape():
    """The offline choice of the kernel configuration (host-only handles assume 256 CUs):
    (token tile, rows per workgroup, workgroups) for the shapes the choices were measured on."""
    def plan(N, K, M, sparsity, tuning=None):
        W = wl.sparse_weight(N, K, sparsity, keys=(81, N, K))
        h = sp.spmm_pack_host(W)
        try:
            if tuning:
                sp.spmm_set_tuning(h, *tuning)
            return tuple(sp.spmm_plan(h, M, "s8"))
        finally:
            sp.spmm_destroy(h)

    assert plan(4096, 1024, 6144, 0.9) == (128, 256, 256)       # 16 row groups x 16 streams of 3 tiles
    assert plan(1024, 1024, 6144, 0.9) == (96, 256, 256)        # 4 row groups: 64 tiles of 96 fill the CUs, 48 of 128 do not
    assert plan(1024, 1024, 6144, 0.8) == (96, 256, 256)
    assert plan(768, 768, 4096, 0.9) == (128, 128, 192)         # few row groups: 8-wave workgroups
    assert plan(1024, 1024, 6144, 0.5)[1] == 128                # more than 6 steps per segment: 8 waves
    assert plan(1024, 1024, 6144, 0.9, (128, 8)) == (128, 128, 256)
    assert plan(1024, 1024, 6144, 0.9, (96, 16)) == (96, 256, 256)
    assert plan(256, 256, 128, 0.9, (64, 102))[0] == 64
    # short batch: simple kernel, 6 row groups x 8 tiles of 16; the packed weight is larger than X, so a row
    # group's workgroups share an XCD and the grid is padded to 8 row groups
    assert plan(768, 768, 128, 0.9) == (16, 128, 64)
    assert plan(768, 3072, 1024, 0.9) == (32, 128, 192)          # 6 x 32 tiles of 32 still fit the 256 CUs, 6 x 64 do not
    assert plan(3072, 768, 384, 0.9) == (64, 128, 144)           # 24 row groups: only 64-token tiles fit (24 x 6)
    assert plan(768, 768, 128, 0.9, (32, 101)) == (32, 128, 32)
    assert plan(768, 768, 128, 0.9, (16, 101)) == (16, 128, 64)

    def kernel(N, K, M, tuning=None):
        h = sp.spmm_pack_host(wl.sparse_weight(N, K, 0.9, keys=(81, N, K)))
        try:
            if tuning:
                sp.spmm_set_tuning(h, *tuning)
            return sp.spmm_kernel_variant(h, M, "s8", "gelu")
        finally:
            sp.spmm_destroy(h)

    # short batches: the short-batch kernel from five K segments on, up to the eight it holds
    assert kernel(768, 3072, 128) == "void spmm::spmm_rowtile_mfma_slab<16, 8, 2, 1>(spmm::KernelArgs)"
    assert kernel(1024, 4096, 32) == "void spmm::spmm_rowtile_mfma_slab<16, 8, 2, 1>(spmm::KernelArgs)"
    assert kernel(768, 2048, 128) == "void spmm::spmm_rowtile_mfma_simple<16, 8, 1, 2, 1>(spmm::KernelArgs)"
    assert kernel(768, 4608, 128) == "void spmm::spmm_rowtile_mfma_stream<16, 8, 2, 1>(spmm::KernelArgs)"
    assert kernel(768, 768, 128, (16, 103)) == "void spmm::spmm_rowtile_mfma_slab<16, 8, 2, 1>(spmm::KernelArgs)"
    assert kernel(768, 3072, 1024) == "void spmm::spmm_rowtile_mfma_slab<32, 8, 2, 1>(spmm::KernelArgs)"
    assert kernel(1024, 4096, 1024) == "void spmm::spmm_rowtile_mfma_stream<32, 8, 2, 1>(spmm::KernelArgs)"
    assert kernel(768, 768, 128, (64, 104)) == "void spmm::spmm_rowtile_mfma_stream<64, 8, 2, 1>(spmm::KernelArgs)"
    assert kernel(768, 3072, 6144) == "void spmm::spmm_rowtile_mfma<96, 16, 4, 2, 1, 0>(spmm::KernelArgs)"
    assert kernel(4096, 1024, 6144) == "void spmm::spmm_rowtile_mfma<128, 16, 4, 2, 1, 0>(spmm::KernelArgs)"
    assert plan(768, 768, 128, 0.9, (128, 8)) == (128, 128, 6)

    # 4-byte outputs: workgroups of 12 or 8 compute waves plus 4 loader waves
    def kernel32(N, K, M, out_type="f32", tuning=None):
        h = sp.spmm_pack_host(wl.sparse_weight(N, K, 0.9, keys=(81, N, K)))
        try:
            if tuning:
                sp.spmm_set_tuning(h, *tuning)
            return sp.spmm_kernel_variant(h, M, out_type, "none"), tuple(sp.spmm_plan(h, M, out_type))
        finally:
            sp.spmm_destroy(h)

    assert kernel32(3072, 768, 4096) == ("void spmm::spmm_rowtile_mfma_fed<128, 12, 4, 4, 1, 0>(spmm::KernelArgs)",
                                         (128, 192, 256))           # 16 row groups x 16 streams of 2 tiles
    assert kernel32(768, 3072, 4096)[0] == "void spmm::spmm_rowtile_mfma_fed<64, 12, 4, 4, 1, 0>(spmm::KernelArgs)"
    assert kernel32(768, 768, 4096, "s32")[0] == "void spmm::spmm_rowtile_mfma_fed<64, 12, 4, 4, 0, 0>(spmm::KernelArgs)"
    assert kernel32(1024, 1024, 4096)[0] == "void spmm::spmm_rowtile_mfma_fed<128, 8, 4, 4, 1, 0>(spmm::KernelArgs)"
    assert kernel32(768, 3072, 6144)[0] == "void spmm::spmm_rowtile_mfma_fed<96, 12, 4, 4, 1, 0>(spmm::KernelArgs)"
    assert kernel32(768, 768, 128)[0].startswith("void spmm::spmm_rowtile_mfma_simple<16")    # short batches: unchanged
    assert kernel32(1024, 1024, 6144, "f32", (96, 112))[0] == "void spmm::spmm_rowtile_mfma_fed<96, 12, 4, 4, 1, 0>(spmm::KernelArgs)"
    assert kernel32(1024, 1024, 6144, "f32", (128, 108))[1] == (128, 128, 256)


# ---- offline row ordering (Section 3.2: the blocking is tunable offline) -------------------------

ORDER_CASES = [("n4k1", 256, 256, 0.9, 0), ("n1k4", 256, 256, 0.9, 0), ("n4k1", 50, 70, 0.5, 0),
               ("n4k1", 3, 5, 0.0, 0), ("n1k4", 37, 131, 0.7, 0), ("n4k1", 512, 1024, 0.9, 8),
               ("n1k4", 128, 1024, 0.9, 4), ("n4k1", 130, 600, 0.8, 3)]


@pytest.mark.parametrize("orient,N,K,s,clusters", ORDER_CASES)
def test_reordered_pack_is_a_block_row_permutation_and_round_trips(orient, N, K, s, clusters):
    W = wl.sparse_weight(N, K, s, orient, jitter=0.2, keys=(78, N, K), clusters=clusters)
    plain = sp.spmm_pack_host(W, orient)
    h = sp.spmm_pack_ex(W, orient, host_only=True, reorder_rows=True)
    try:
        order = sp.spmm_row_order(h)
        assert sorted(order.tolist()) == list(range(N))                    # a permutation of the rows
        if orient == "n4k1":                                               # ... that moves whole block-rows
            full = N // 4 * 4
            blocks = order[:full].reshape(-1, 4)
            assert np.all(blocks[:, 0] % 4 == 0) and np.all(blocks == blocks[:, :1] + np.arange(4))
            assert np.array_equal(order[full:], np.arange(full, N))        # the partial block-row stays last
        assert np.array_equal(sp.spmm_unpack(h), W)                        # unpack: the matrix as given
        assert np.array_equal(sp.spmm_row_order(plain), np.arange(N))
        # the handle IS the plain packing of the row-permuted matrix, bit for bit
        ref = sp.spmm_pack_host(np.ascontiguousarray(W[order]), orient)
        try:
            assert sp.spmm_layout_dims(h) == sp.spmm_layout_dims(ref)
            for a, b in zip(sp.spmm_layout_export(h), sp.spmm_layout_export(ref)):
                assert np.array_equal(a, b)
        finally:
            sp.spmm_destroy(ref)
        # ... and its layout replays to the oracle's accumulator of the permuted rows
        X = wl.activations(K, 24, keys=(78, N, K))
        assert np.array_equal(decode_layout_acc(h, X), oracle.acc_s32(W, X).astype(np.int64)[order])
        assert sp.spmm_info(h)[2] == sp.spmm_info(plain)[2]                # same non-zero blocks
    finally:
        sp.spmm_destroy(h)
        sp.spmm_destroy(plain)


def test_reordering_finds_planted_clusters():
    """Block-rows that follow 8 prototype patterns, in random order: after clustering a row tile
    multiplies little more than one pattern instead of the union of four."""
    W = wl.sparse_weight(1024, 1024, 0.9, "n4k1", keys=(79,), clusters=8)
    plain = sp.spmm_pack_host(W)
    h = sp.spmm_pack_ex(W, host_only=True, reorder_rows=True)
    try:
        assert sp.spmm_info(h)[3] <= 0.65 * sp.spmm_info(plain)[3]
    finally:
        sp.spmm_destroy(h)
        sp.spmm_destroy(plain)
    # and never makes a uniformly random pattern worse
    W = wl.sparse_weight(1024, 1024, 0.9, "n4k1", jitter=0.2, keys=(80,))
    plain = sp.spmm_pack_host(W)
    h = sp.spmm_pack_ex(W, host_only=True, reorder_rows=True)
    try:
        assert sp.spmm_info(h)[3] <= sp.spmm_info(plain)[3]
    finally:
        sp.spmm_destroy(h)
        sp.spmm_destroy(plain)


def test_pack_ex_rejects_unknown_flags():
    W = np.zeros((8, 8), dtype=np.int8)
    h = ctypes.c_void_p()
    rc = sp.lib().spmm_pack_ex(W.ctypes.data_as(ctypes.c_void_p), 8, 8, 8, 0, 4, ctypes.byref(h))
    assert rc == 1 and not h.value


def test_binding_refuses_buffers_smaller_than_the_call_touches():
    """Marshalling-side guard: a tensor built for another shape raises in Python instead of reaching the device."""
    torch = pytest.importorskip("torch")
    h = sp.spmm_pack_host(wl.sparse_weight(256, 256, 0.9, keys=(85,)))
    try:
        ep = sp.make_epilogue(None, 1.0, 0, None, "none", "s8", 1.0, 0, 1.0, None)
        X = torch.zeros((256, 128), dtype=torch.uint8)
        small = torch.zeros((64, 128), dtype=torch.int8)
        for fn, args in ((sp.spmm_run, (h, X, 128, 128, ep, small, 128)), (sp.spmm_run_bound, (h, X, 128, 128, ep, small, 128)),
                         (sp.spmm_run_tiled, (h, X, 128, 128, ep, small, 128, 3)),
                         (sp.spmm_run_tiled_bound, (h, torch.zeros((100, 128), dtype=torch.uint8), 128, 128, ep,
                                                    torch.zeros((256, 128), dtype=torch.int8), 128, 1))):
            with pytest.raises(ValueError):
                fn(*args)
        # a view into a larger storage counts from its own offset; a sufficient one reaches the library
        # (which refuses this host-only handle)
        big = torch.zeros(256 * 128 + 64, dtype=torch.int8)
        with pytest.raises(sp.SpmmError):
            sp.spmm_run(h, X, 128, 128, ep, big[64:].view(256, 128), 128)
        with pytest.raises(ValueError):
            sp.spmm_run(h, X, 128, 128, ep, big[65:], 128)
    finally:
        sp.spmm_destroy(h)
