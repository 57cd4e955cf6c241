"""The synthetic inputs have the structure the configurations ask for."""
import numpy as np
import pytest

import workloads as wl


def test_tiny_exact_counts_n4k1():
    c = wl.tiny_cases(wl.N4K1)[0]
    W = wl.make(c)["W"]
    assert W.dtype == np.int8 and W.shape == (256, 256)
    blk = (W.reshape(64, 4, 256) != 0)
    # kept blocks are full (no zero inside), dropped blocks are empty
    assert np.array_equal(blk.any(axis=1), blk.all(axis=1))
    per_block_row = blk.any(axis=1).sum(axis=1)
    assert (per_block_row == 26).all()                 # floor(0.1*256 + 0.5)
    nz, tot = wl.realised_block_sparsity(W, wl.N4K1)
    assert nz == 64 * 26 and tot == 64 * 256
    assert W.min() >= -127 and W.max() <= 127


def test_tiny_exact_counts_n1k4():
    c = wl.tiny_cases(wl.N1K4)[0]
    W = wl.make(c)["W"]
    blk = (W.reshape(256, 64, 4) != 0)
    assert np.array_equal(blk.any(axis=2), blk.all(axis=2))
    assert (blk.any(axis=2).sum(axis=1) == 6).all()    # floor(0.1*64 + 0.5)


def test_same_seed_same_bytes_and_distinct_streams():
    c = wl.mini_cases()[0]
    a, b = wl.make(c), wl.make(c)
    for k in ("W", "X", "w_scale", "bias"):
        assert wl.sha256(a[k]) == wl.sha256(b[k])
    other = wl.make(wl.mini_cases()[1])
    assert wl.sha256(a["X"]) != wl.sha256(other["X"][:256, :])


def test_value_distributions():
    d = wl.make(wl.mini_cases()[0])
    X, ws, b = d["X"], d["w_scale"], d["bias"]
    assert X.dtype == np.uint8 and X.min() == 0 and X.max() == 255
    assert abs(X.mean() - 127.5) < 1.0
    assert ws.dtype == np.float32 and ws.min() >= 1e-3 and ws.max() <= 1e-2
    assert b.dtype == np.float32 and abs(float(b.mean())) < 0.15 and 0.85 < float(b.std()) < 1.15
    assert d["x_scale"] == 0.02


def test_jitter_spreads_counts_within_20_percent():
    W = wl.sparse_weight(512, 1024, 0.8, wl.N4K1, jitter=0.2, keys=(5, 1))
    cnt = (W.reshape(128, 4, 1024) != 0).any(axis=1).sum(axis=1)
    c = 0.2 * 1024
    assert cnt.min() >= np.floor(c * 0.8) and cnt.max() <= np.ceil(c * 1.2) + 1
    assert cnt.std() > 5


def test_ragged_dims():
    W = wl.sparse_weight(10, 9, 0.5, wl.N4K1, keys=(6,))
    assert W.shape == (10, 9)
    W = wl.sparse_weight(10, 9, 0.5, wl.N1K4, keys=(6,))
    assert W.shape == (10, 9)


def test_grid_has_23_shape_pairs_and_92_shapes():
    assert len(wl.grid_shapes()) == 23
    assert len(wl.grid_cases(sparsities=(0.9,))) == 92
    assert len(wl.grid_cases()) == 460


def test_config_catalogue():
    assert [c.out_type for c in wl.mini_cases()] == ["f32", "s8"]
    assert [c.postop for c in wl.mini_cases()] == ["gelu", "none"]
    assert len(wl.base_cases()) == 3 * 5 * 3
    lc = wl.large_cases()
    assert len(lc) == 6 and all(c.M == 6144 and c.out_type == "s8" and c.postop == "gelu" for c in lc)


def test_quant_scales_clip_a_small_fraction():
    import oracle
    c = wl.mini_cases()[1]
    d = wl.make(c)
    y = oracle.spmm(d["W"], d["X"], d["w_scale"], d["x_scale"], d["bias"], "none", "f32")
    sigma = wl.preact_sigma(c.K, c.sparsity)
    assert 0.8 * sigma < float(y.std()) < 1.2 * sigma
    q = oracle.spmm(d["W"], d["X"], d["w_scale"], d["x_scale"], d["bias"], "none", "s8", d["out_scale"])
    sat = float(((q == 127) | (q == -128)).mean())
    assert 0.0 < sat < 0.02


def test_chain_pair_inputs_link_the_two_stages():
    cases = wl.chain_cases()
    d1, d2 = wl.make_chain(cases)
    assert cases[0].N == cases[1].K and cases[0].M == cases[1].M
    assert d2["X"] is None and d2["x_scale"] == d1["out_scale"] and d2["x_zero_point"] == d1["out_zero_point"]
    assert 0 < d1["out_zero_point"] < 64 and d1["out_scale"] > 0 and d2["out_scale"] > 0
