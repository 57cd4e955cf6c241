"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle on the
same seeded inputs.  Bars: int32 / int8 / uint8 outputs bit-exact; fp32 without GELU
bit-equal (same fused multiply-add); fp32 with GELU |gpu - ref| <= 1e-5*|ref| + 1e-7
(two different erfc implementations; the absolute term covers the cancelling tail).
"""
import numpy as np
import pytest

import oracle
import paper_2306_16601_amd as sp
import workloads as wl

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

GUARD = 64          # poisoned elements before and after the output buffer
POISON = {"s32": 0x5A5A5A5A, "f32": 12345.678, "s8": 0x5A, "u8": 0xA5}
TORCH_DT = {"s32": torch.int32, "f32": torch.float32, "s8": torch.int8, "u8": torch.uint8}


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def gpu_spmm(W, X, d, case, ldx=None, ldo=None, tuning=None, stream=None, x_offset=0, out_offset=0, x_tiled=False):
    """Pack W, run the library on device copies of the inputs, return (out, guards_ok).
    x_tiled: hand the activations over in token-tile-major order (spmm_run_tiled)."""
    N, K = W.shape
    M = X.shape[1]
    ldx = ldx or M
    ldo = ldo or M
    h = sp.spmm_pack(W, case.orientation)
    try:
        if tuning:
            sp.spmm_set_tuning(h, *tuning)
        Xbuf = torch.zeros(K * ldx + x_offset + 16, dtype=torch.uint8, device="cuda")
        Xv = Xbuf[x_offset:x_offset + K * ldx].view(K, ldx)
        Xv[:, :M] = dev(X)
        if ldx > M:
            Xv[:, M:] = 0xEE                                   # must never influence the result
        ot = case.out_type
        total = N * ldo + 2 * GUARD + out_offset
        obuf = torch.full((total,), POISON[ot], dtype=TORCH_DT[ot], device="cuda")
        oview = obuf[GUARD + out_offset:GUARD + out_offset + N * ldo].view(N, ldo)
        lut = None
        if case.postop == "gelu" and ot in ("s8", "u8"):
            lut = dev(sp.spmm_make_gelu_lut(d["mid_scale"], d["out_scale"], d["out_zero_point"], ot))
        w_scale = dev(d["w_scale"]) if d.get("w_scale") is not None else None
        bias = dev(d["bias"]) if d.get("bias") is not None else None
        ep = sp.make_epilogue(w_scale, d["x_scale"], d["x_zero_point"], bias, case.postop, ot,
                              d["out_scale"], d["out_zero_point"], d["mid_scale"], lut)
        st = stream.cuda_stream if stream is not None else torch.cuda.current_stream().cuda_stream
        if x_tiled:
            Xt = dev(sp.tile_major(X))
            Xt[-1, :, M - sp.binding.SPMM_X_TILE * (Xt.shape[0] - 1):] = 0xEE      # the padding of the last tile must never matter
            sp.spmm_run_tiled(h, Xt, M, 0, ep, oview, ldo, sp.binding.SPMM_TILED_X, st)
        else:
            sp.spmm_run(h, Xv, M, ldx, ep, oview, ldo, st)
        torch.cuda.synchronize()
        out = oview[:, :M].cpu().numpy()
        full = obuf.cpu().numpy()
        poison = np.array(POISON[ot]).astype(full.dtype)
        guards_ok = (full[:GUARD + out_offset] == poison).all() and (full[GUARD + out_offset + N * ldo:] == poison).all()
        if ldo > M:
            guards_ok = guards_ok and (oview[:, M:].cpu().numpy() == poison).all()
        return out, bool(guards_ok)
    finally:
        sp.spmm_destroy(h)


def oracle_spmm(W, X, d, case):
    return oracle.spmm(W, X, d["w_scale"], d["x_scale"], d["bias"], case.postop, case.out_type,
                       d["out_scale"], d["out_zero_point"], d["mid_scale"], d["x_zero_point"])


def assert_parity(got, ref, case):
    assert got.shape == ref.shape and got.dtype == ref.dtype
    if case.out_type == "f32" and case.postop == "gelu":
        err = np.abs(got.astype(np.float64) - ref.astype(np.float64))
        tol = 1e-5 * np.abs(ref.astype(np.float64)) + 1e-7
        bad = err > tol
        assert not bad.any(), "fp32 GELU: %d of %d outside 1e-5 rel + 1e-7 abs, worst %g" % (
            bad.sum(), bad.size, (err / tol).max())
    elif case.out_type == "f32":
        assert np.array_equal(got.view(np.uint32), ref.view(np.uint32)), "fp32 outputs differ bitwise"
    else:
        neq = got != ref
        assert not neq.any(), "%d of %d outputs differ (first at %s)" % (
            neq.sum(), neq.size, np.argwhere(neq)[0] if neq.any() else None)


def check_case(case, **kw):
    d = wl.make(case)
    got, guards_ok = gpu_spmm(d["W"], d["X"], d, case, **kw)
    ref = oracle_spmm(d["W"], d["X"], d, case)
    assert guards_ok, "write outside the output extent"
    assert_parity(got, ref, case)
    return got


# ---------------------------------------------------------------------------- configs 1-4
@pytest.mark.parametrize("orient", [wl.N4K1, wl.N1K4])
def test_config1_tiny(orient):
    check_case(wl.tiny_cases(orient)[0])


@pytest.mark.parametrize("orient", [wl.N4K1, wl.N1K4])
def test_config2_mini_ffn_pair(orient):
    for case in wl.mini_cases(orient):
        check_case(case)


@pytest.mark.parametrize("case", wl.base_cases(batches=(1,)), ids=lambda c: c.name)
def test_config3_base_sweep_m128(case):
    check_case(case)


@pytest.mark.parametrize("case", wl.base_cases(batches=(8, 32)), ids=lambda c: c.name)
def test_config3_base_larger_batches(case):
    check_case(case)


@pytest.mark.parametrize("case", wl.large_cases(), ids=lambda c: c.name)
def test_config4_large_full_size(case):
    check_case(case)


def test_config4_large_all_kernel_variants_agree_bitwise():
    # int32 accumulation is order-free: every kernel configuration must give identical bytes
    case = wl.large_cases()[0]
    d = wl.make(case)
    a, _ = gpu_spmm(d["W"], d["X"], d, case)
    for tuning in ((128, 0), (128, 8), (128, 16), (96, 0), (96, 16), (128, 112), (128, 108), (96, 112), (64, 112), (64, 101), (64, 102), (32, 101), (16, 101), (16, 103), (32, 103), (64, 104), (32, 104), (16, 104)):
        b, _ = gpu_spmm(d["W"], d["X"], d, case, tuning=tuning)
        assert np.array_equal(a, b), tuning


# ---------------------------------------------------------------------------- beyond the five configs
def _run_with_table(d, case, table):
    """spmm_run with a caller-built 256-entry table in place of the GELU one."""
    h = sp.spmm_pack(d["W"], case.orientation)
    try:
        out = torch.empty((case.N, case.M), dtype=TORCH_DT[case.out_type], device="cuda")
        w_scale, bias, lut, X = dev(d["w_scale"]), dev(d["bias"]), dev(table), dev(d["X"])   # alive until the sync
        ep = sp.make_epilogue(w_scale, d["x_scale"], d["x_zero_point"], bias, "table",
                              case.out_type, d["out_scale"], d["out_zero_point"], d["mid_scale"], lut)
        sp.spmm_run(h, X, case.M, case.M, ep, out, case.M, torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        return out.cpu().numpy()
    finally:
        sp.spmm_destroy(h)


@pytest.mark.parametrize("out_type", ["s8", "u8"])
def test_table_of_any_elementwise_chain(out_type):
    # Algorithm 2 holds for every element-wise chain with a low-precision input: the library only
    # looks the key up, so a table of some other chain (here tanh -> requantise, and a random
    # permutation) must come out exactly as the oracle's look-up of the same table.
    case = wl.Case("table", 80, 300, 333, 0.8, wl.N4K1, out_type, "gelu", keys=(91, 80, 300, 333))
    d = wl.make(case)
    keys = np.arange(-128, 128, dtype=np.float64)
    lo, hi = (0, 255) if out_type == "u8" else (-128, 127)
    tanh_q = np.clip(np.rint(np.tanh(keys * float(d["mid_scale"])) * 100.0) + (128 if out_type == "u8" else 0), lo, hi)
    perm = wl.rng_for(92, 7).permutation(256) + lo
    for table in (tanh_q, perm):
        table = table.astype(np.uint8 if out_type == "u8" else np.int8)
        got = _run_with_table(d, case, table.view(np.int8))
        ref = oracle.spmm(d["W"], d["X"], d["w_scale"], d["x_scale"], d["bias"], "table", out_type, d["out_scale"],
                          d["out_zero_point"], d["mid_scale"], d["x_zero_point"], lut=table)
        assert np.array_equal(got, ref)
        assert len(np.unique(got)) > 8      # the table is really exercised


def test_chained_ffn_pair_stays_quantised_on_device():
    # Figure 3 / Algorithm 2: W1 -> bias -> GELU -> uint8 (table chain, with a zero point) feeds W2 -> int8
    # directly: the first launch's output buffer is the second launch's activation matrix, no fp32 tensor
    # and no host round trip between them.  Both stages against the oracle chained the same way.
    cases = wl.chain_cases()
    d1, d2 = wl.make_chain(cases)
    c1, c2 = cases
    h1, h2 = sp.spmm_pack(d1["W"], c1.orientation), sp.spmm_pack(d2["W"], c2.orientation)
    try:
        M = c1.M
        X = dev(d1["X"])
        hid = torch.full((c1.N, M), 0xA5, dtype=torch.uint8, device="cuda")
        out = torch.full((c2.N, M), 0x5A, dtype=torch.int8, device="cuda")
        lut = dev(sp.spmm_make_gelu_lut(d1["mid_scale"], d1["out_scale"], d1["out_zero_point"], "u8"))
        ep1 = sp.make_epilogue(dev(d1["w_scale"]), d1["x_scale"], 0, dev(d1["bias"]), "gelu", "u8",
                               d1["out_scale"], d1["out_zero_point"], d1["mid_scale"], lut)
        ep2 = sp.make_epilogue(dev(d2["w_scale"]), d2["x_scale"], d2["x_zero_point"], dev(d2["bias"]), "none", "s8",
                               d2["out_scale"], 0)
        st = torch.cuda.current_stream().cuda_stream
        sp.spmm_run(h1, X, M, M, ep1, hid, M, st)
        sp.spmm_run(h2, hid, M, M, ep2, out, M, st)       # same stream: ordered behind the first
        torch.cuda.synchronize()
        ref1 = oracle.spmm(d1["W"], d1["X"], d1["w_scale"], d1["x_scale"], d1["bias"], "gelu", "u8",
                           d1["out_scale"], d1["out_zero_point"], d1["mid_scale"])
        ref2 = oracle.spmm(d2["W"], ref1, d2["w_scale"], d2["x_scale"], d2["bias"], "none", "s8",
                           d2["out_scale"], 0, 1.0, d2["x_zero_point"])
        assert d1["out_zero_point"] > 0 and len(np.unique(ref1)) > 100 and len(np.unique(ref2)) > 100
        assert np.array_equal(hid.cpu().numpy(), ref1)
        assert np.array_equal(out.cpu().numpy(), ref2)
    finally:
        sp.spmm_destroy(h1)
        sp.spmm_destroy(h2)


def test_stacked_qkv_is_three_projections():
    # Q, K and V share one X (Figure 3(a)): packing the three weights as one [3N, K] matrix gives
    # one launch whose output is the three separate outputs stacked, bit for bit.
    N, K, M = 256, 256, 640
    cases = [wl.Case("qkv%d" % i, N, K, M, 0.85, wl.N4K1, "s8", "none", keys=(93, i)) for i in range(3)]
    ds = [wl.make(c) for c in cases]
    X = ds[0]["X"]
    sep = []
    for c, d in zip(cases, ds):
        d = dict(d, X=X, out_scale=ds[0]["out_scale"], x_scale=ds[0]["x_scale"])
        out, ok = gpu_spmm(d["W"], X, d, c)
        assert ok
        ref = oracle_spmm(d["W"], X, d, c)
        assert np.array_equal(out, ref)
        sep.append(out)
    stacked = dict(ds[0], W=np.concatenate([d["W"] for d in ds]), X=X,
                   w_scale=np.concatenate([d["w_scale"] for d in ds]), bias=np.concatenate([d["bias"] for d in ds]))
    big = wl.Case("qkv", 3 * N, K, M, 0.85, wl.N4K1, "s8", "none", keys=(93,))
    out, ok = gpu_spmm(stacked["W"], X, stacked, big)
    assert ok
    assert np.array_equal(out, np.concatenate(sep))


def _run_sum(d, case, R, ld_sum, tuning=None, r_offset=0):
    h = sp.spmm_pack(d["W"], case.orientation)
    try:
        if tuning:
            sp.spmm_set_tuning(h, *tuning)
        N, M = case.N, case.M
        out = torch.full((N, M), POISON[case.out_type], dtype=TORCH_DT[case.out_type], device="cuda")
        rbuf = torch.full((N * ld_sum + r_offset + 8,), 7.25, dtype=torch.float32, device="cuda")
        rv = rbuf[r_offset:r_offset + N * ld_sum].view(N, ld_sum)
        rv[:, :M] = dev(R)
        w_scale, bias, X = dev(d["w_scale"]), dev(d["bias"]), dev(d["X"])
        ep = sp.make_epilogue(w_scale, d["x_scale"], d["x_zero_point"], bias, case.postop, case.out_type,
                              d["out_scale"], d["out_zero_point"], d["mid_scale"], None, rv, ld_sum)
        sp.spmm_run(h, X, M, M, ep, out, M, torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        return out.cpu().numpy()
    finally:
        sp.spmm_destroy(h)


@pytest.mark.parametrize("out_type,postop", [("f32", "none"), ("f32", "gelu"), ("s8", "none"), ("u8", "none")])
@pytest.mark.parametrize("N,K,M", [(272, 600, 384), (100, 130, 333), (512, 1024, 1000)])
def test_sum_postop(N, K, M, out_type, postop):
    # Sum (Figure 3): a second fp32 tensor added after BiasAdd / GeLU and before Quantize
    case = wl.Case("sum", N, K, M, 0.8, wl.N4K1, out_type, postop, keys=(94, N, K, M))
    d = wl.make(case)
    R = (wl.rng_for(95, N, M).standard_normal((N, M)) * wl.preact_sigma(K, case.sparsity)).astype(np.float32)
    ref = oracle.spmm(d["W"], d["X"], d["w_scale"], d["x_scale"], d["bias"], postop, out_type, d["out_scale"],
                      d["out_zero_point"], d["mid_scale"], d["x_zero_point"], sum=R)
    plain = oracle_spmm(d["W"], d["X"], d, case)
    assert np.mean(ref != plain) > 0.5                     # the residual matters in this test
    for ld_sum, off, tuning in ((M, 0, None), (M + 4, 0, (96, 16)), (M + 3, 1, None), (M + 8, 4, (128, 8)),
                                (M, 0, (64, 102)), (M + 4, 0, (32, 101)), (M + 1, 3, (16, 101)), (M, 0, (16, 103)),
                                (M + 2, 2, (16, 103)), (M + 4, 0, (32, 103)), (M, 0, (64, 104)), (M + 1, 1, (32, 104))):
        got = _run_sum(d, case, R, ld_sum, tuning, off)
        if out_type == "f32" and postop == "gelu":
            # the two sides' erfc differ by <= 1e-5 relative in GELU(y); the add then rounds once
            g = np.abs(ref.astype(np.float64) - R.astype(np.float64))
            tol = 1e-5 * g + 1e-7 + 2.0 ** -23 * np.abs(ref.astype(np.float64))
            assert (np.abs(got.astype(np.float64) - ref.astype(np.float64)) <= tol).all(), (ld_sum, off, tuning)
        else:
            assert_parity(got, ref, case)


def test_sum_argument_errors():
    case = wl.Case("sumerr", 32, 64, 48, 0.5, wl.N4K1, "s8", "gelu", keys=(96,))
    d = wl.make(case)
    h = sp.spmm_pack(d["W"])
    try:
        X = dev(d["X"])
        R = torch.zeros((32, 48), dtype=torch.float32, device="cuda")
        ws, lut = dev(d["w_scale"]), dev(sp.spmm_make_gelu_lut(d["mid_scale"], d["out_scale"], 0, "s8"))
        out8 = torch.zeros((32, 48), dtype=torch.int8, device="cuda")
        out32 = torch.zeros((32, 48), dtype=torch.int32, device="cuda")
        ep = sp.make_epilogue(ws, d["x_scale"], 0, None, "gelu", "s8", d["out_scale"], 0, d["mid_scale"], lut, R, 48)
        assert sp.spmm_run_status(h, X, 48, 48, ep, out8, 48) == sp.SPMM_E_UNSUPPORTED    # table chain + Sum
        ep = sp.make_epilogue(ws, d["x_scale"], 0, None, "none", "s32", sum=R, ld_sum=48)
        assert sp.spmm_run_status(h, X, 48, 48, ep, out32, 48) == sp.SPMM_E_UNSUPPORTED   # raw accumulators + Sum
        ep = sp.make_epilogue(ws, d["x_scale"], 0, None, "none", "s8", d["out_scale"], 0, sum=R, ld_sum=47)
        assert sp.spmm_run_status(h, X, 48, 48, ep, out8, 48) == sp.SPMM_E_ARG            # ld_sum < M
        torch.cuda.synchronize()
        assert int(out8.abs().sum()) == 0 and int(out32.abs().sum()) == 0                 # outputs untouched
    finally:
        sp.spmm_destroy(h)


def test_gelu_f32_dense_sweep_of_preactivations():
    # One non-zero weight (+1) per row: acc = x in [0, 255], y = x * s[n] + b[n].  Rows are given
    # scales and biases that make y sweep [-13, 13] in ~260 k distinct steps, dense around 0 and
    # through the negative tail where GELU is tiny; every value must meet the fp32 bar.
    N, K, M = 1024, 256, 256
    W = np.zeros((N, K), np.int8)
    W[np.arange(N), np.arange(N) % K] = 1
    X = np.tile(np.arange(256, dtype=np.uint8)[None, :], (K, 1))     # X[k][m] = m: acc[n][m] = m
    rows = np.arange(N)
    w_scale = np.where(rows < 512, 26.0 / 255.0, 2.0 / 255.0).astype(np.float32)       # wide / fine sweeps
    bias = np.where(rows < 512, -13.0 + (rows % 512) * (26.0 / 255.0 / 512.0),
                    -6.0 + ((rows - 512) // 64) * 1.5 + (rows % 64) * (2.0 / 255.0 / 64.0)).astype(np.float32)
    d = dict(W=W, X=X, w_scale=w_scale, x_scale=1.0, bias=bias, out_scale=1.0, out_zero_point=0, mid_scale=1.0,
             x_zero_point=0)
    case = wl.Case("gelusweep", N, K, M, 0.0, wl.N4K1, "f32", "gelu", keys=(98,))
    got, ok = gpu_spmm(W, X, d, case)
    assert ok
    ref = oracle_spmm(W, X, d, case)
    y = oracle.spmm(W, X, w_scale, 1.0, bias, "none", "f32")
    assert y.min() < -12.9 and y.max() > 12.9 and len(np.unique(y)) > 200_000
    err = np.abs(got.astype(np.float64) - ref.astype(np.float64))
    tol = 1e-5 * np.abs(ref.astype(np.float64)) + 1e-7
    worst = float((err / tol).max())
    assert worst <= 1.0, "worst error / tolerance = %g at y = %g" % (worst, float(y.flat[int((err / tol).argmax())]))
    print("gelu sweep: worst error / tolerance = %.4f" % worst)


# ---------------------------------------------------------------------------- config 5 (sample of the grid)
def _grid_sample():
    allc = wl.grid_cases(out_type="s32")
    picks = [c for c in allc if (c.N, c.K, c.M) in {
        (256, 256, 128), (512, 256, 384), (256, 1024, 1024), (768, 768, 384), (1024, 4096, 128),
        (2048, 512, 384), (3072, 768, 128), (4096, 4096, 128), (768, 3072, 1024), (2048, 2048, 384)}]
    return [c for c in picks if c.sparsity in (0.7, 0.8, 0.9)]


@pytest.mark.parametrize("case", _grid_sample(), ids=lambda c: c.name)
def test_config5_grid_sample_s32_and_s8(case):
    check_case(case)
    check_case(case.with_(out_type="s8"))


@pytest.mark.parametrize("NK", wl.grid_shapes(), ids=lambda nk: "%dx%d" % nk)
def test_config5_whole_grid_at_full_size(NK):
    """Every case of the grid (4 token counts x 5 sparsities per shape, jittered block counts), in the
    launch configuration spmm_run picks: int32 and int8 outputs bit-exact against the oracle, every
    element of both.  On top, the column sums of the int32 output are checked against their closed
    form, sum_n out[n][m] = sum_k (sum_n W[n][k]) X[k][m], in int64."""
    N, K = NK
    for case in [c for c in wl.grid_cases() if (c.N, c.K) == NK]:
        d = wl.make(case)
        W, X = d["W"], d["X"]
        got32, ok32 = gpu_spmm(W, X, d, case)
        case8 = case.with_(out_type="s8")
        d8 = wl.make(case8)
        assert np.array_equal(d8["W"], W) and np.array_equal(d8["X"], X)
        got8, ok8 = gpu_spmm(W, X, d8, case8)
        assert ok32 and ok8, case.name
        acc = oracle.acc_s32(W, X)
        assert np.array_equal(got32, acc), case.name
        colsum = W.sum(axis=0, dtype=np.int64) @ X.astype(np.int64)
        assert np.array_equal(got32.sum(axis=0, dtype=np.int64), colsum), case.name
        ref8 = oracle.epilogue(acc, d8["w_scale"], d8["x_scale"], d8["bias"], "none", "s8",
                               d8["out_scale"], d8["out_zero_point"], d8["mid_scale"])
        assert np.array_equal(got8, ref8), case.name


# ---------------------------------------------------------------------------- edge cases
@pytest.mark.parametrize("N,K,M", [
    (1, 1, 1), (3, 5, 2), (4, 4, 4), (17, 33, 65), (50, 70, 130), (130, 1025, 63), (16, 2049, 100),
    (260, 100, 257), (5, 3000, 7),
])
@pytest.mark.parametrize("out_type", ["s32", "s8"])
@pytest.mark.parametrize("tuning", [None, (128, 16), (128, 8), (96, 16), (128, 112), (128, 108), (96, 112), (64, 112), (64, 102), (32, 101), (16, 101), (16, 103), (32, 103),
                                    (64, 104), (32, 104), (16, 104)],
                         ids=["default", "tile128", "tile128w8", "tile96", "fed12", "fed8", "fed12tile96", "fed12tile64", "simple", "simple32", "simple16", "slab", "slab32",
                              "stream64", "stream32", "stream16"])
def test_ragged_shapes(N, K, M, out_type, tuning):
    case = wl.Case("ragged", N, K, M, 0.6, wl.N4K1, out_type, "none", keys=(60, N, K, M))
    check_case(case, tuning=tuning)
    check_case(case.with_(orientation=wl.N1K4), tuning=tuning)


@pytest.mark.parametrize("N,K,M,s", [(300, 1100, 700, 0.9), (256, 1536, 1300, 0.8), (272, 512, 2100, 0.7),
                                     (64, 3000, 513, 0.5), (1024, 256, 4100, 0.0)])
def test_many_token_tiles_and_segments(N, K, M, s):
    """Several token tiles per workgroup stream, 1 / 2 / 3+ K segments (resident and
    re-streamed weights), ragged last tile, every step-count variant of the kernel."""
    for ot, po in (("s32", "none"), ("s8", "gelu")):
        for tuning in (None, (128, 0), (128, 8), (96, 0), (128, 112), (128, 108), (96, 112), (64, 112)):
            check_case(wl.Case("multi", N, K, M, s, wl.N4K1, ot, po, keys=(66, N, K, M)), tuning=tuning)
    # 4-byte outputs: the plan's own choice there is a workgroup with loader waves
    for ot, po in (("f32", "none"), ("f32", "gelu")):
        check_case(wl.Case("multi", N, K, M, s, wl.N4K1, ot, po, keys=(66, N, K, M)))


@pytest.mark.parametrize("N,K,M,s", [(300, 1100, 701, 0.9), (256, 600, 1299, 0.8), (272, 512, 2103, 0.7),
                                     (1024, 1024, 1531, 0.9), (64, 3000, 517, 0.5)])
def test_ragged_token_count_in_aligned_rows(N, K, M, s):
    """A token count that is not a multiple of 16 in rows whose pitch is: the last tile's cut piece
    is read whole and masked (the bytes between M and the pitch hold 0xEE and must not count), in
    every kernel; outputs beyond M must stay untouched (the guards of gpu_spmm)."""
    ld = (M + 15) // 16 * 16 + 16
    for ot, po in (("s32", "none"), ("s8", "gelu"), ("f32", "none")):
        case = wl.Case("raggedm", N, K, M, s, wl.N4K1, ot, po, keys=(68, N, K, M))
        for tuning in (None, (128, 16), (128, 8), (96, 16), (64, 101), (32, 101), (16, 103), (32, 104)):
            check_case(case, tuning=tuning, ldx=ld, ldo=ld)


@pytest.mark.parametrize("out_type,postop", [("s32", "none"), ("f32", "none"), ("f32", "gelu"),
                                             ("s8", "none"), ("u8", "none"), ("s8", "gelu"), ("u8", "gelu")])
def test_every_epilogue_with_unaligned_leading_dims(out_type, postop):
    case = wl.Case("ep", 70, 300, 90, 0.8, wl.N4K1, out_type, postop, keys=(61, 70, 300, 90),
                   out_zero_point=(3 if postop == "none" and out_type in ("s8", "u8") else 0))
    check_case(case)                                   # aligned, ragged tail
    check_case(case, ldx=101, ldo=93)                  # odd pitches: byte paths
    check_case(case, ldx=112, ldo=96, x_offset=3, out_offset=1)   # misaligned bases
    for tuning in ((128, 0), (64, 101), (32, 101), (16, 101), (16, 103), (32, 103), (64, 104), (16, 104)):   # (the default here is the 16-token simple kernel)
        check_case(case, tuning=tuning)
        check_case(case, ldx=101, ldo=93, tuning=tuning)


@pytest.mark.parametrize("N,K,M,s", [(768, 3072, 32, 0.9), (768, 3072, 128, 0.8), (1024, 4096, 100, 0.9),
                                     (200, 4096, 37, 0.0), (48, 2600, 16, 0.999), (130, 4097, 50, 0.8),
                                     (96, 8192, 33, 0.9)])
def test_short_batches_long_reduction(N, K, M, s):
    """The paper's token counts (32 to 384) on long K: the automatic choice is the short-batch
    kernel (whole K resident in LDS) up to K = 4096 and the 16-token simple kernel beyond; a dense
    weight runs more steps than the three register sets hold at once, a 99.9 % sparse one has
    segments without any step."""
    W = wl.sparse_weight(N, K, s, keys=(97, N, K))
    h = sp.spmm_pack(W)
    try:
        name = sp.spmm_kernel_variant(h, M, "s32", "none")
        assert ("mfma_slab<" in name) == (2048 < K <= 4096), name
        sp.spmm_set_tuning(h, 16, 103)          # forced: longer K still takes the simple kernel
        assert ("mfma_slab<16" in sp.spmm_kernel_variant(h, M, "s32", "none")) == (K <= 4096)
        sp.spmm_set_tuning(h, 32, 103)
        assert ("mfma_slab<32" in sp.spmm_kernel_variant(h, M, "s32", "none")) == (K <= 3072)
        sp.spmm_set_tuning(h, 0, 0)             # mid-size batches: 32-token tiles, resident from five segments on
        assert ("mfma_slab<32" in sp.spmm_kernel_variant(h, 1024, "s32", "none")) == (N >= 768 and 2048 < K <= 3072)
        if K > 4096:                            # seven segments and more without a slab: the streamed kernel
            assert "mfma_stream<16" in sp.spmm_kernel_variant(h, M, "s32", "none")
    finally:
        sp.spmm_destroy(h)
    for ot, po in (("s32", "none"), ("f32", "gelu"), ("s8", "gelu"), ("u8", "none")):
        case = wl.Case("short", N, K, M, s, wl.N4K1, ot, po, keys=(97, N, K, M))
        check_case(case)
        for tm in (16, 32):                     # (32-token tiles hold K <= 3072, else the simple kernel runs)
            check_case(case, tuning=(tm, 103))
            check_case(case, tuning=(tm, 103), ldx=M + 5, ldo=M + 3)      # byte paths
        for tm in (64, 32, 16):                 # the streamed kernel: waves cross segments at their own steps
            check_case(case, tuning=(tm, 104))
        check_case(case, tuning=(32, 104), ldx=M + 5, ldo=M + 3)
    check_case(wl.Case("short", N, K, M, s, wl.N1K4, "s32", "none", keys=(98, N, K, M)), tuning=(16, 103))
    check_case(wl.Case("short", N, K, M, s, wl.N1K4, "s8", "gelu", keys=(98, N, K, M)), tuning=(32, 103))


def test_largest_reduction_length_and_extreme_sums():
    # K = 65536 is the largest reduction the 16-bit segment-local indices of the layout are used
    # with (128 segments); one dense row of +127 and one of -128 against X = 255 reach within 1.2 %
    # of the int32 range, in the signed-activation form the kernel multiplies in as well.
    N, K, M = 20, 65536, 40
    case = wl.Case("maxk", N, K, M, 0.9, wl.N4K1, "s32", "none", keys=(67,))
    d = wl.make(case)
    W = d["W"].copy()
    W[0:4, :] = 127
    W[4:8, :] = -128
    X = d["X"].copy()
    X[:, 0] = 255
    X[:, 1] = 0
    d = dict(d, W=W, X=X)
    got, ok = gpu_spmm(W, X, d, case)
    ref = oracle_spmm(W, X, d, case)
    assert ok and np.array_equal(got, ref)
    assert int(ref[0, 0]) == 65536 * 127 * 255 and int(ref[4, 0]) == -65536 * 128 * 255
    case8 = case.with_(out_type="s8", postop="gelu")
    d8 = dict(wl.make(case8), W=W, X=X)
    got, ok = gpu_spmm(W, X, d8, case8)
    assert ok and np.array_equal(got, oracle_spmm(W, X, d8, case8))
    h = None
    try:
        with pytest.raises(sp.SpmmError):
            h = sp.spmm_pack(np.zeros((4, 65537), np.int8))
    finally:
        sp.spmm_destroy(h)


def test_without_bias_and_with_activation_zero_point():
    case = wl.Case("nobias", 64, 256, 128, 0.8, wl.N4K1, "f32", "none", with_bias=False, keys=(62,))
    check_case(case)
    case = wl.Case("xzp", 64, 256, 128, 0.8, wl.N4K1, "s32", "none", x_zero_point=37, keys=(63,))
    check_case(case)
    check_case(case.with_(out_type="s8", x_zero_point=128))


def test_degenerate_weights():
    K, M = 128, 96
    X = wl.activations(K, M, keys=(64,))
    case = wl.Case("deg", 32, K, M, 0.0, wl.N4K1, "f32", "none", keys=(64,))
    d = wl.make(case)
    # all-zero W: bias only
    d["W"] = np.zeros((32, K), np.int8)
    got, ok = gpu_spmm(d["W"], X, d, case)
    assert ok and np.array_equal(got, np.repeat(d["bias"][:, None], M, axis=1))
    # empty block-rows next to fully dense rows, extreme values
    W = np.zeros((32, K), np.int8)
    W[4:8] = -128
    W[12:16] = 127
    W[20] = 1
    d["W"] = W
    Xmax = np.full((K, M), 255, np.uint8)
    for c in (case.with_(out_type="s32"), case.with_(out_type="s8")):
        got, ok = gpu_spmm(W, Xmax, d, c)
        assert ok
        assert_parity(got, oracle_spmm(W, Xmax, d, c), c)
    got, _ = gpu_spmm(W, Xmax, d, case.with_(out_type="s32"))
    assert got[4, 0] == -128 * 255 * K and got[12, 0] == 127 * 255 * K and got[0, 0] == 0


def test_saturation_and_rounding_pins_on_device():
    # acc = 1 * x with w_scale 0.5: y = x / 2 hits every .5 tie; out_scale 1
    K, M = 4, 256
    W = np.zeros((4, K), np.int8)
    W[0, 0] = 1
    W[1, 0] = -1
    W[2, 0] = 3
    X = np.zeros((K, M), np.uint8)
    X[0] = np.arange(256)
    d = dict(w_scale=np.full(4, 0.5, np.float32), bias=None, x_scale=1.0, x_zero_point=0,
             mid_scale=1.0, out_scale=1.0, out_zero_point=0)
    for ot in ("s8", "u8"):
        case = wl.Case("pins", 4, K, M, 0.0, wl.N4K1, ot, "none", with_bias=False)
        got, ok = gpu_spmm(W, X, d, case)
        assert ok
        assert_parity(got, oracle_spmm(W, X, d, case), case)
    got, _ = gpu_spmm(W, X, d, wl.Case("pins", 4, K, M, 0.0, wl.N4K1, "s8", "none", with_bias=False))
    assert got[0, 1] == 0 and got[0, 3] == 2 and got[0, 5] == 2 and got[0, 7] == 4      # ties to even
    assert got[1, 3] == -2 and got[1, 5] == -2 and got[2, 255] == 127 and got[1, 255] == -128


def test_non_default_stream_and_repeated_runs():
    case = wl.mini_cases()[1]
    d = wl.make(case)
    ref = oracle_spmm(d["W"], d["X"], d, case)
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        for _ in range(3):
            got, ok = gpu_spmm(d["W"], d["X"], d, case, stream=s)
            assert ok
            assert_parity(got, ref, case)


def test_run_argument_errors_leave_output_untouched():
    W = wl.sparse_weight(32, 64, 0.5, keys=(65,))
    h = sp.spmm_pack(W)
    try:
        X = torch.zeros(64 * 16, dtype=torch.uint8, device="cuda")
        out = torch.full((32 * 16,), 77, dtype=torch.int32, device="cuda")
        ws = torch.ones(32, dtype=torch.float32, device="cuda")
        ok_ep = sp.make_epilogue(ws, 1.0, 0, None, "none", "s32")
        E = sp.SPMM_E_ARG
        assert sp.spmm_run_status(h, None, 16, 16, ok_ep, out, 16) == E
        assert sp.spmm_run_status(h, X, 16, 16, None, out, 16) == E
        assert sp.spmm_run_status(h, X, 16, 16, ok_ep, None, 16) == E
        assert sp.spmm_run_status(h, X, 0, 16, ok_ep, out, 16) == E
        assert sp.spmm_run_status(h, X, 16, 15, ok_ep, out, 16) == E
        assert sp.spmm_run_status(h, X, 16, 16, ok_ep, out, 15) == E
        assert sp.spmm_run_status(None, X, 16, 16, ok_ep, out, 16) == E
        bad = sp.make_epilogue(ws, 1.0, 0, None, "none", "s32"); bad.out_type = 9
        assert sp.spmm_run_status(h, X, 16, 16, bad, out, 16) == E
        bad = sp.make_epilogue(ws, 1.0, 0, None, "none", "s32"); bad.postop = 5
        assert sp.spmm_run_status(h, X, 16, 16, bad, out, 16) == E
        assert sp.spmm_run_status(h, X, 16, 16, sp.make_epilogue(None, 1.0, 0, None, "none", "f32"), out, 16) == E
        assert sp.spmm_run_status(h, X, 16, 16, sp.make_epilogue(ws, 1.0, 0, None, "gelu", "s8", 1.0, 0, 1.0, None), out, 16) == E
        assert sp.spmm_run_status(h, X, 16, 16, sp.make_epilogue(ws, 1.0, 0, None, "none", "s8", 0.0), out, 16) == E
        assert sp.spmm_run_status(h, X, 16, 16, sp.make_epilogue(ws, 1.0, 0, None, "none", "s8", 1.0, 200), out, 16) == E
        assert sp.spmm_run_status(h, X, 16, 16, sp.make_epilogue(ws, 1.0, 300, None, "none", "s32"), out, 16) == E
        torch.cuda.synchronize()
        assert (out == 77).all()
        assert sp.spmm_run_status(h, X, 16, 16, ok_ep, out, 16) == sp.SPMM_OK
        torch.cuda.synchronize()
        assert (out == 0).all()
    finally:
        sp.spmm_destroy(h)


def test_info_reports_device_bytes_and_plan():
    W = wl.make(wl.large_cases()[0])["W"]
    h = sp.spmm_pack(W)
    try:
        N, K, nnzb, padded, dev_bytes = sp.spmm_info(h)
        steps = sp.spmm_layout_dims(h)[5]
        assert dev_bytes >= steps * (1024 + 128) and padded == steps * 256
        tm, rows, wgs = sp.spmm_plan(h, 6144, "s8")
        assert tm > 0 and rows % 16 == 0 and wgs * tm * rows >= 6144 * N
    finally:
        sp.spmm_destroy(h)


# ------------------------------------------------ offline row ordering (Section 3.2)
@pytest.mark.parametrize("orient,N,K,M,s,clusters,out_type,postop", [
    (wl.N4K1, 512, 1024, 700, 0.9, 8, "s8", "gelu"), (wl.N4K1, 1024, 1024, 1536, 0.8, 16, "f32", "none"),
    (wl.N4K1, 130, 600, 333, 0.8, 3, "s32", "none"), (wl.N1K4, 256, 1024, 384, 0.9, 4, "u8", "none"),
    (wl.N4K1, 768, 3072, 32, 0.9, 6, "f32", "gelu")])
def test_reordered_rows_are_the_oracles_rows_in_the_reported_order(orient, N, K, M, s, clusters, out_type, postop):
    """A weight packed with SPMM_PACK_REORDER_ROWS computes the rows of the product in the order
    spmm_row_order reports, with the per-row operands read in that order."""
    case = wl.Case("reordered", N, K, M, s, orient, out_type, postop, jitter=0.2, keys=(81, N, K, M), clusters=clusters)
    d = wl.make(case)
    ref = oracle_spmm(d["W"], d["X"], d, case)
    h = sp.spmm_pack_ex(d["W"], orient, reorder_rows=True)
    try:
        order = sp.spmm_row_order(h)
        assert sorted(order.tolist()) == list(range(N))
        lut = None
        if postop == "gelu" and out_type in ("s8", "u8"):
            lut = dev(sp.spmm_make_gelu_lut(d["mid_scale"], d["out_scale"], d["out_zero_point"], out_type))
        ep = sp.make_epilogue(dev(d["w_scale"][order]), d["x_scale"], d["x_zero_point"], dev(d["bias"][order]), postop,
                              out_type, d["out_scale"], d["out_zero_point"], d["mid_scale"], lut)
        out = torch.zeros((N, M), dtype=TORCH_DT[out_type], device="cuda")
        sp.spmm_run(h, dev(d["X"]), M, M, ep, out, M, torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        assert_parity(out.cpu().numpy(), np.ascontiguousarray(ref[order]), case)
    finally:
        sp.spmm_destroy(h)


# ------------------------------------------------ token-tile-major activations (Section 3.2: re-structured input)
@pytest.mark.parametrize("tuning", [None, (128, 16), (128, 8), (96, 16), (128, 112), (128, 108), (96, 112), (64, 112), (64, 101),
                                    (64, 102), (32, 101), (16, 101), (16, 103), (32, 103), (64, 104), (32, 104), (16, 104)],
                         ids=lambda t: "auto" if t is None else "%d_%d" % t)
@pytest.mark.parametrize("N,K,M,s,out_type,postop", [(272, 1100, 700, 0.9, "s8", "gelu"), (100, 600, 333, 0.8, "s32", "none"),
                                                      (512, 2048, 1280, 0.9, "f32", "none"), (64, 520, 50, 0.7, "u8", "none")])
def test_tile_major_activations(N, K, M, s, out_type, postop, tuning):
    """spmm_run_tiled reads X as [ceil(M / 32)][K][32]: same results as the oracle on the row-major X,
    in every kernel family, with ragged token counts (the padding of the last tile is poisoned)."""
    case = wl.Case("xtiled", N, K, M, s, wl.N4K1, out_type, postop, keys=(83, N, K, M))
    check_case(case, tuning=tuning, x_tiled=True)


def test_tile_major_large_case_and_argument_errors():
    case = wl.large_cases()[4]                                   # 1024 x 4096, 6144 tokens: eight K segments, 96-token tiles
    check_case(case, x_tiled=True)
    d = wl.make(wl.tiny_cases()[0])
    h = sp.spmm_pack(d["W"])
    try:
        ep = sp.make_epilogue(None, 1.0, 0, None, "none", "s32", 1.0, 0, 1.0, None)
        Xt = dev(sp.tile_major(d["X"]))
        out = torch.zeros((256, 128), dtype=torch.int32, device="cuda")
        shifted = torch.zeros(Xt.numel() + 16, dtype=torch.uint8, device="cuda")[1:]
        with pytest.raises(sp.SpmmError):                        # activations must be 16-byte aligned
            sp.spmm_run_tiled(h, shifted, 100, 0, ep, out, 128, sp.binding.SPMM_TILED_X, None)
        with pytest.raises(ValueError):                          # ... and large enough (checked by the binding)
            sp.spmm_run_tiled(h, Xt.view(-1)[16:], 100, 0, ep, out, 128, sp.binding.SPMM_TILED_X, None)
    finally:
        sp.spmm_destroy(h)


def _run_tiled_out(d, case, tuning, x_tiled):
    """1-byte output written token-tile-major into an exactly sized, guarded buffer; returned row-major."""
    W, X = d["W"], d["X"]
    N, K = W.shape
    M = X.shape[1]
    ot = case.out_type
    h = sp.spmm_pack(W, case.orientation)
    try:
        if tuning:
            sp.spmm_set_tuning(h, *tuning)
        tiles = (M + 31) // 32
        obuf = torch.full((tiles * N * 32 + 2 * GUARD,), POISON[ot], dtype=TORCH_DT[ot], device="cuda")
        oview = obuf[GUARD:GUARD + tiles * N * 32]
        lut = None
        if case.postop == "gelu":
            lut = dev(sp.spmm_make_gelu_lut(d["mid_scale"], d["out_scale"], d["out_zero_point"], ot))
        ep = sp.make_epilogue(dev(d["w_scale"]), d["x_scale"], d["x_zero_point"], dev(d["bias"]), case.postop, ot,
                              d["out_scale"], d["out_zero_point"], d["mid_scale"], lut)
        Xd = dev(sp.tile_major(X)) if x_tiled else dev(X)
        flags = sp.binding.SPMM_TILED_OUT | (sp.binding.SPMM_TILED_X if x_tiled else 0)
        sp.spmm_run_tiled(h, Xd, M, M, ep, oview, 0, flags, torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        full = obuf.cpu().numpy()
        poison = np.array(POISON[ot]).astype(full.dtype)
        assert (full[:GUARD] == poison).all() and (full[GUARD + tiles * N * 32:] == poison).all()
        T = full[GUARD:GUARD + tiles * N * 32].reshape(tiles, N, 32)
        if M % 32:
            assert (T[-1, :, M % 32:] == poison).all()          # the padding of the last tile is not written
        return sp.from_tile_major(T, M)
    finally:
        sp.spmm_destroy(h)


@pytest.mark.parametrize("tuning", [None, (128, 16), (128, 8), (96, 16), (128, 112), (128, 108), (64, 112), (64, 101), (32, 101),
                                    (16, 101), (16, 103), (32, 103), (64, 104), (16, 104)],
                         ids=lambda t: "auto" if t is None else "%d_%d" % t)
@pytest.mark.parametrize("N,K,M,s,out_type,postop,x_tiled", [(272, 1100, 704, 0.9, "s8", "gelu", True), (100, 600, 333, 0.8, "u8", "none", False),
                                                              (512, 1536, 1280, 0.8, "s8", "none", True), (64, 520, 50, 0.7, "u8", "gelu", True)])
def test_tile_major_output(N, K, M, s, out_type, postop, x_tiled, tuning):
    """SPMM_TILED_OUT writes the 1-byte output as the next layer's tile-major activations: same values as the
    oracle's row-major output, nothing outside the tiles, in every kernel family."""
    case = wl.Case("otiled", N, K, M, s, wl.N4K1, out_type, postop, keys=(84, N, K, M))
    d = wl.make(case)
    got = _run_tiled_out(d, case, tuning, x_tiled)
    assert_parity(got, oracle_spmm(d["W"], d["X"], d, case), case)


@pytest.mark.parametrize("large", [False, True])
def test_chained_ffn_pair_in_tile_major_order(large):
    """The chained pair of Section 3.3 with every activation tile-major: layer 1 reads tile-major X and writes its
    u8 code tile-major, layer 2 reads that buffer as is; both bit-equal to the oracle chained the same way.
    large: at the feed-forward shapes and token count of BERT-Large (the pipelined kernels, whose tile-major
    1-byte stores go out at agent scope, feeding each other)."""
    c1, c2 = wl.chain_cases(large=large)
    d1, d2 = wl.make_chain([c1, c2])
    M = c1.M
    ref1 = oracle_spmm(d1["W"], d1["X"], d1, c1)
    ref2 = oracle_spmm(d2["W"], ref1, d2, c2)
    h1, h2 = sp.spmm_pack(d1["W"]), sp.spmm_pack(d2["W"])
    try:
        st = torch.cuda.current_stream().cuda_stream
        lut = dev(sp.spmm_make_gelu_lut(d1["mid_scale"], d1["out_scale"], d1["out_zero_point"], "u8"))
        ep1 = sp.make_epilogue(dev(d1["w_scale"]), d1["x_scale"], 0, dev(d1["bias"]), "gelu", "u8", d1["out_scale"],
                               d1["out_zero_point"], d1["mid_scale"], lut)
        ep2 = sp.make_epilogue(dev(d2["w_scale"]), d2["x_scale"], d2["x_zero_point"], dev(d2["bias"]), "none", "s8",
                               d2["out_scale"], 0, d2["mid_scale"], None)
        hid = torch.zeros(((M + 31) // 32) * c1.N * 32, dtype=torch.uint8, device="cuda")
        out = torch.zeros((c2.N, M), dtype=torch.int8, device="cuda")
        both = sp.binding.SPMM_TILED_X | sp.binding.SPMM_TILED_OUT
        sp.spmm_run_tiled(h1, dev(sp.tile_major(d1["X"])), M, 0, ep1, hid, 0, both, st)
        sp.spmm_run_tiled(h2, hid, M, 0, ep2, out, M, sp.binding.SPMM_TILED_X, st)
        torch.cuda.synchronize()
        got1 = sp.from_tile_major(hid.cpu().numpy().reshape(-1, c1.N, 32), M)
        assert np.array_equal(got1, ref1)
        assert np.array_equal(out.cpu().numpy(), ref2)
        with pytest.raises(sp.SpmmError):                        # 4-byte outputs have no tile-major form
            ep3 = sp.make_epilogue(dev(d2["w_scale"]), d2["x_scale"], 0, None, "none", "f32", 1.0, 0, 1.0, None)
            sp.spmm_run_tiled(h2, hid, M, 0, ep3, torch.zeros((c2.N, M), dtype=torch.float32, device="cuda"), M, both, st)
    finally:
        sp.spmm_destroy(h1)
        sp.spmm_destroy(h2)
