"""Pins for the CPU oracle: everything here checks `oracle/` against something
other than itself -- a library routine, Python big-integer / rational
arithmetic, arbitrary-precision erfc, closed forms, invariants and hand-worked
fixtures -- so that a dropped term, a wrong sign or index, a transposed operand
or a wrong rounding rule fails at least one test.  CPU only.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------------------
# helpers that are independent of the oracle's C code
# ----------------------------------------------------------------------------
def f32_round(fr: Fraction) -> float:
    """Round an exact rational to the nearest binary32 (ties to even); normal range only."""
    if fr == 0:
        return 0.0
    sign = -1 if fr < 0 else 1
    a = abs(fr)
    e = math.floor(math.log2(a))
    # fix possible off-by-one of floating log2
    while Fraction(2) ** e > a:
        e -= 1
    while Fraction(2) ** (e + 1) <= a:
        e += 1
    assert -126 <= e <= 127
    scaled = a / (Fraction(2) ** (e - 23))          # in [2^23, 2^24)
    q, r = divmod(scaled.numerator, scaled.denominator)
    twice = 2 * r
    if twice > scaled.denominator or (twice == scaled.denominator and (q & 1)):
        q += 1
    return sign * float(Fraction(q) * Fraction(2) ** (e - 23))


def py_round_half_even(v: float) -> int:
    """Python's round() on a float is exact round-half-to-even."""
    return int(round(v))


def load_table(name):
    rows = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                rows.append(line.split())
    return rows


# ----------------------------------------------------------------------------
# O1: the int32 accumulator
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("N,K,M", [(1, 1, 1), (3, 5, 2), (8, 8, 4), (5, 7, 3)])
def test_acc_bruteforce_bigint(N, K, M):
    rng = np.random.default_rng(N * 100 + K * 10 + M)
    W = rng.integers(-128, 128, size=(N, K), dtype=np.int8)
    X = rng.integers(0, 256, size=(K, M), dtype=np.uint8)
    for zp in (0, 3, 128):
        got = oracle.acc_s32(W, X, zp)
        for n in range(N):
            for m in range(M):
                ref = sum(int(W[n, k]) * (int(X[k, m]) - zp) for k in range(K))
                assert int(got[n, m]) == ref


def test_acc_exhaustive_two_block_patterns():
    """One block-row (4 rows), K = 6: every placement of two 4x1 blocks."""
    rng = np.random.default_rng(7)
    K, M = 6, 3
    X = rng.integers(0, 256, size=(K, M), dtype=np.uint8)
    for k0 in range(K):
        for k1 in range(k0 + 1, K):
            W = np.zeros((4, K), dtype=np.int8)
            W[:, k0] = rng.integers(-127, 128, size=4)
            W[:, k1] = rng.integers(-127, 128, size=4)
            got = oracle.acc_s32(W, X)
            for n in range(4):
                for m in range(M):
                    ref = int(W[n, k0]) * int(X[k0, m]) + int(W[n, k1]) * int(X[k1, m])
                    assert int(got[n, m]) == ref


def _small_cases():
    cases = wl.tiny_cases(wl.N4K1) + wl.tiny_cases(wl.N1K4) + wl.mini_cases(wl.N4K1)
    cases += [c for c in wl.base_cases(batches=(1,), sparsities=(0.7, 0.9)) if c.N == 768 and c.K == 768]
    return cases


@pytest.mark.parametrize("case", _small_cases(), ids=lambda c: c.name + "_" + c.orientation)
def test_acc_equals_library_matmul(case):
    d = wl.make(case)
    ref = d["W"].astype(np.int64) @ d["X"].astype(np.int64)
    assert np.abs(ref).max() < 2 ** 31
    got = oracle.acc_s32(d["W"], d["X"])
    assert got.dtype == np.int32
    assert np.array_equal(got.astype(np.int64), ref)


def test_acc_strided_inputs():
    rng = np.random.default_rng(11)
    Wbig = rng.integers(-128, 128, size=(9, 20), dtype=np.int8)
    Xbig = rng.integers(0, 256, size=(13, 17), dtype=np.uint8)
    W, X = Wbig[:, :13], Xbig[:, :11]          # ldw = 20, ldx = 17
    ref = W.astype(np.int64) @ X.astype(np.int64)
    assert np.array_equal(oracle.acc_s32(W, X).astype(np.int64), ref)


def test_acc_extreme_values_fit_int32():
    K = 4096
    W = np.full((2, K), -128, dtype=np.int8)
    W[1, :] = 127
    X = np.full((K, 2), 255, dtype=np.uint8)
    got = oracle.acc_s32(W, X)
    assert got[0, 0] == -128 * 255 * K and got[1, 1] == 127 * 255 * K


def test_acc_special_cases():
    rng = np.random.default_rng(3)
    N, K, M = 12, 32, 9
    X = rng.integers(0, 256, size=(K, M), dtype=np.uint8)
    # W = 0
    assert not oracle.acc_s32(np.zeros((N, K), np.int8), X).any()
    # single 1 at k -> row k of X ; single -1 -> minus row
    W = np.zeros((N, K), np.int8)
    for n in range(N):
        W[n, (5 * n + 1) % K] = 1 if n % 2 == 0 else -1
    got = oracle.acc_s32(W, X)
    for n in range(N):
        row = X[(5 * n + 1) % K].astype(np.int32)
        assert np.array_equal(got[n], row if n % 2 == 0 else -row)
    # all ones -> column sums
    got = oracle.acc_s32(np.ones((N, K), np.int8), X)
    assert np.array_equal(got[0], X.astype(np.int32).sum(axis=0))
    # X = 0 and X = 128
    W = rng.integers(-128, 128, size=(N, K), dtype=np.int8)
    assert not oracle.acc_s32(W, np.zeros((K, M), np.uint8)).any()
    got = oracle.acc_s32(W, np.full((K, M), 128, np.uint8))
    assert np.array_equal(got, np.repeat(128 * W.astype(np.int32).sum(axis=1)[:, None], M, axis=1))
    # zero point: acc(X, zp) = acc(X, 0) - zp * rowsum
    got = oracle.acc_s32(W, X, 17)
    ref = oracle.acc_s32(W, X, 0) - 17 * W.astype(np.int32).sum(axis=1)[:, None]
    assert np.array_equal(got, ref)


def test_acc_invariants():
    rng = np.random.default_rng(5)
    N, K, M = 16, 40, 11
    W = wl.sparse_weight(N, K, 0.8, wl.N4K1, keys=(99, 1))
    X1 = rng.integers(0, 128, size=(K, M), dtype=np.uint8)
    X2 = rng.integers(0, 128, size=(K, M), dtype=np.uint8)
    a1, a2 = oracle.acc_s32(W, X1), oracle.acc_s32(W, X2)
    # linearity in X
    assert np.array_equal(oracle.acc_s32(W, (X1 + X2).astype(np.uint8)), a1 + a2)
    assert np.array_equal(oracle.acc_s32(W, (2 * X1).astype(np.uint8)), 2 * a1)
    # additivity in W over disjoint supports
    Wa, Wb = W.copy(), W.copy()
    Wa[:, ::2] = 0
    Wb[:, 1::2] = 0
    assert np.array_equal(oracle.acc_s32(Wa, X1) + oracle.acc_s32(Wb, X1), a1)
    # permuting k consistently leaves the result unchanged
    p = rng.permutation(K)
    assert np.array_equal(oracle.acc_s32(np.ascontiguousarray(W[:, p]), np.ascontiguousarray(X1[p])), a1)
    # permuting rows of W permutes rows of out; permuting tokens permutes columns
    r = rng.permutation(N)
    assert np.array_equal(oracle.acc_s32(np.ascontiguousarray(W[r]), X1), a1[r])
    c = rng.permutation(M)
    assert np.array_equal(oracle.acc_s32(W, np.ascontiguousarray(X1[:, c])), a1[:, c])
    # a transposed-operand mistake would break this asymmetric case
    W2 = np.array([[1, 2], [3, 4]], np.int8)
    X3 = np.array([[5, 6], [7, 8]], np.uint8)
    assert oracle.acc_s32(W2, X3).tolist() == [[19, 22], [43, 50]]


# ----------------------------------------------------------------------------
# O2: dequantise + bias, one fused binary32 operation
# ----------------------------------------------------------------------------
def test_dequant_bias_is_single_rounding_fma():
    rng = np.random.default_rng(17)
    N, M = 64, 33
    acc = rng.integers(-3_000_000, 3_000_000, size=(N, M), dtype=np.int32)
    acc[0, :4] = [0, 1, -1, 2 ** 24 + 1]          # int->float conversion must round (RNE)
    acc[1, :2] = [2 ** 31 - 1, -2 ** 31]
    w_scale = rng.uniform(1e-3, 1e-2, size=N).astype(np.float32)
    bias = rng.standard_normal(N).astype(np.float32)
    x_scale = np.float32(0.02)
    got = oracle.epilogue(acc, w_scale, x_scale, bias, "none", "f32")
    n_diff_unfused = 0
    for n in range(N):
        s = np.float32(w_scale[n]) * x_scale                      # one binary32 multiply
        s_exact = f32_round(Fraction(float(w_scale[n])) * Fraction(float(x_scale)))
        assert float(s) == s_exact
        for m in range(M):
            a_f32 = f32_round(Fraction(int(acc[n, m])))           # int32 -> binary32, RNE
            y = f32_round(Fraction(a_f32) * Fraction(s_exact) + Fraction(float(bias[n])))
            assert float(got[n, m]) == y, (n, m)
            unfused = np.float32(np.float32(a_f32) * s) + bias[n]
            n_diff_unfused += int(float(unfused) != y)
    # the pin is only meaningful if fused and unfused differ somewhere in the sample
    assert n_diff_unfused > 0


def test_no_bias_means_zero_bias():
    acc = np.arange(-8, 8, dtype=np.int32).reshape(4, 4)
    w = np.array([0.5, 0.25, 2.0, 1.0], np.float32)
    got = oracle.epilogue(acc, w, 2.0, None, "none", "f32")
    assert np.array_equal(got, acc.astype(np.float32) * (w * np.float32(2.0))[:, None])


def test_s32_output_ignores_epilogue_parameters():
    d = wl.make(wl.tiny_cases()[0])
    a = oracle.spmm(d["W"], d["X"], out_type="s32")
    b = oracle.spmm(d["W"], d["X"], d["w_scale"], 0.5, d["bias"], "gelu", "s32", 3.0, 7, 2.0)
    assert np.array_equal(a, b)


# ----------------------------------------------------------------------------
# O3: GELU
# ----------------------------------------------------------------------------
def test_gelu_textbook_normal_cdf_values():
    for xs, ps in load_table("normal_cdf.txt"):
        x, phi = float(xs), float(ps)
        assert oracle.gelu(x) == pytest.approx(x * phi, rel=2e-15, abs=1e-300)


def test_gelu_against_arbitrary_precision_erfc():
    mpmath = pytest.importorskip("mpmath")
    mpmath.mp.dps = 60
    for x in np.concatenate([np.linspace(-12, 12, 241), [-30.0, -20.0, 1e-3, -1e-3, 37.5]]):
        ref = mpmath.mpf(float(x)) * mpmath.erfc(-mpmath.mpf(float(x)) / mpmath.sqrt(2)) / 2
        got = oracle.gelu(float(x))
        if ref == 0:
            assert got == 0
        else:
            # erfc's condition number ~2 z^2 amplifies the rounding of -x/sqrt(2) in the far tail
            rel = 1e-13 if abs(x) <= 12 else 1e-12
            assert abs((mpmath.mpf(got) - ref) / ref) < rel, x


def test_gelu_closed_form_properties():
    g = oracle.gelu
    assert g(0.0) == 0.0
    for y in (0.1, 0.75, 1.0, 2.5, 5.0, 9.0):
        assert g(y) - g(-y) == pytest.approx(y, rel=1e-15)          # x*Phi(x) + x*Phi(-x) = x
    for y in (8.5, 10.0, 40.0):
        assert g(y) == pytest.approx(y, rel=1e-15)
        assert -1e-14 < g(-y) <= 0.0
    xs = np.linspace(-3, 1, 4001)
    vals = np.array([g(float(x)) for x in xs])
    i = int(vals.argmin())
    assert xs[i] == pytest.approx(-0.7518, abs=2e-3) and vals[i] == pytest.approx(-0.16997, abs=1e-4)
    assert np.all(np.diff(vals[i:]) > 0) and np.all(np.diff(vals[: i + 1]) < 0)
    # independent library erf in the well-conditioned range
    for x in np.linspace(-3, 6, 91):
        assert g(float(x)) == pytest.approx(0.5 * x * (1.0 + math.erf(x / math.sqrt(2.0))), rel=1e-11, abs=1e-15)


def test_gelu_f32_output_is_rounded_double_gelu():
    mpmath = pytest.importorskip("mpmath")
    mpmath.mp.dps = 50
    acc = np.array([[-90000, -40000, -5000, -100, 0, 100, 5000, 40000, 90000]], np.int32)
    w = np.array([0.0078125], np.float32)
    b = np.array([0.25], np.float32)
    got = oracle.epilogue(acc, w, 0.015625, b, "gelu", "f32")
    for m in range(acc.shape[1]):
        y = float(acc[0, m]) * 0.0078125 * 0.015625 + 0.25          # exact in binary32
        ref = mpmath.mpf(y) * mpmath.erfc(-mpmath.mpf(y) / mpmath.sqrt(2)) / 2
        assert float(got[0, m]) == pytest.approx(float(ref), rel=2e-7, abs=1e-45)


# ----------------------------------------------------------------------------
# O4: Quantize (round half to even, saturate) and the lookup table
# ----------------------------------------------------------------------------
def test_rounding_pins_fixture():
    for acc, ws, xs, b, os_, zp, ot, exp in load_table("rounding_pins.txt"):
        a = np.array([[int(acc)]], np.int32)
        got = oracle.epilogue(a, np.array([float(ws)], np.float32), float(xs),
                              np.array([float(b)], np.float32), "none", ot, float(os_), int(zp))
        assert int(got[0, 0]) == int(exp), (acc, ws, xs, b, os_, zp, ot)


@pytest.mark.parametrize("out_type,lo,hi", [("s8", -128, 127), ("u8", 0, 255)])
def test_quantize_against_python_rounding(out_type, lo, hi):
    rng = np.random.default_rng(23)
    N, M = 32, 64
    acc = rng.integers(-400_000, 400_000, size=(N, M), dtype=np.int32)
    w_scale = rng.uniform(1e-3, 1e-2, size=N).astype(np.float32)
    bias = rng.standard_normal(N).astype(np.float32)
    out_scale, zp = np.float32(0.0731), 5
    y = oracle.epilogue(acc, w_scale, 0.02, bias, "none", "f32")      # pinned above
    got = oracle.epilogue(acc, w_scale, 0.02, bias, "none", out_type, out_scale, zp)
    inv = np.float32(1.0) / out_scale
    assert float(inv) == f32_round(Fraction(1) / Fraction(float(out_scale)))
    for n in range(N):
        for m in range(M):
            t = float(np.float32(y[n, m]) * inv)                      # one binary32 multiply
            assert t == f32_round(Fraction(float(y[n, m])) * Fraction(float(inv)))
            q = min(hi, max(lo, py_round_half_even(t) + zp))
            assert int(got[n, m]) == q


def _mp_gelu_lut(mid_scale, out_scale, zp, lo, hi):
    import mpmath
    mpmath.mp.dps = 60
    out = []
    for i in range(-128, 128):
        x = mpmath.mpf(i) * mpmath.mpf(float(np.float32(mid_scale)))
        v = x * mpmath.erfc(-x / mpmath.sqrt(2)) / 2
        t = v / mpmath.mpf(float(np.float32(out_scale)))
        fl = mpmath.floor(t)
        frac = t - fl
        if frac > mpmath.mpf(1) / 2 or (frac == mpmath.mpf(1) / 2 and int(fl) % 2 == 1):
            q = int(fl) + 1
        else:
            q = int(fl)
        out.append(min(hi, max(lo, q + zp)))
    return out


@pytest.mark.parametrize("mid,outs,zp,ot", [
    (0.1, 0.1, 0, "s8"), (0.42, 0.42, 0, "s8"), (0.05, 0.02, -100, "s8"),
    (0.3, 0.15, 4, "u8"), (0.033, 0.0165, 0, "u8"), (1.0, 1.0, 0, "s8"),
])
def test_gelu_lut_all_256_entries_recomputed(mid, outs, zp, ot):
    pytest.importorskip("mpmath")
    lo, hi = (-128, 127) if ot == "s8" else (0, 255)
    lut = oracle.gelu_lut(mid, outs, zp, ot)
    assert lut.shape == (256,)
    assert [int(v) for v in lut] == _mp_gelu_lut(mid, outs, zp, lo, hi)


def test_gelu_lut_structure():
    lut = oracle.gelu_lut(1.0, 1.0, 0, "s8")
    # GELU(i) for integer i: 0 at i <= 0 rounds to 0 (|GELU| < 0.17), ~i for i >= 1
    assert all(int(lut[i + 128]) == 0 for i in range(-128, 1))
    assert int(lut[1 + 128]) == 1 and int(lut[2 + 128]) == 2 and int(lut[127 + 128]) == 127
    with pytest.raises(ValueError):
        oracle.gelu_lut(1.0, 1.0, 0, "f32")


def test_gelu_int8_path_is_quantise_then_table():
    rng = np.random.default_rng(29)
    N, M = 16, 48
    acc = rng.integers(-300_000, 300_000, size=(N, M), dtype=np.int32)
    w_scale = rng.uniform(1e-3, 1e-2, size=N).astype(np.float32)
    bias = rng.standard_normal(N).astype(np.float32)
    mid, outs = np.float32(0.21), np.float32(0.19)
    lut = oracle.gelu_lut(mid, outs, 0, "s8")
    y = oracle.epilogue(acc, w_scale, 0.02, bias, "none", "f32")
    got = oracle.epilogue(acc, w_scale, 0.02, bias, "gelu", "s8", outs, 0, mid, lut)
    inv = np.float32(1.0) / mid
    for n in range(N):
        for m in range(M):
            t = min(127, max(-128, py_round_half_even(float(np.float32(y[n, m]) * inv))))
            assert int(got[n, m]) == int(lut[t + 128])
    assert (got == 127).any() or (np.abs(y).max() < 127 * mid)       # saturation exercised or impossible
    # the same chain through spmm() builds the table itself
    W = wl.sparse_weight(N, 32, 0.75, keys=(98,))
    X = wl.activations(32, M, keys=(98,))
    a = oracle.acc_s32(W, X)
    full = oracle.spmm(W, X, w_scale, 0.02, bias, "gelu", "s8", outs, 0, mid)
    assert np.array_equal(full, oracle.epilogue(a, w_scale, 0.02, bias, "gelu", "s8", outs, 0, mid, lut))
    # a caller's table of some other chain goes through the same look-up ("table" post-operator)
    other = rng.integers(-128, 128, size=256).astype(np.int8)
    got = oracle.epilogue(acc, w_scale, 0.02, bias, "table", "s8", outs, 0, mid, other)
    for n in range(N):
        for m in range(M):
            t = min(127, max(-128, py_round_half_even(float(np.float32(y[n, m]) * inv))))
            assert int(got[n, m]) == int(other[t + 128])
    with pytest.raises(ValueError):      # a table yields low-precision codes only
        oracle.epilogue(acc, w_scale, 0.02, bias, "table", "f32", outs, 0, mid, other)
    with pytest.raises(ValueError):
        oracle.epilogue(acc, w_scale, 0.02, bias, "table", "s8", outs, 0, mid, None)


# ----------------------------------------------------------------------------
# whole-chain special cases
# ----------------------------------------------------------------------------
def test_zero_weight_gives_bias_only():
    N, K, M = 8, 16, 5
    W = np.zeros((N, K), np.int8)
    X = wl.activations(K, M, keys=(97,))
    w_scale, bias = wl.channel_params(N, keys=(97,))
    assert not oracle.spmm(W, X).any()
    f = oracle.spmm(W, X, w_scale, 0.02, bias, "none", "f32")
    assert np.array_equal(f, np.repeat(bias[:, None], M, axis=1))
    g = oracle.spmm(W, X, w_scale, 0.02, bias, "gelu", "f32")
    for n in range(N):
        assert float(g[n, 0]) == pytest.approx(oracle.gelu(float(bias[n])), rel=1e-7)
    q = oracle.spmm(W, X, w_scale, 0.02, bias, "none", "s8", 0.05, 0)
    inv = np.float32(1.0) / np.float32(0.05)
    for n in range(N):
        assert int(q[n, 0]) == min(127, max(-128, py_round_half_even(float(bias[n] * inv))))


def test_invalid_combinations_raise():
    acc = np.zeros((2, 2), np.int32)
    with pytest.raises(ValueError):
        oracle.epilogue(acc, None, 1.0, None, "none", "f32")
    with pytest.raises(ValueError):
        oracle.epilogue(acc, np.ones(2, np.float32), 1.0, None, "gelu", "s8", 1.0, 0, 1.0, None)


# ----------------------------------------------------------------------------
# Sum post-operator (Figure 3): a second [N, M] binary32 tensor added after BiasAdd / GeLU and
# before Quantize, one correctly rounded binary32 add
# ----------------------------------------------------------------------------
def _sum_inputs(seed=31, N=24, M=19):
    rng = np.random.default_rng(seed)
    acc = rng.integers(-2_000_000, 2_000_000, size=(N, M), dtype=np.int32)
    w_scale = rng.uniform(1e-3, 1e-2, size=N).astype(np.float32)
    bias = rng.standard_normal(N).astype(np.float32)
    R = (rng.standard_normal((N, M)) * 37.0).astype(np.float32)
    return acc, w_scale, bias, R


def test_sum_is_one_rounded_add_after_bias():
    acc, w_scale, bias, R = _sum_inputs()
    y = oracle.epilogue(acc, w_scale, 0.02, bias, "none", "f32")          # pinned above
    got = oracle.epilogue(acc, w_scale, 0.02, bias, "none", "f32", sum=R)
    n_inexact = 0
    for n in range(acc.shape[0]):
        for m in range(acc.shape[1]):
            exact = Fraction(float(y[n, m])) + Fraction(float(R[n, m]))
            assert float(got[n, m]) == f32_round(exact), (n, m)
            n_inexact += int(Fraction(float(got[n, m])) != exact)
    assert n_inexact > 0                       # the add really rounds somewhere in the sample
    # the residual is indexed [n][m]: a transposed read would change this asymmetric case
    acc2 = np.zeros((2, 3), np.int32)
    R2 = np.arange(6, dtype=np.float32).reshape(2, 3)
    out = oracle.epilogue(acc2, np.ones(2, np.float32), 1.0, None, "none", "f32", sum=R2)
    assert np.array_equal(out, R2)


def test_sum_of_zeros_changes_nothing():
    acc, w_scale, bias, R = _sum_inputs(32)
    Z = np.zeros_like(R)
    for post, ot in (("none", "f32"), ("gelu", "f32"), ("none", "s8"), ("none", "u8")):
        a = oracle.epilogue(acc, w_scale, 0.02, bias, post, ot, 0.11, 3)
        b = oracle.epilogue(acc, w_scale, 0.02, bias, post, ot, 0.11, 3, sum=Z)
        assert np.array_equal(a, b), (post, ot)      # (by value: -0.0 + 0.0 is +0.0)


def test_sum_comes_after_gelu():
    mpmath = pytest.importorskip("mpmath")
    acc, w_scale, bias, R = _sum_inputs(33)
    g = oracle.epilogue(acc, w_scale, 0.002, bias, "gelu", "f32")          # pinned above
    got = oracle.epilogue(acc, w_scale, 0.002, bias, "gelu", "f32", sum=R)
    y = oracle.epilogue(acc, w_scale, 0.002, bias, "none", "f32")
    differs_from_wrong_order = 0
    for n in range(acc.shape[0]):
        for m in range(acc.shape[1]):
            assert float(got[n, m]) == f32_round(Fraction(float(g[n, m])) + Fraction(float(R[n, m])))
            x = mpmath.mpf(float(y[n, m])) + mpmath.mpf(float(R[n, m]))
            wrong = 0.5 * x * mpmath.erfc(-x / mpmath.sqrt(2))              # GELU(y + r)
            differs_from_wrong_order += int(abs(float(wrong) - float(got[n, m])) > 1e-3)
    assert differs_from_wrong_order > 100


@pytest.mark.parametrize("out_type,lo,hi", [("s8", -128, 127), ("u8", 0, 255)])
def test_sum_comes_before_quantize(out_type, lo, hi):
    acc, w_scale, bias, R = _sum_inputs(34)
    R = (R / 8).astype(np.float32)
    out_scale, zp = np.float32(0.173), 7
    z = oracle.epilogue(acc, w_scale, 0.002, bias, "none", "f32", sum=R)   # pinned above
    got = oracle.epilogue(acc, w_scale, 0.002, bias, "none", out_type, out_scale, zp, sum=R)
    inv = np.float32(1.0) / out_scale
    for n in range(acc.shape[0]):
        for m in range(acc.shape[1]):
            t = f32_round(Fraction(float(z[n, m])) * Fraction(float(inv)))
            assert int(got[n, m]) == min(hi, max(lo, py_round_half_even(t) + zp))
    assert len(np.unique(got)) > 20 and np.mean((got == lo) | (got == hi)) < 0.6   # not all saturated
    # an exact tie after the add: (0.5 + 2.0) / 1.0 = 2.5 -> 2, (1.5 + 2.0) -> 4  (half to even)
    a = np.array([[1, 3]], np.int32)
    r = np.array([[2.0, 2.0]], np.float32)
    q = oracle.epilogue(a, np.array([0.5], np.float32), 1.0, None, "none", out_type, 1.0, 0, sum=r)
    assert q.tolist() == [[2, 4]]


def test_sum_invalid_combinations_raise():
    acc = np.zeros((2, 2), np.int32)
    R = np.zeros((2, 2), np.float32)
    lut = np.zeros(256, np.int8)
    with pytest.raises(ValueError):      # a table entry is a function of one key: no second operand
        oracle.epilogue(acc, np.ones(2, np.float32), 1.0, None, "gelu", "s8", 1.0, 0, 1.0, lut, sum=R)
    with pytest.raises(ValueError):      # raw accumulators take no post-operators
        oracle.epilogue(acc, np.ones(2, np.float32), 1.0, None, "none", "s32", sum=R)
