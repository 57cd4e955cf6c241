"""CPU oracle for the 4x1 structured-sparse INT8 SpMM (test infrastructure).

Thin ctypes wrapper over `spmm_oracle.c`, the plain triple-loop definition of
what the hot path computes (Section 3.2 / Algorithm 1, post-operators of
Section 3.3, lookup table of Algorithm 2).  Only tests, the smoke check and the
bench's CPU-baseline leg may import this package; it imports nothing from the
HIP library and the HIP library imports nothing from here.
"""
from __future__ import annotations

import ctypes
from typing import Optional

import numpy as np

from .build import build as _build

OUT_TYPES = {"s32": 0, "f32": 1, "s8": 2, "u8": 3}
POSTOPS = {"none": 0, "gelu": 1, "table": 2}
_OUT_DTYPES = {"s32": np.int32, "f32": np.float32, "s8": np.int8, "u8": np.uint8}

_lib = None


def load(path: str) -> ctypes.CDLL:
    """dlopen an oracle shared object and declare its prototypes."""
    L = ctypes.CDLL(path)
    i64, i32, f32, vp = ctypes.c_int64, ctypes.c_int32, ctypes.c_float, ctypes.c_void_p
    L.oracle_gelu.restype = ctypes.c_double
    L.oracle_gelu.argtypes = [ctypes.c_double]
    L.oracle_acc_s32.restype = None
    L.oracle_acc_s32.argtypes = [vp, i64, vp, i64, i64, i64, i64, i32, vp]
    L.oracle_gelu_lut.restype = ctypes.c_int
    L.oracle_gelu_lut.argtypes = [f32, f32, i32, ctypes.c_int, vp]
    L.oracle_epilogue_sum.restype = ctypes.c_int
    L.oracle_epilogue_sum.argtypes = [vp, i64, i64, vp, f32, vp, ctypes.c_int, vp, i64, ctypes.c_int,
                                      f32, i32, f32, vp, vp, i64]
    L.oracle_num_threads.restype = ctypes.c_int
    L.oracle_set_num_threads.argtypes = [ctypes.c_int]
    return L


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        _lib = load(_build())
    return _lib


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def set_num_threads(n: int) -> None:
    lib().oracle_set_num_threads(int(n))


def gelu(x: float) -> float:
    """Exact GELU in double."""
    return float(lib().oracle_gelu(float(x)))


def acc_s32(W: np.ndarray, X: np.ndarray, x_zero_point: int = 0) -> np.ndarray:
    """int32 [N, M] accumulator: sum_k W[n,k] * (X[k,m] - x_zero_point)."""
    assert W.dtype == np.int8 and X.dtype == np.uint8 and W.ndim == 2 and X.ndim == 2
    assert W.shape[1] == X.shape[0]
    assert W.strides[1] == 1 and X.strides[1] == 1, "rows must be contiguous"
    N, K = W.shape
    M = X.shape[1]
    acc = np.empty((N, M), dtype=np.int32)
    lib().oracle_acc_s32(_ptr(W), W.strides[0], _ptr(X), X.strides[0], N, K, M,
                         int(x_zero_point), _ptr(acc))
    return acc


def gelu_lut(mid_scale: float, out_scale: float, out_zero_point: int = 0,
             out_type: str = "s8") -> np.ndarray:
    """256-entry table of Algorithm 2 for dequantise -> GELU -> quantise.
    Returned as int8 (s8 output) or uint8 (u8 output); entry [i + 128] belongs to key i."""
    lut = np.empty(256, dtype=np.int8)
    rc = lib().oracle_gelu_lut(float(np.float32(mid_scale)), float(np.float32(out_scale)),
                               int(out_zero_point), OUT_TYPES[out_type], _ptr(lut))
    if rc != 0:
        raise ValueError("gelu_lut: out_type must be s8 or u8")
    return lut.view(np.uint8) if out_type == "u8" else lut


def epilogue(acc: np.ndarray, w_scale: Optional[np.ndarray], x_scale: float = 1.0,
             bias: Optional[np.ndarray] = None, postop: str = "none", out_type: str = "s32",
             out_scale: float = 1.0, out_zero_point: int = 0, mid_scale: float = 1.0,
             lut: Optional[np.ndarray] = None, sum: Optional[np.ndarray] = None) -> np.ndarray:
    """Post-operator chain applied to an int32 accumulator matrix; `sum` is the optional second
    operand of the Sum post-operator, fp32 [N, M]."""
    assert acc.dtype == np.int32 and acc.flags.c_contiguous
    N, M = acc.shape
    if w_scale is not None:
        w_scale = np.ascontiguousarray(w_scale, dtype=np.float32)
        assert w_scale.shape == (N,)
    if bias is not None:
        bias = np.ascontiguousarray(bias, dtype=np.float32)
        assert bias.shape == (N,)
    if lut is not None:
        lut = np.ascontiguousarray(lut).view(np.int8)
        assert lut.shape == (256,)
    if sum is not None:
        sum = np.ascontiguousarray(sum, dtype=np.float32)
        assert sum.shape == (N, M)
    out = np.empty((N, M), dtype=_OUT_DTYPES[out_type])
    rc = lib().oracle_epilogue_sum(_ptr(acc), N, M, _ptr(w_scale), float(np.float32(x_scale)),
                                   _ptr(bias), POSTOPS[postop], _ptr(sum), M, OUT_TYPES[out_type],
                                   float(np.float32(out_scale)), int(out_zero_point),
                                   float(np.float32(mid_scale)), _ptr(lut), _ptr(out), M)
    if rc != 0:
        raise ValueError("oracle_epilogue_sum: invalid argument combination")
    return out


def spmm(W: np.ndarray, X: np.ndarray, w_scale: Optional[np.ndarray] = None,
         x_scale: float = 1.0, bias: Optional[np.ndarray] = None, postop: str = "none",
         out_type: str = "s32", out_scale: float = 1.0, out_zero_point: int = 0,
         mid_scale: float = 1.0, x_zero_point: int = 0,
         lut: Optional[np.ndarray] = None, sum: Optional[np.ndarray] = None) -> np.ndarray:
    """out = epilogue(W . X) on the dense-with-zeros W.  For GELU with an int8
    output the lookup table is built here unless one is passed."""
    acc = acc_s32(W, X, x_zero_point)
    if out_type == "s32":
        return acc
    if postop == "gelu" and out_type in ("s8", "u8") and lut is None:
        lut = gelu_lut(mid_scale, out_scale, out_zero_point, out_type)
    return epilogue(acc, w_scale, x_scale, bias, postop, out_type, out_scale,
                    out_zero_point, mid_scale, lut, sum)
