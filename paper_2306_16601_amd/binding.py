"""ctypes binding of libspmm4x1.so: argument marshalling only.

Every function has the name and the argument order of its C declaration in
include/spmm.h; nothing of the method is computed here.  Host buffers are numpy
arrays, device buffers are anything with a `data_ptr()` (torch tensors) or a
raw integer address.  The library must have been built (see build.py); a
missing shared object is an error, there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libspmm4x1.so")

SPMM_OK, SPMM_E_ARG, SPMM_E_UNSUPPORTED, SPMM_E_ALLOC, SPMM_E_DEVICE = range(5)
SPMM_BLOCK_N4K1, SPMM_BLOCK_N1K4 = 0, 1
SPMM_POST_NONE, SPMM_POST_GELU, SPMM_POST_TABLE = 0, 1, 2
SPMM_OUT_S32, SPMM_OUT_F32, SPMM_OUT_S8, SPMM_OUT_U8 = 0, 1, 2, 3

BLOCKS = {"n4k1": SPMM_BLOCK_N4K1, "n1k4": SPMM_BLOCK_N1K4}
POSTOPS = {"none": SPMM_POST_NONE, "gelu": SPMM_POST_GELU, "table": SPMM_POST_TABLE}
OUT_TYPES = {"s32": SPMM_OUT_S32, "f32": SPMM_OUT_F32, "s8": SPMM_OUT_S8, "u8": SPMM_OUT_U8}

SPMM_X_TILE = 32                         # tokens per tile of the tile-major activation layout
SPMM_TILED_X, SPMM_TILED_OUT = 1, 2     # layout flags of spmm_run_tiled

EXPORTS = (
    "spmm_pack", "spmm_pack_host", "spmm_pack_ex", "spmm_row_order", "spmm_unpack", "spmm_info", "spmm_layout_dims",
    "spmm_layout_export", "spmm_run", "spmm_run_tiled", "spmm_make_gelu_lut", "spmm_plan", "spmm_set_tuning",
    "spmm_kernel_name", "spmm_kernel_variant", "spmm_kernel_variant_tiled", "spmm_measure_peak", "spmm_destroy", "spmm_status_string",
)


class spmm_epilogue_t(ctypes.Structure):
    _fields_ = [
        ("w_scale", ctypes.c_void_p),
        ("x_scale", ctypes.c_float),
        ("x_zero_point", ctypes.c_int32),
        ("bias", ctypes.c_void_p),
        ("postop", ctypes.c_int),
        ("out_type", ctypes.c_int),
        ("out_scale", ctypes.c_float),
        ("out_zero_point", ctypes.c_int32),
        ("mid_scale", ctypes.c_float),
        ("lut", ctypes.c_void_p),
        ("sum", ctypes.c_void_p),
        ("ld_sum", ctypes.c_int64),
    ]


class SpmmError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s: %s (status %d)" % (where, spmm_status_string(status), status))


_lib = None


def lib() -> ctypes.CDLL:
    """Load the built library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                "%s is missing: build it first (python -c 'import __graft_entry__ as g; g.build()')" % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        i64, i32, vp, f32, ci = ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p, ctypes.c_float, ctypes.c_int
        P = ctypes.POINTER
        L.spmm_pack.restype = ci
        L.spmm_pack.argtypes = [vp, i64, i64, i64, ci, P(vp)]
        L.spmm_pack_host.restype = ci
        L.spmm_pack_host.argtypes = [vp, i64, i64, i64, ci, P(vp)]
        L.spmm_pack_ex.restype = ci
        L.spmm_pack_ex.argtypes = [vp, i64, i64, i64, ci, ctypes.c_uint32, P(vp)]
        L.spmm_row_order.restype = ci
        L.spmm_row_order.argtypes = [vp, vp]
        L.spmm_unpack.restype = ci
        L.spmm_unpack.argtypes = [vp, vp, i64]
        L.spmm_info.restype = ci
        L.spmm_info.argtypes = [vp, P(i64), P(i64), P(i64), P(i64), P(i64)]
        L.spmm_layout_dims.restype = ci
        L.spmm_layout_dims.argtypes = [vp, P(i32), P(i32), P(i32), P(i64), P(i64), P(i64)]
        L.spmm_layout_export.restype = ci
        L.spmm_layout_export.argtypes = [vp, vp, vp, vp, vp]
        L.spmm_run.restype = ci
        L.spmm_run.argtypes = [vp, vp, i64, i64, P(spmm_epilogue_t), vp, i64, vp]
        L.spmm_run_tiled.restype = ci
        L.spmm_run_tiled.argtypes = [vp, vp, i64, i64, P(spmm_epilogue_t), vp, i64, ctypes.c_uint32, vp]
        L.spmm_make_gelu_lut.restype = ci
        L.spmm_make_gelu_lut.argtypes = [f32, f32, i32, ci, vp]
        L.spmm_plan.restype = ci
        L.spmm_plan.argtypes = [vp, i64, ci, P(i32), P(i32), P(i64)]
        L.spmm_set_tuning.restype = ci
        L.spmm_set_tuning.argtypes = [vp, i32, i32]
        L.spmm_kernel_name.restype = ctypes.c_char_p
        L.spmm_kernel_name.argtypes = []
        L.spmm_kernel_variant.restype = ci
        L.spmm_kernel_variant.argtypes = [vp, i64, ci, ci, ctypes.c_char_p, i64]
        L.spmm_kernel_variant_tiled.restype = ci
        L.spmm_kernel_variant_tiled.argtypes = [vp, i64, ci, ci, ctypes.c_uint32, ctypes.c_char_p, i64]
        L.spmm_measure_peak.restype = ci
        L.spmm_measure_peak.argtypes = [i32, P(ctypes.c_double)]
        L.spmm_destroy.restype = None
        L.spmm_destroy.argtypes = [vp]
        L.spmm_status_string.restype = ctypes.c_char_p
        L.spmm_status_string.argtypes = [ci]
        _lib = L
    return _lib


def _dev_ptr(x) -> Optional[int]:
    if x is None:
        return None
    if hasattr(x, "data_ptr"):
        return int(x.data_ptr())
    return int(x)


def _nbytes(x) -> Optional[int]:
    """Bytes from a tensor-like argument's data pointer to the end of its storage view, or None for a raw address."""
    if x is None or not hasattr(x, "data_ptr"):
        return None
    if hasattr(x, "untyped_storage") and hasattr(x, "storage_offset"):      # torch: what lies behind data_ptr()
        return int(x.untyped_storage().nbytes()) - int(x.storage_offset()) * int(x.element_size())
    if hasattr(x, "nbytes"):
        return int(x.nbytes)
    return None


def _check_extents(handle: int, X_dev, M: int, ldx: int, ep, out_dev, ldo: int, tiled: int) -> None:
    """Marshalling-side guard: when X / out / the Sum operand are tensors (not raw addresses), the memory
    behind them must cover what the kernels will touch -- a buffer built for another shape is an error
    here instead of a memory fault on the device."""
    N, K = spmm_info(handle)[:2]
    M, ldx, ldo = int(M), int(ldx), int(ldo)
    if M <= 0:
        return                                               # the library rejects it
    tiles = (M + SPMM_X_TILE - 1) // SPMM_X_TILE
    need_x = tiles * K * SPMM_X_TILE if tiled & SPMM_TILED_X else (K - 1) * ldx + M
    esz = 4 if ep is not None and int(ep.out_type) in (SPMM_OUT_S32, SPMM_OUT_F32) else 1
    need_o = tiles * N * SPMM_X_TILE if tiled & SPMM_TILED_OUT else ((N - 1) * ldo + M) * esz
    for name, t, need in (("X", X_dev, need_x), ("out", out_dev, need_o)):
        have = _nbytes(t)
        if have is not None and have < need:
            raise ValueError("spmm_run: %s holds %d bytes behind its data pointer, the call touches %d "
                             "(N=%d K=%d M=%d ldx=%d ldo=%d tiled=%d)" % (name, have, need, N, K, M, ldx, ldo, tiled))


def _check(status: int, where: str) -> None:
    if status != SPMM_OK:
        raise SpmmError(status, where)


def spmm_status_string(status: int) -> str:
    return lib().spmm_status_string(int(status)).decode()


def spmm_kernel_name() -> str:
    return lib().spmm_kernel_name().decode()


def spmm_kernel_variant(handle: int, M: int, out_type="s32", postop="none", tiled: int = 0) -> str:
    ot = OUT_TYPES[out_type] if isinstance(out_type, str) else int(out_type)
    po = POSTOPS[postop] if isinstance(postop, str) else int(postop)
    buf = ctypes.create_string_buffer(256)
    _check(lib().spmm_kernel_variant_tiled(handle, int(M), ot, po, int(tiled), buf, 256), "spmm_kernel_variant")
    return buf.value.decode()


def spmm_measure_peak(which: int) -> float:
    """Measured rate (10^12 operations per second) of the int8 matrix instruction (0) or of the
    4-wide int8 dot product (1) on the current device."""
    v = ctypes.c_double()
    _check(lib().spmm_measure_peak(int(which), ctypes.byref(v)), "spmm_measure_peak")
    return float(v.value)


def _pack(fn, W: np.ndarray, block) -> int:
    assert isinstance(W, np.ndarray) and W.dtype == np.int8 and W.ndim == 2 and W.strides[1] == 1
    N, K = W.shape
    h = ctypes.c_void_p()
    b = BLOCKS[block] if isinstance(block, str) else int(block)
    _check(fn(W.ctypes.data_as(ctypes.c_void_p), N, K, W.strides[0], b, ctypes.byref(h)), fn.__name__)
    return h.value


def spmm_pack(W: np.ndarray, block="n4k1") -> int:
    """Compress host W (int8 [N, K], row stride = ldw) onto the current device; returns a handle."""
    return _pack(lib().spmm_pack, W, block)


def spmm_pack_host(W: np.ndarray, block="n4k1") -> int:
    """Host-only compression (no GPU needed); the handle cannot be run."""
    return _pack(lib().spmm_pack_host, W, block)


SPMM_PACK_HOST_ONLY, SPMM_PACK_REORDER_ROWS = 1, 2


def spmm_pack_ex(W: np.ndarray, block="n4k1", host_only=False, reorder_rows=False) -> int:
    """spmm_pack with options; with reorder_rows the handle stands for W[spmm_row_order(handle)]."""
    assert isinstance(W, np.ndarray) and W.dtype == np.int8 and W.ndim == 2 and W.strides[1] == 1
    N, K = W.shape
    h = ctypes.c_void_p()
    b = BLOCKS[block] if isinstance(block, str) else int(block)
    flags = (SPMM_PACK_HOST_ONLY if host_only else 0) | (SPMM_PACK_REORDER_ROWS if reorder_rows else 0)
    _check(lib().spmm_pack_ex(W.ctypes.data_as(ctypes.c_void_p), N, K, W.strides[0], b, flags, ctypes.byref(h)),
           "spmm_pack_ex")
    return h.value


def spmm_row_order(handle: int) -> np.ndarray:
    """order[i] = row of the packed matrix that row i of the handle's outputs and per-row operands is."""
    N = spmm_info(handle)[0]
    order = np.empty(N, dtype=np.int32)
    _check(lib().spmm_row_order(handle, order.ctypes.data_as(ctypes.c_void_p)), "spmm_row_order")
    return order


def spmm_unpack(handle: int) -> np.ndarray:
    N, K, _, _, _ = spmm_info(handle)
    W = np.empty((N, K), dtype=np.int8)
    _check(lib().spmm_unpack(handle, W.ctypes.data_as(ctypes.c_void_p), K), "spmm_unpack")
    return W


def spmm_info(handle: int) -> Tuple[int, int, int, int, int]:
    """(N, K, nnz_blocks, padded_blocks, device_bytes)"""
    v = [ctypes.c_int64() for _ in range(5)]
    _check(lib().spmm_info(handle, *[ctypes.byref(x) for x in v]), "spmm_info")
    return tuple(int(x.value) for x in v)


def spmm_layout_dims(handle: int) -> Tuple[int, int, int, int, int, int]:
    """(tile_rows, step_k, segment_rows, n_tiles, n_segments, n_steps)"""
    a = [ctypes.c_int32() for _ in range(3)]
    b = [ctypes.c_int64() for _ in range(3)]
    _check(lib().spmm_layout_dims(handle, *[ctypes.byref(x) for x in a + b]), "spmm_layout_dims")
    return tuple(int(x.value) for x in a + b)


def spmm_layout_export(handle: int):
    """(vals uint8 [steps, 64, 16], idx uint32 [steps, 32], seg_ptr int32, rowsum int32)"""
    tile_rows, _, _, n_tiles, n_seg, n_steps = spmm_layout_dims(handle)
    vals = np.zeros((n_steps, 64, 16), dtype=np.uint8)
    idx = np.zeros((n_steps, 32), dtype=np.uint32)
    seg_ptr = np.zeros(n_tiles * n_seg + 1, dtype=np.int32)
    rowsum = np.zeros(n_tiles * tile_rows, dtype=np.int32)
    p = lambda a: a.ctypes.data_as(ctypes.c_void_p)
    _check(lib().spmm_layout_export(handle, p(vals), p(idx), p(seg_ptr), p(rowsum)), "spmm_layout_export")
    return vals, idx, seg_ptr, rowsum


def spmm_make_gelu_lut(mid_scale: float, out_scale: float, out_zero_point: int = 0, out_type="s8") -> np.ndarray:
    ot = OUT_TYPES[out_type] if isinstance(out_type, str) else int(out_type)
    lut = np.zeros(256, dtype=np.int8)
    _check(lib().spmm_make_gelu_lut(float(np.float32(mid_scale)), float(np.float32(out_scale)),
                                    int(out_zero_point), ot, lut.ctypes.data_as(ctypes.c_void_p)),
           "spmm_make_gelu_lut")
    return lut.view(np.uint8) if ot == SPMM_OUT_U8 else lut


def spmm_plan(handle: int, M: int, out_type="s32") -> Tuple[int, int, int]:
    """(token_tile, rows_per_workgroup, workgroups)"""
    ot = OUT_TYPES[out_type] if isinstance(out_type, str) else int(out_type)
    a, b, c = ctypes.c_int32(), ctypes.c_int32(), ctypes.c_int64()
    _check(lib().spmm_plan(handle, int(M), ot, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c)), "spmm_plan")
    return int(a.value), int(b.value), int(c.value)


def spmm_set_tuning(handle: int, token_tile: int = 0, variant: int = 0) -> None:
    _check(lib().spmm_set_tuning(handle, int(token_tile), int(variant)), "spmm_set_tuning")


def make_epilogue(w_scale=None, x_scale: float = 1.0, x_zero_point: int = 0, bias=None, postop="none",
                  out_type="s32", out_scale: float = 1.0, out_zero_point: int = 0, mid_scale: float = 1.0,
                  lut=None, sum=None, ld_sum: int = 0) -> spmm_epilogue_t:
    ep = spmm_epilogue_t()
    ep.w_scale = _dev_ptr(w_scale)
    ep.x_scale = float(np.float32(x_scale))
    ep.x_zero_point = int(x_zero_point)
    ep.bias = _dev_ptr(bias)
    ep.postop = POSTOPS[postop] if isinstance(postop, str) else int(postop)
    ep.out_type = OUT_TYPES[out_type] if isinstance(out_type, str) else int(out_type)
    ep.out_scale = float(np.float32(out_scale))
    ep.out_zero_point = int(out_zero_point)
    ep.mid_scale = float(np.float32(mid_scale))
    ep.lut = _dev_ptr(lut)
    ep.sum = _dev_ptr(sum)
    ep.ld_sum = int(ld_sum)
    ep._keepalive = (w_scale, bias, lut, sum)   # the struct holds raw addresses: keep their owners alive with it
    return ep


def spmm_run_status(handle: int, X_dev, M: int, ldx: int, ep: Optional[spmm_epilogue_t], out_dev, ldo: int,
                    stream=None) -> int:
    """Raw call returning the status code (used by the error-path tests)."""
    st = None if stream is None else int(stream)
    return int(lib().spmm_run(handle, _dev_ptr(X_dev), int(M), int(ldx),
                              None if ep is None else ctypes.byref(ep), _dev_ptr(out_dev), int(ldo), st))


def spmm_run(handle: int, X_dev, M: int, ldx: int, ep: spmm_epilogue_t, out_dev, ldo: int, stream=None) -> None:
    """out = postops(W . X), asynchronous on `stream` (a raw hipStream_t value, None = default stream)."""
    _check_extents(handle, X_dev, M, ldx, ep, out_dev, ldo, 0)
    _check(spmm_run_status(handle, X_dev, M, ldx, ep, out_dev, ldo, stream), "spmm_run")


def tile_major(X: np.ndarray) -> np.ndarray:
    """Host helper: 1-byte [R, M] row-major -> token-tile-major [ceil(M / 32), R, 32], last tile
    zero-padded (data movement only)."""
    R, M = X.shape
    T = (M + SPMM_X_TILE - 1) // SPMM_X_TILE
    Xp = np.zeros((R, T * SPMM_X_TILE), dtype=X.dtype)
    Xp[:, :M] = X
    return np.ascontiguousarray(Xp.reshape(R, T, SPMM_X_TILE).transpose(1, 0, 2))


def from_tile_major(T: np.ndarray, M: int) -> np.ndarray:
    """Inverse of tile_major: [tiles, R, 32] -> row-major [R, M]."""
    tiles, R, w = T.shape
    return np.ascontiguousarray(T.transpose(1, 0, 2).reshape(R, tiles * w)[:, :M])


def spmm_run_tiled(handle: int, X_dev, M: int, ldx: int, ep: spmm_epilogue_t, out_dev, ldo: int, tiled: int,
                   stream=None) -> None:
    """spmm_run with X (SPMM_TILED_X) and / or a 1-byte output (SPMM_TILED_OUT) in token-tile-major order."""
    st = None if stream is None else int(stream)
    _check_extents(handle, X_dev, M, ldx, ep, out_dev, ldo, int(tiled))
    _check(int(lib().spmm_run_tiled(handle, _dev_ptr(X_dev), int(M), int(ldx), ctypes.byref(ep), _dev_ptr(out_dev),
                                    int(ldo), int(tiled), st)), "spmm_run_tiled")


def spmm_run_tiled_bound(handle: int, X_dev, M: int, ldx: int, ep: spmm_epilogue_t, out_dev, ldo: int, tiled: int,
                         stream=None):
    """spmm_run_tiled with its arguments marshalled once (see spmm_run_bound)."""
    _check_extents(handle, X_dev, M, ldx, ep, out_dev, ldo, int(tiled))
    fn = lib().spmm_run_tiled
    args = (ctypes.c_void_p(handle), ctypes.c_void_p(_dev_ptr(X_dev)), ctypes.c_int64(int(M)), ctypes.c_int64(int(ldx)),
            ctypes.byref(ep), ctypes.c_void_p(_dev_ptr(out_dev)), ctypes.c_int64(int(ldo)), ctypes.c_uint32(int(tiled)),
            ctypes.c_void_p(None if stream is None else int(stream)))

    def call() -> int:
        return fn(*args)
    call._keepalive = (ep, X_dev, out_dev)
    return call


def spmm_run_bound(handle: int, X_dev, M: int, ldx: int, ep: spmm_epilogue_t, out_dev, ldo: int, stream=None):
    """spmm_run with its arguments marshalled once: returns a callable that makes the C call and
    returns its status (for launch loops of microsecond kernels, where converting the arguments
    every time costs as much as the kernel).  The caller keeps the tensors and `ep` alive."""
    _check_extents(handle, X_dev, M, ldx, ep, out_dev, ldo, 0)
    fn = lib().spmm_run
    args = (ctypes.c_void_p(handle), ctypes.c_void_p(_dev_ptr(X_dev)), ctypes.c_int64(int(M)), ctypes.c_int64(int(ldx)),
            ctypes.byref(ep), ctypes.c_void_p(_dev_ptr(out_dev)), ctypes.c_int64(int(ldo)),
            ctypes.c_void_p(None if stream is None else int(stream)))

    def call() -> int:
        return fn(*args)
    call._keepalive = (ep, X_dev, out_dev)
    return call


def spmm_destroy(handle: Optional[int]) -> None:
    if handle:
        lib().spmm_destroy(handle)
