"""CPU oracle for the generalized sparse convolution (Sec. III-B, Eq. 2).

TEST INFRASTRUCTURE ONLY: imported by tests, the smoke check and the
benchmark's cpu_baseline leg.  The product package never imports this.

The arithmetic lives in `sp_oracle.c` (plain C, double accumulation, sort +
binary search instead of hashing); this file only compiles it with gcc and
marshals numpy arrays.  Every function states the passage it follows.

Parity status: every function here is pinned by tests/test_oracle_pins.py
(dense 3-D convolution from a library routine, closed-form pair counts,
brute-force coordinate comparison, adjoint identities); none is unpinned.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sp_oracle.c")
_LIB = os.path.join(_HERE, "libsp_oracle.so")
_lib = None

_i32p = np.ctypeslib.ndpointer(np.int32, flags="C_CONTIGUOUS")
_i64p = np.ctypeslib.ndpointer(np.int64, flags="C_CONTIGUOUS")
_f32p = np.ctypeslib.ndpointer(np.float32, flags="C_CONTIGUOUS")
_f64p = np.ctypeslib.ndpointer(np.float64, flags="C_CONTIGUOUS")


def build(force: bool = False) -> str:
    """Compile sp_oracle.c with gcc (-O2, scalar, no OpenMP) into libsp_oracle.so."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-Wall", "-o", _LIB, _SRC])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = C.CDLL(build())
        lib.sp_oracle_unique.restype = C.c_int64
        lib.sp_oracle_unique.argtypes = [_i32p, C.c_int64, C.c_int32, _i32p, _i32p]
        lib.sp_oracle_kmap.restype = C.c_int64
        lib.sp_oracle_kmap.argtypes = [_i32p, C.c_int64, _i32p, C.c_int64, C.c_int32, C.c_int32,
                                       C.c_void_p, C.c_void_p, _i64p]
        for name, arr in (("sp_oracle_conv_fwd", [_f32p, _f32p, _f64p, C.c_int64]),
                          ("sp_oracle_conv_bwd_data", [_f32p, _f32p, _f64p, C.c_int64]),
                          ("sp_oracle_conv_bwd_weight", [_f32p, _f32p, _f64p])):
            fn = getattr(lib, name)
            fn.restype = None
            fn.argtypes = [_i32p, _i32p, _i64p, C.c_int32] + arr + [C.c_int32, C.c_int32]
        _lib = lib
    return _lib


def _coords(a) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.int32)
    if a.ndim != 2 or a.shape[1] != 4:
        raise ValueError("coordinates must be [n][4] rows (b,x,y,z)")
    return a


def unique_coords(raw, floor_step: int = 1):
    """Merge duplicate (b,x,y,z) rows, first-occurrence order (Sec. III-B sparse tensor).

    With floor_step > 1 the spatial coordinates are first floored to a multiple of
    floor_step: the strided output-coordinate rule of step 1.
    Returns (coords [N][4] int32, inverse [n_raw] int32).
    """
    raw = _coords(raw)
    n = raw.shape[0]
    uniq = np.empty((max(n, 1), 4), dtype=np.int32)
    inv = np.empty(max(n, 1), dtype=np.int32)
    N = _load().sp_oracle_unique(raw if n else np.zeros((1, 4), np.int32), n, int(floor_step), uniq, inv)
    if N < 0:
        raise MemoryError
    return uniq[:N].copy(), inv[:n].copy()


def strided_coords(c_in, tensor_stride: int, stride: int):
    """Step 1 (Sec. III-B): output coordinates of a stride-`stride` layer on a tensor of stride `tensor_stride`.

    Stride 1 keeps the input coordinates.  Returns (c_out, parent [n_in] -> out row, new tensor stride).
    """
    c_in = _coords(c_in)
    if stride == 1:
        return c_in.copy(), np.arange(c_in.shape[0], dtype=np.int32), tensor_stride
    c_out, parent = unique_coords(c_in, tensor_stride * stride)
    return c_out, parent, tensor_stride * stride


def kernel_map(c_in, c_out, kernel_size: int, step: int):
    """Step 2 (Sec. III-B): per-offset (in,out) pair lists, each sorted by (in,out).

    step = dilation * input tensor stride.  Returns (pair_in, pair_out, counts[K^3]);
    the lists of all offsets are concatenated in offset order.
    """
    c_in, c_out = _coords(c_in), _coords(c_out)
    kvol = kernel_size ** 3
    counts = np.zeros(kvol, dtype=np.int64)
    lib = _load()
    dummy = np.zeros((1, 4), np.int32)
    a = c_in if c_in.shape[0] else dummy
    b = c_out if c_out.shape[0] else dummy
    total = lib.sp_oracle_kmap(a, c_in.shape[0], b, c_out.shape[0], kernel_size, step, None, None, counts)
    if total < 0:
        raise MemoryError
    pin = np.empty(max(total, 1), dtype=np.int32)
    pout = np.empty(max(total, 1), dtype=np.int32)
    lib.sp_oracle_kmap(a, c_in.shape[0], b, c_out.shape[0], kernel_size, step,
                       pin.ctypes.data_as(C.c_void_p), pout.ctypes.data_as(C.c_void_p), counts)
    return pin[:total].copy(), pout[:total].copy(), counts


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _pad(a):
    return a if a.size else np.zeros(1, a.dtype)


def conv_fwd(pair_in, pair_out, counts, X, W, n_out: int) -> np.ndarray:
    """Eq. 2: Y[o] = sum_k sum_{(i,o) in M_k} W_k X[i];  W is [K^3][cout][cin].  Returns float64 [n_out][cout]."""
    X, W = _f32(X), _f32(W)
    kvol, cout, cin = W.shape
    Y = np.zeros((max(n_out, 1), cout), dtype=np.float64)
    _load().sp_oracle_conv_fwd(_pad(pair_in), _pad(pair_out), np.ascontiguousarray(counts, np.int64), kvol,
                               _pad(X.reshape(-1)), W.reshape(-1), Y.reshape(-1), n_out, cin, cout)
    return Y[:n_out]


def conv_bwd_data(pair_in, pair_out, counts, dY, W, n_in: int) -> np.ndarray:
    """d/dx_in of Eq. 2: dX[i] = sum_k sum_{(i,o) in M_k} W_k^T dY[o].  Returns float64 [n_in][cin]."""
    dY, W = _f32(dY), _f32(W)
    kvol, cout, cin = W.shape
    dX = np.zeros((max(n_in, 1), cin), dtype=np.float64)
    _load().sp_oracle_conv_bwd_data(_pad(pair_in), _pad(pair_out), np.ascontiguousarray(counts, np.int64), kvol,
                                    _pad(dY.reshape(-1)), W.reshape(-1), dX.reshape(-1), n_in, cin, cout)
    return dX[:n_in]


def conv_bwd_weight(pair_in, pair_out, counts, X, dY) -> np.ndarray:
    """d/dW of Eq. 2: dW_k = sum_{(i,o) in M_k} dY[o] X[i]^T.  Returns float64 [K^3][cout][cin]."""
    X, dY = _f32(X), _f32(dY)
    kvol = len(counts)
    cin, cout = X.shape[1], dY.shape[1]
    dW = np.zeros((kvol, cout, cin), dtype=np.float64)
    _load().sp_oracle_conv_bwd_weight(_pad(pair_in), _pad(pair_out), np.ascontiguousarray(counts, np.int64), kvol,
                                      _pad(X.reshape(-1)), _pad(dY.reshape(-1)), dW.reshape(-1), cin, cout)
    return dW


def transpose_map(pair_in, pair_out, counts):
    """Kernel map of the transposed (upsampling) convolution: the forward strided map with roles swapped.

    The paper does not define a transposed sparse convolution; the reading taken is that it
    reuses the cached coordinate hierarchy: M_k^T = {(o,i) : (i,o) in M_k}, same offset numbering.
    Lists are re-sorted by their new (in,out) columns.
    """
    pin = np.empty_like(pair_in)
    pout = np.empty_like(pair_out)
    base = 0
    for c in counts:
        a, b = pair_out[base:base + c], pair_in[base:base + c]
        order = np.lexsort((b, a))
        pin[base:base + c], pout[base:base + c] = a[order], b[order]
        base += c
    return pin, pout, np.asarray(counts, dtype=np.int64).copy()
