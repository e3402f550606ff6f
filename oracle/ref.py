"""ctypes front end of the C oracle (oracle/bcq_ref.c).

TEST INFRASTRUCTURE: plain fp64 evaluation of the binary-coded product
(paper Eq. 3 dequantisation, Eq. 11 fused form).  Operands are numpy arrays in
the canonical layout documented in bcq_ref.c; nothing here does arithmetic of
its own beyond reshaping and dtype checks.
"""
import ctypes
import os

import numpy as np

from . import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.LIB
        if not os.path.exists(path):
            _build.build()
        L = ctypes.CDLL(path)
        i64, i32, vp = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p
        L.bcq_ref_half_to_double.restype = ctypes.c_double
        L.bcq_ref_half_to_double.argtypes = [ctypes.c_uint16]
        L.bcq_ref_dequant.restype = i32
        L.bcq_ref_dequant.argtypes = [vp, vp, vp, i64, i64, i32, i64, vp]
        L.bcq_ref_dense_matmul.restype = i32
        L.bcq_ref_dense_matmul.argtypes = [vp, vp, i64, i64, i64, vp]
        L.bcq_ref_gemm.restype = i32
        L.bcq_ref_gemm.argtypes = [vp, vp, vp, vp, i64, i64, i32, i64, i64, vp]
        L.bcq_ref_brute.restype = i32
        L.bcq_ref_brute.argtypes = [vp, vp, vp, vp, i64, i64, i32, i64, i64, vp]
        L.bcq_ref_num_threads.restype = i32
        L.bcq_ref_set_num_threads.argtypes = [i32]
        _lib = L
    return _lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _canon(planes, alpha, z, X=None):
    planes = np.ascontiguousarray(planes, dtype=np.uint32)
    alpha = np.ascontiguousarray(alpha).view(np.uint16)
    q, M, words = planes.shape
    N = words * 32
    assert alpha.shape[0] == M and alpha.shape[2] == q, "alpha is [M][G][q]"
    G = alpha.shape[1]
    assert N % G == 0
    if z is not None:
        z = np.ascontiguousarray(z).view(np.uint16)
        assert z.shape == (M, G), "offset is [M][G]"
    if X is not None:
        X = np.ascontiguousarray(X).view(np.uint16)
        if X.ndim == 1:
            X = X[None, :]
        assert X.shape[1] == N
    return planes, alpha, z, X, M, N, q, N // G


def half_to_double(bits):
    """binary16 bit pattern(s) -> float64, through the C routine."""
    L = lib()
    bits = np.asarray(bits, dtype=np.uint16)
    out = np.empty(bits.shape, dtype=np.float64)
    flat_in, flat_out = bits.ravel(), out.ravel()
    for t in range(flat_in.size):
        flat_out[t] = L.bcq_ref_half_to_double(int(flat_in[t]))
    return out


def dequant(planes, alpha, z=None):
    """Dense fp64 W[M][N] (Eq. 3 dequant / Eq. 11)."""
    planes, alpha, z, _, M, N, q, g = _canon(planes, alpha, z)
    W = np.empty((M, N), dtype=np.float64)
    rc = lib().bcq_ref_dequant(_ptr(planes), _ptr(alpha), _ptr(z), M, N, q, g, _ptr(W))
    if rc:
        raise ValueError("bcq_ref_dequant: bad argument")
    return W


def dense_matmul(W, X):
    W = np.ascontiguousarray(W, dtype=np.float64)
    X = np.ascontiguousarray(X).view(np.uint16)
    if X.ndim == 1:
        X = X[None, :]
    M, N = W.shape
    b = X.shape[0]
    Y = np.empty((b, M), dtype=np.float64)
    rc = lib().bcq_ref_dense_matmul(_ptr(W), _ptr(X), M, N, b, _ptr(Y))
    if rc:
        raise ValueError("bcq_ref_dense_matmul: bad argument")
    return Y


def gemm(planes, alpha, z, X):
    """Y[b][M] fp64 = X W_q^T, W_q dequantised row by row (the oracle proper)."""
    planes, alpha, z, X, M, N, q, g = _canon(planes, alpha, z, X)
    b = X.shape[0]
    Y = np.empty((b, M), dtype=np.float64)
    rc = lib().bcq_ref_gemm(_ptr(planes), _ptr(alpha), _ptr(z), _ptr(X), M, N, q, g, b, _ptr(Y))
    if rc:
        raise ValueError("bcq_ref_gemm: bad argument")
    return Y


def brute(planes, alpha, z, X):
    """Independent grouped-order evaluation of Eq. 11 (small shapes)."""
    planes, alpha, z, X, M, N, q, g = _canon(planes, alpha, z, X)
    b = X.shape[0]
    Y = np.empty((b, M), dtype=np.float64)
    rc = lib().bcq_ref_brute(_ptr(planes), _ptr(alpha), _ptr(z), _ptr(X), M, N, q, g, b, _ptr(Y))
    if rc:
        raise ValueError("bcq_ref_brute: bad argument")
    return Y


def num_threads():
    return int(lib().bcq_ref_num_threads())


def set_num_threads(n):
    lib().bcq_ref_set_num_threads(int(n))
