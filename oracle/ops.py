"""ctypes face of the C oracle (oracle_ops.c).  TEST INFRASTRUCTURE ONLY.

All results come back as float64 numpy arrays.  Inputs are numpy arrays holding the
stored bits: float32, float16, or uint16 for bfloat16.
"""
from __future__ import annotations

import ctypes as C

import numpy as np

from . import build as _build

_DT = {"f32": 0, "f16": 1, "bf16": 2}
_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(_build.build())
        i64, dbl, ptr, i32 = C.c_int64, C.c_double, C.c_void_p, C.c_int
        L.oracle_decode.restype = dbl
        L.oracle_decode.argtypes = [i32, ptr, i64]
        L.oracle_num_threads.restype = i32
        L.oracle_gemm.restype = i32
        L.oracle_gemm.argtypes = [i32, i32, i32, i64, i64, i64, dbl, ptr, i64, ptr, i64, dbl, ptr, i64]
        L.oracle_bmm.restype = i32
        L.oracle_bmm.argtypes = [i32, i32, i32, i64, i64, i64, i64, dbl, ptr, i64, i64, ptr, i64, i64,
                                 dbl, ptr, i64, i64]
        L.oracle_bmm_at.restype = i32
        L.oracle_bmm_at.argtypes = [i32, i32, i32, i64, dbl, ptr, i64, i64, ptr, i64, i64, i64, ptr, ptr]
        L.oracle_conv2d.restype = i32
        L.oracle_conv2d.argtypes = [i32] + [i64] * 9 + [ptr, ptr, ptr]
        L.oracle_conv2d_at.restype = i32
        L.oracle_conv2d_at.argtypes = [i32] + [i64] * 9 + [ptr, ptr, i64, ptr, ptr]
        L.oracle_gemv.argtypes = [i32, i64, i64, dbl, ptr, i64, ptr, dbl, ptr]
        L.oracle_avgpool2d.argtypes = [i32] + [i64] * 6 + [ptr, ptr]
        L.oracle_avgpool2d_at.argtypes = [i32] + [i64] * 5 + [ptr, i64, ptr, ptr]
        _lib = L
    return _lib


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def _check(arr: np.ndarray, dtype: str) -> np.ndarray:
    want = {"f32": np.float32, "f16": np.float16, "bf16": np.uint16}[dtype]
    if arr.dtype != want:
        raise TypeError(f"{dtype} operand must be stored as {want}, got {arr.dtype}")
    return np.ascontiguousarray(arr)


def _p(a: np.ndarray):
    return a.ctypes.data_as(C.c_void_p)


def decode(arr: np.ndarray, dtype: str) -> np.ndarray:
    a = _check(arr, dtype).reshape(-1)
    L = lib()
    return np.array([L.oracle_decode(_DT[dtype], _p(a), i) for i in range(a.size)]).reshape(arr.shape)


def gemm(A, B, dtype, transA=0, transB=0, alpha=1.0, beta=0.0, C0=None):
    """C = alpha op(A) op(B) + beta C0.  A is [M][K] (or [K][M] if transA), B is [K][N]
    (or [N][K] if transB); leading dimensions are the stored row lengths."""
    A = _check(A, dtype)
    B = _check(B, dtype)
    M, K = (A.shape[1], A.shape[0]) if transA else A.shape
    K2, N = (B.shape[1], B.shape[0]) if transB else B.shape
    assert K == K2, (A.shape, B.shape)
    Cd = np.zeros((M, N), dtype=np.float64) if C0 is None else np.array(C0, dtype=np.float64)
    rc = lib().oracle_gemm(_DT[dtype], transA, transB, M, N, K, float(alpha), _p(A), A.shape[1],
                           _p(B), B.shape[1], float(beta), _p(Cd), N)
    assert rc == 0
    return Cd


def bmm(A, B, dtype, transA=0, transB=0, alpha=1.0, beta=0.0, C0=None):
    A = _check(A, dtype)
    B = _check(B, dtype)
    nb = A.shape[0]
    M, K = (A.shape[2], A.shape[1]) if transA else A.shape[1:]
    K2, N = (B.shape[2], B.shape[1]) if transB else B.shape[1:]
    assert K == K2 and B.shape[0] == nb
    Cd = np.zeros((nb, M, N), dtype=np.float64) if C0 is None else np.array(C0, dtype=np.float64)
    rc = lib().oracle_bmm(_DT[dtype], transA, transB, nb, M, N, K, float(alpha),
                          _p(A), A.shape[2], A.shape[1] * A.shape[2],
                          _p(B), B.shape[2], B.shape[1] * B.shape[2],
                          float(beta), _p(Cd), N, M * N)
    assert rc == 0
    return Cd


def bmm_at(A, B, dtype, coords, transA=0, transB=0, alpha=1.0):
    """alpha * (op(A_b) op(B_b))[i][j] at each row (b, i, j) of `coords`.  2-D operands
    are taken as a batch of one."""
    A = _check(A, dtype)
    B = _check(B, dtype)
    if A.ndim == 2:
        A, B = A[None], B[None]
    K = A.shape[1] if transA else A.shape[2]
    co = np.ascontiguousarray(coords, dtype=np.int64).reshape(-1, 3)
    out = np.zeros(co.shape[0], dtype=np.float64)
    rc = lib().oracle_bmm_at(_DT[dtype], transA, transB, K, float(alpha),
                             _p(A), A.shape[2], A.shape[1] * A.shape[2],
                             _p(B), B.shape[2], B.shape[1] * B.shape[2],
                             co.shape[0], _p(co), _p(out))
    assert rc == 0
    return out


def conv_out_shape(n, c, h, w, k, r, s, stride, pad):
    p = (h + 2 * pad - r) // stride + 1 if h + 2 * pad - r >= 0 else 0
    q = (w + 2 * pad - s) // stride + 1 if w + 2 * pad - s >= 0 else 0
    return (n, k, p, q)


def conv2d(I, W, dtype, stride=1, pad=0):
    I = _check(I, dtype)
    W = _check(W, dtype)
    n, c, h, w = I.shape
    k, c2, r, s = W.shape
    assert c == c2
    O = np.zeros(conv_out_shape(n, c, h, w, k, r, s, stride, pad), dtype=np.float64)
    rc = lib().oracle_conv2d(_DT[dtype], n, c, h, w, k, r, s, stride, pad, _p(I), _p(W), _p(O))
    assert rc == 0
    return O


def conv2d_at(I, W, dtype, coords, stride=1, pad=0):
    I = _check(I, dtype)
    W = _check(W, dtype)
    n, c, h, w = I.shape
    k, _, r, s = W.shape
    co = np.ascontiguousarray(coords, dtype=np.int64).reshape(-1, 4)
    out = np.zeros(co.shape[0], dtype=np.float64)
    rc = lib().oracle_conv2d_at(_DT[dtype], n, c, h, w, k, r, s, stride, pad, _p(I), _p(W),
                                co.shape[0], _p(co), _p(out))
    assert rc == 0
    return out


def gemv(A, x, dtype, alpha=1.0, beta=0.0, y0=None):
    """y = alpha A x + beta y0 for a row-major A [M][N] (GEMV row of the operator table)."""
    A = _check(A, dtype)
    x = _check(x, dtype)
    M, N = A.shape
    assert x.shape == (N,)
    y = np.zeros(M, dtype=np.float64) if y0 is None else np.array(y0, dtype=np.float64)
    rc = lib().oracle_gemv(_DT[dtype], M, N, float(alpha), _p(A), N, _p(x), float(beta), _p(y))
    assert rc == 0
    return y


def pool_out_shape(n, c, h, w, f, stride):
    return (n, c, (h - f) // stride + 1, (w - f) // stride + 1)


def avgpool2d(I, dtype, f, stride):
    """O = average over f x f windows at the given stride of an NCHW input, no padding."""
    I = _check(I, dtype)
    n, c, h, w = I.shape
    O = np.zeros(pool_out_shape(n, c, h, w, f, stride), dtype=np.float64)
    rc = lib().oracle_avgpool2d(_DT[dtype], n, c, h, w, f, stride, _p(I), _p(O))
    assert rc == 0
    return O


def avgpool2d_at(I, dtype, coords, f, stride):
    I = _check(I, dtype)
    n, c, h, w = I.shape
    co = np.ascontiguousarray(coords, dtype=np.int64)
    out = np.zeros(co.shape[0], dtype=np.float64)
    rc = lib().oracle_avgpool2d_at(_DT[dtype], c, h, w, f, stride, _p(I), co.shape[0], _p(co), _p(out))
    assert rc == 0
    return out


def rel_frobenius(got, want) -> float:
    """||got - want||_F / ||want||_F in float64."""
    g = np.asarray(got, dtype=np.float64)
    w = np.asarray(want, dtype=np.float64)
    den = np.sqrt(np.sum(w * w))
    num = np.sqrt(np.sum((g - w) ** 2))
    return float(num / den) if den > 0 else float(num)
