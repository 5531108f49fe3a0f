"""ctypes front end of the C oracle (Eq. 1, Eq. 2 and the transpose of Section III).

TEST INFRASTRUCTURE ONLY; see ``mtnn_oracle.c`` for the arithmetic.  These
wrappers only check shapes and pass pointers.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

from . import build as _build

_lib = None


def _load():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        lib = ctypes.CDLL(path)
        gemm_args = [ctypes.c_int] * 3 + [ctypes.c_void_p, ctypes.c_long, ctypes.c_void_p, ctypes.c_long,
                                           ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
        lib.oracle_nt_ref.argtypes = gemm_args
        lib.oracle_nt_ref.restype = None
        lib.oracle_nn_ref.argtypes = gemm_args
        lib.oracle_nn_ref.restype = None
        lib.oracle_transpose_ref.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_long,
                                             ctypes.c_void_p, ctypes.c_long]
        lib.oracle_transpose_ref.restype = None
        lib.oracle_num_threads.restype = ctypes.c_int
        for name in ("oracle_f64_nt", "oracle_f64_nn", "oracle_f64_tn"):
            fn = getattr(lib, name)
            fn.argtypes = [ctypes.c_int] * 3 + [ctypes.c_void_p] * 3
            fn.restype = None
        _lib = lib
    return _lib


def num_threads() -> int:
    """Threads the row-parallel loops will use."""
    return int(_load().oracle_num_threads())


def _as_f32_2d(x, name):
    x = np.asarray(x)
    if x.dtype != np.float32 or x.ndim != 2:
        raise ValueError(f"{name} must be a 2-D float32 array")
    if x.size and ((x.shape[1] > 1 and x.strides[1] != 4) or (x.shape[0] > 1 and x.strides[0] % 4)):
        raise ValueError(f"{name} must be a 2-D float32 array with unit column stride")
    return x


def _ld(x):
    return x.strides[0] // 4 if (x.shape[0] > 1 and x.size) else max(x.shape[1], 1)


def _gemm(fn, m, n, k, A, B, rows, want_s):
    if rows is not None:
        rows = np.ascontiguousarray(rows, dtype=np.int32)
        if rows.size and (rows.min() < 0 or rows.max() >= m):
            raise ValueError("row index out of range")
        count = rows.size
    else:
        count = m
    C = np.zeros((count, n), dtype=np.float64)
    S = np.zeros((count, n), dtype=np.float64) if want_s else None
    if count and n:
        fn(m, n, k, A.ctypes.data, _ld(A), B.ctypes.data, _ld(B),
           rows.ctypes.data if rows is not None else None, count,
           C.ctypes.data, S.ctypes.data if want_s else None)
    return (C, S) if want_s else C


def nt_ref(A, B, rows=None, with_bound=False):
    """C = A x B^T (Eq. 2) in float64.  A is m x k, B is n x k (views with a row stride are fine).

    rows: optional row indices of C to compute.  with_bound: also return S = |A| x |B|^T.
    """
    A = _as_f32_2d(A, "A")
    B = _as_f32_2d(B, "B")
    if A.shape[1] != B.shape[1]:
        raise ValueError("A and B must have the same number of columns (k)")
    return _gemm(_load().oracle_nt_ref, A.shape[0], B.shape[0], A.shape[1], A, B, rows, with_bound)


def nn_ref(A, B, rows=None, with_bound=False):
    """C = A x B (Eq. 1) in float64.  A is m x k, B is k x n."""
    A = _as_f32_2d(A, "A")
    B = _as_f32_2d(B, "B")
    if A.shape[1] != B.shape[0]:
        raise ValueError("A columns must equal B rows (k)")
    return _gemm(_load().oracle_nn_ref, A.shape[0], B.shape[1], A.shape[1], A, B, rows, with_bound)


def transpose_ref(X, ldout=None, fill=np.nan):
    """Out-of-place transpose of a float32 matrix, copied as 32-bit words (B^T_{ji} = B_{ij}).

    Returns a cols x rows view of a buffer whose leading dimension is ldout (>= rows);
    padding columns keep `fill`.
    """
    X = _as_f32_2d(X, "X")
    r, c = X.shape
    ldout = r if ldout is None else int(ldout)
    if ldout < r:
        raise ValueError("ldout must be >= rows of the input")
    buf = np.full((c, max(ldout, 1)), fill, dtype=np.float32)
    if r and c:
        _load().oracle_transpose_ref(r, c, X.ctypes.data, _ld(X), buf.ctypes.data, max(ldout, 1))
    return buf[:, :r]


def tnn_ref(A, B, rows=None, with_bound=False):
    """Algorithm 1 on the CPU: transpose B, then the NN product.  Used to test the oracle against itself."""
    return nn_ref(A, np.ascontiguousarray(transpose_ref(B)), rows=rows, with_bound=with_bound)


def _f64(x, name):
    x = np.ascontiguousarray(x, dtype=np.float64)
    if x.ndim != 2:
        raise ValueError(f"{name} must be 2-D")
    return x


def nt_f64(A, B):
    """A x B^T (Eq. 2) on float64 operands: A m x k, B n x k."""
    A, B = _f64(A, "A"), _f64(B, "B")
    if A.shape[1] != B.shape[1]:
        raise ValueError("A and B must have the same number of columns (k)")
    C = np.zeros((A.shape[0], B.shape[0]), dtype=np.float64)
    if C.size:
        _load().oracle_f64_nt(A.shape[0], B.shape[0], A.shape[1], A.ctypes.data, B.ctypes.data, C.ctypes.data)
    return C


def nn_f64(A, B):
    """A x B (Eq. 1) on float64 operands: A m x k, B k x n."""
    A, B = _f64(A, "A"), _f64(B, "B")
    if A.shape[1] != B.shape[0]:
        raise ValueError("A columns must equal B rows (k)")
    C = np.zeros((A.shape[0], B.shape[1]), dtype=np.float64)
    if C.size:
        _load().oracle_f64_nn(A.shape[0], B.shape[1], A.shape[1], A.ctypes.data, B.ctypes.data, C.ctypes.data)
    return C


def tn_f64(A, B):
    """A^T x B on float64 operands: A k x m, B k x n, the sum running over the shared row index."""
    A, B = _f64(A, "A"), _f64(B, "B")
    if A.shape[0] != B.shape[0]:
        raise ValueError("A and B must have the same number of rows (k)")
    C = np.zeros((A.shape[1], B.shape[1]), dtype=np.float64)
    if C.size:
        _load().oracle_f64_tn(A.shape[1], B.shape[1], A.shape[0], A.ctypes.data, B.ctypes.data, C.ctypes.data)
    return C
