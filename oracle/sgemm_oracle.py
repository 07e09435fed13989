"""Python face of the C oracle (oracle/sgemm_oracle.c).  TEST INFRASTRUCTURE ONLY.

`sgemm(...)` returns the plain-definition result of the paper's matrix-multiplication case
study (first equation of that section), C = alpha*op(A)*op(B) + beta*C, as float64;
`sgemm_sample(...)` returns the same values for chosen (row, col) pairs; `tolerance(...)`
is the per-element error bound every GPU variant must meet:
    |C_gpu - C_ref| <= 1e-5 * K * max|a| * max|b| + 1e-6 * |C_ref|.
`sgemm_python(...)` is an independent pure-Python loop used only to pin the C code on tiny
inputs.
"""
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
        fp = ctypes.POINTER(ctypes.c_float)
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int)
        lib.oracle_sgemm.argtypes = [ctypes.c_int] * 3 + [ctypes.c_float, fp, ctypes.c_int, fp,
                                                          ctypes.c_int, ctypes.c_float, fp,
                                                          ctypes.c_int, ctypes.c_int, dp]
        lib.oracle_sgemm.restype = None
        lib.oracle_sgemm_sample.argtypes = [ctypes.c_int] * 3 + [ctypes.c_float, fp, ctypes.c_int,
                                                                 fp, ctypes.c_int, ctypes.c_float,
                                                                 fp, ctypes.c_int, ctypes.c_int,
                                                                 ctypes.c_longlong, ip, ip, dp]
        lib.oracle_sgemm_sample.restype = None
        lib.oracle_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def threads() -> int:
    return int(_load().oracle_threads())


def _f32(x):
    x = np.ascontiguousarray(x, dtype=np.float32)
    return x, x.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def _dims(A, B, layout):
    """(M, N, K, lda, ldb) from the stored 2-D arrays and the layout bits."""
    if layout & 1:
        K, M = A.shape
    else:
        M, K = A.shape
    if layout & 2:
        N, Kb = B.shape
    else:
        Kb, N = B.shape
    if K != Kb:
        raise ValueError("inner dimensions differ")
    return M, N, K, A.shape[1], B.shape[1]


def sgemm(alpha, A, B, beta, C_in, layout=0):
    """Full oracle result as an (M, N) float64 array.  A, B, C_in are 2-D arrays in their
    *stored* shapes (A is K x M when layout bit 0 is set, B is N x K when bit 1 is set);
    a leading dimension larger than the row length is expressed by passing a view's base
    array through `sgemm_ld`."""
    A, pa = _f32(A)
    B, pb = _f32(B)
    M, N, K, lda, ldb = _dims(A, B, layout)
    if C_in is None:
        C_in = np.zeros((M, N), dtype=np.float32)
    C_in, pc = _f32(C_in)
    out = np.empty((M, N), dtype=np.float64)
    _load().oracle_sgemm(M, N, K, alpha, pa, max(lda, 1), pb, max(ldb, 1), beta, pc,
                         max(C_in.shape[1], 1), layout,
                         out.ctypes.data_as(ctypes.POINTER(ctypes.c_double)))
    return out


def sgemm_ld(M, N, K, alpha, A, lda, B, ldb, beta, C_in, ldc, layout=0):
    """Same, with explicit leading dimensions over flat float32 buffers."""
    A, pa = _f32(A)
    B, pb = _f32(B)
    C_in, pc = _f32(C_in)
    out = np.empty((M, N), dtype=np.float64)
    _load().oracle_sgemm(M, N, K, alpha, pa, lda, pb, ldb, beta, pc, ldc, layout,
                         out.ctypes.data_as(ctypes.POINTER(ctypes.c_double)))
    return out


def sgemm_sample(alpha, A, B, beta, C_in, rows, cols, layout=0):
    """Oracle values at the (rows[s], cols[s]) positions only, as float64."""
    A, pa = _f32(A)
    B, pb = _f32(B)
    M, N, K, lda, ldb = _dims(A, B, layout)
    if C_in is None:
        C_in = np.zeros((1, 1), dtype=np.float32)
        beta = 0.0
    C_in, pc = _f32(C_in)
    rows = np.ascontiguousarray(rows, dtype=np.int32)
    cols = np.ascontiguousarray(cols, dtype=np.int32)
    if rows.shape != cols.shape:
        raise ValueError("rows and cols differ in length")
    if rows.size and (rows.min() < 0 or rows.max() >= M or cols.min() < 0 or cols.max() >= N):
        raise ValueError("sample index out of range")
    out = np.empty(rows.shape, dtype=np.float64)
    ip = ctypes.POINTER(ctypes.c_int)
    _load().oracle_sgemm_sample(M, N, K, alpha, pa, max(lda, 1), pb, max(ldb, 1), beta, pc,
                                max(C_in.shape[1], 1), layout, rows.size,
                                rows.ctypes.data_as(ip), cols.ctypes.data_as(ip),
                                out.ctypes.data_as(ctypes.POINTER(ctypes.c_double)))
    return out


def tolerance(K, amax, bmax, C_ref):
    """Per-element bound on |C_gpu - C_ref|, applied literally."""
    return 1e-5 * K * float(amax) * float(bmax) + 1e-6 * np.abs(np.asarray(C_ref, dtype=np.float64))


def sgemm_python(alpha, A, B, beta, C_in, layout=0):
    """Pure-Python loops over Python floats (which are IEEE doubles): a second, independent
    writing of the definition, for tiny inputs only."""
    A = np.asarray(A, dtype=np.float32)
    B = np.asarray(B, dtype=np.float32)
    M, N, K, _, _ = _dims(A, B, layout)
    out = [[0.0] * N for _ in range(M)]
    for j in range(N):            # deliberately a different loop order from the C code
        for i in range(M):
            s = 0.0
            if alpha != 0:
                for k in range(K):
                    a = float(A[k][i]) if layout & 1 else float(A[i][k])
                    b = float(B[j][k]) if layout & 2 else float(B[k][j])
                    s += a * b
            r = float(np.float32(alpha)) * s
            if beta != 0:
                r += float(np.float32(beta)) * float(np.float32(C_in[i][j]))
            out[i][j] = r
    return np.array(out, dtype=np.float64).reshape(M, N)
