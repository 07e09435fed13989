"""Python face of the blocked multithreaded CPU SGEMM (oracle/cpu_blocked_sgemm.c): a reported
baseline, checked against the oracle, never used by the product."""
import ctypes

import numpy as np

from . import build as _build

_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(_build.build_baseline(force=False))
        fp = ctypes.POINTER(ctypes.c_float)
        lib.cpu_blocked_sgemm.argtypes = [ctypes.c_int] * 3 + [ctypes.c_float, fp, ctypes.c_int, fp,
                                                               ctypes.c_int, ctypes.c_float, fp,
                                                               ctypes.c_int, ctypes.c_int]
        lib.cpu_blocked_sgemm.restype = None
        lib.cpu_blocked_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def threads():
    return int(_load().cpu_blocked_threads())


def sgemm(alpha, A, B, beta, C, layout=0):
    """C_out (float32) for stored-shape 2-D inputs; C is not modified."""
    A = np.ascontiguousarray(A, dtype=np.float32)
    B = np.ascontiguousarray(B, dtype=np.float32)
    out = np.array(C, dtype=np.float32, order="C", copy=True)
    M, N = out.shape
    K = A.shape[0] if layout & 1 else A.shape[1]
    fp = ctypes.POINTER(ctypes.c_float)
    _load().cpu_blocked_sgemm(M, N, K, alpha, A.ctypes.data_as(fp), max(A.shape[1], 1),
                              B.ctypes.data_as(fp), max(B.shape[1], 1), beta,
                              out.ctypes.data_as(fp), max(N, 1), layout)
    return out
