"""Helpers of the GPU parity tests: run one configuration through the C ABI on torch device
tensors and compare it element by element with the CPU oracle under the stated bound
    |C_gpu - C_ref| <= 1e-5 * K * max|a| * max|b| + 1e-6 * |C_ref|."""
import numpy as np

from oracle import sgemm_oracle as orc
from paper_1703_06503_amd import binding as b


def run_gpu(cfg, A, B, C, alpha, beta, layout=0, entry="config"):
    """C_out (numpy float32) of one call through the C ABI; A, B, C are host arrays in stored
    shapes.  entry = "config" -> sgemm_run_config(cfg), "tuned" -> sgemm_tuned,
    "reference" -> sgemm_reference."""
    import torch
    M, N = C.shape
    K = A.shape[0] if layout & 1 else A.shape[1]
    dA = torch.from_numpy(np.ascontiguousarray(A)).cuda()
    dB = torch.from_numpy(np.ascontiguousarray(B)).cuda()
    dC = torch.from_numpy(np.ascontiguousarray(C)).cuda()
    lda, ldb, ldc = max(A.shape[1], 1), max(B.shape[1], 1), max(N, 1)
    if entry == "config":
        b.sgemm_run_config(None, cfg, M, N, K, alpha, dA, lda, dB, ldb, beta, dC, ldc, layout)
    elif entry == "padded":
        b.sgemm_run_config_padded(None, cfg, M, N, K, alpha, dA, lda, dB, ldb, beta, dC, ldc, layout)
    elif entry == "tuned":
        b.sgemm_tuned_on(None, M, N, K, alpha, dA, lda, dB, ldb, beta, dC, ldc, layout)
    elif entry == "reference":
        b.sgemm_reference(None, M, N, K, alpha, dA, lda, dB, ldb, beta, dC, ldc, layout)
    else:
        raise ValueError(entry)
    torch.cuda.synchronize()
    return dC.cpu().numpy()


def check_against_oracle(got, A, B, C, alpha, beta, layout=0, ref=None, what=""):
    K = A.shape[0] if layout & 1 else A.shape[1]
    if ref is None:
        ref = orc.sgemm(alpha, A, B, beta, C, layout)
    amax = float(np.max(np.abs(A))) if A.size else 0.0
    bmax = float(np.max(np.abs(B))) if B.size else 0.0
    tol = orc.tolerance(K, amax, bmax, ref)
    err = np.abs(got.astype(np.float64) - ref)
    bad = ~(err <= tol)
    if bad.any():
        i, j = np.unravel_index(np.argmax(np.where(bad, err, 0)), err.shape)
        raise AssertionError(f"{what}: {int(bad.sum())} elements outside the bound; worst at "
                             f"({i},{j}): got {got[i, j]!r}, oracle {ref[i, j]!r}, bound {tol[i, j]:.3e}")
    return float(np.max(err / np.maximum(tol, 1e-300))) if err.size else 0.0
