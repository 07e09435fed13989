"""Seeded synthetic inputs for the SGEMM workloads (and, at the end, for the 2D convolution).
This module holds no GEMM, convolution or tuner arithmetic: it only draws matrices.  It is the one module that both the tests' oracle side
and the GPU side take their inputs from.

Recipe: numpy's PCG64 generator seeded with the workload's seed; matrices are drawn in the
order A, B, C, each as float32 in its *stored* shape (A is K x M when layout bit 0 is set,
B is N x K when bit 1 is set, C is M x N).  `dist` is "uniform" (i.i.d. on [-1, 1)) or
"normal" (i.i.d. N(0, 1)).
"""
from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    M: int
    N: int
    K: int
    alpha: float
    beta: float
    layout: int
    seed: int
    dist: str


# The benchmark configurations, one entry per problem shape.
WORKLOADS = {
    "cfg1_256": Workload("cfg1_256", 256, 256, 256, 1.0, 0.0, 0, 0, "uniform"),
    "cfg2_2048": Workload("cfg2_2048", 2048, 2048, 2048, 2.0, 0.5, 0, 1, "uniform"),
    "cfg3_1000": Workload("cfg3_1000", 1000, 1000, 1000, 1.0, 1.0, 0, 2, "uniform"),
    "cfg3_1536": Workload("cfg3_1536", 1536, 1536, 1536, 1.0, 1.0, 0, 2, "uniform"),
    "cfg3_3000": Workload("cfg3_3000", 3000, 3000, 3000, 1.0, 1.0, 0, 2, "uniform"),
    "cfg4_4096": Workload("cfg4_4096", 4096, 4096, 4096, 1.0, 0.0, 0, 3, "normal"),
    "cfg4_8192": Workload("cfg4_8192", 8192, 8192, 8192, 1.0, 0.0, 0, 3, "normal"),
    "cfg5_128x4096x4096": Workload("cfg5_128x4096x4096", 128, 4096, 4096, 1.0, 0.0, 1, 4,
                                   "uniform"),
    "cfg5_4096x64x9216": Workload("cfg5_4096x64x9216", 4096, 64, 9216, 1.0, 0.0, 1, 4,
                                  "uniform"),
}


def _draw(rng, shape, dist):
    if dist == "uniform":
        return rng.uniform(-1.0, 1.0, size=shape).astype(np.float32)
    if dist == "normal":
        return rng.standard_normal(size=shape, dtype=np.float32)
    if dist == "smallint":          # integers in [-3, 3]: every summation order is exact
        return rng.integers(-3, 4, size=shape).astype(np.float32)
    raise ValueError(f"unknown distribution {dist!r}")


def stored_shapes(M, N, K, layout):
    a = (K, M) if layout & 1 else (M, K)
    b = (N, K) if layout & 2 else (K, N)
    return a, b, (M, N)


def make_inputs(M, N, K, layout=0, seed=0, dist="uniform"):
    """(A, B, C) as float32 host arrays in stored shapes, drawn in that order."""
    rng = np.random.default_rng(seed)
    sa, sb, sc = stored_shapes(M, N, K, layout)
    A = _draw(rng, sa, dist)
    B = _draw(rng, sb, dist)
    C = _draw(rng, sc, dist)
    return A, B, C


def make_workload(w: Workload):
    return make_inputs(w.M, w.N, w.K, w.layout, w.seed, w.dist)


def sample_positions(M, N, seed, rows=64, cols=64, scattered=4096, edge=128):
    """(row_idx, col_idx) pairs for sampled checks at sizes the oracle cannot cover in full:
    `rows` whole rows, `cols` whole columns, the last `edge` rows and columns of the matrix
    (edge tiles) sub-sampled, and `scattered` uniformly random elements."""
    rng = np.random.default_rng(seed ^ 0x5EED)
    r_list, c_list = [], []
    pick_r = rng.choice(M, size=min(rows, M), replace=False)
    for r in pick_r:
        r_list.append(np.full(N, r)); c_list.append(np.arange(N))
    pick_c = rng.choice(N, size=min(cols, N), replace=False)
    for c in pick_c:
        r_list.append(np.arange(M)); c_list.append(np.full(M, c))
    e = min(edge, M, N)
    er = rng.integers(M - e, M, size=scattered // 4) if e else np.zeros(0, dtype=np.int64)
    ec = rng.integers(N - e, N, size=scattered // 4) if e else np.zeros(0, dtype=np.int64)
    r_list.append(er); c_list.append(rng.integers(0, N, size=er.size))
    r_list.append(rng.integers(0, M, size=ec.size)); c_list.append(ec)
    r_list.append(rng.integers(0, M, size=scattered)); c_list.append(rng.integers(0, N, size=scattered))
    r = np.concatenate(r_list).astype(np.int32)
    c = np.concatenate(c_list).astype(np.int32)
    return r, c


# ---- 2D convolution (the paper's first case study) --------------------------------------------
@dataclass(frozen=True)
class ConvWorkload:
    name: str
    X: int       # output width (fastest index)
    Y: int       # output height
    Xf: int      # filter width
    Yf: int      # filter height
    w: float     # weighing factor
    seed: int


# The paper's image (8192 by 4096) with its three filter sizes, and a small case.
CONV_WORKLOADS = {
    "conv_small_5x5": ConvWorkload("conv_small_5x5", 300, 200, 5, 5, 0.04, 10),
    "conv_3x3": ConvWorkload("conv_3x3", 8192, 4096, 3, 3, 1.0 / 9, 11),
    "conv_7x7": ConvWorkload("conv_7x7", 8192, 4096, 7, 7, 1.0 / 49, 12),
    "conv_11x11": ConvWorkload("conv_11x11", 8192, 4096, 11, 11, 1.0 / 121, 13),
    # not a multiple of any workgroup tile: the guarded builds
    "conv_7x7_ragged": ConvWorkload("conv_7x7_ragged", 8190, 4090, 7, 7, 1.0 / 49, 14),
}


def make_conv_inputs(X, Y, Xf, Yf, seed, dist="uniform", lda=None):
    """The input image WITH its halo, (Y + Yf - 1) x lda float32 with lda >= X + Xf - 1, and the
    filter, Yf x Xf float32; drawn in that order from PCG64(seed)."""
    rng = np.random.default_rng(seed)
    lda = lda or X + Xf - 1
    A = _draw(rng, (Y + Yf - 1, lda), dist)
    F = _draw(rng, (Yf, Xf), dist)
    return A, F


def make_conv_workload(w: ConvWorkload):
    """Rows of the stored image are padded to a multiple of 16 floats (64-byte aligned rows)."""
    return make_conv_inputs(w.X, w.Y, w.Xf, w.Yf, w.seed, lda=(w.X + w.Xf - 1 + 15) // 16 * 16)
