"""Pins for the CPU GEMM oracle: each test fixes it to something other than itself (closed
forms, structural identities, an independent pure-Python loop, numpy's fp64 matmul).  The
paper prints no worked numeric GEMM example, so there is nothing to pin from its text beyond
the definition C = alpha*A^T*B + beta*C of its matrix-multiplication case study."""
import itertools

import numpy as np
import pytest

from oracle import sgemm_oracle as orc
from paper_1703_06503_amd import synth


def test_identity_left_gives_alpha_B_plus_beta_C():
    rng = np.random.default_rng(10)
    n, m = 37, 23
    B = rng.uniform(-1, 1, (m, n)).astype(np.float32)
    C = rng.uniform(-1, 1, (m, n)).astype(np.float32)
    I = np.eye(m, dtype=np.float32)
    out = orc.sgemm(2.0, I, B, 0.5, C)
    expect = 2.0 * B.astype(np.float64) + 0.5 * C.astype(np.float64)
    assert np.array_equal(out, expect)          # one non-zero term per sum: exact


def test_identity_right_gives_A():
    rng = np.random.default_rng(11)
    A = rng.uniform(-1, 1, (19, 31)).astype(np.float32)
    out = orc.sgemm(1.0, A, np.eye(31, dtype=np.float32), 0.0, None)
    assert np.array_equal(out, A.astype(np.float64))


def test_permutation_matrix_permutes_rows_exactly():
    rng = np.random.default_rng(12)
    m, n = 29, 17
    perm = rng.permutation(m)
    P = np.zeros((m, m), dtype=np.float32)
    P[np.arange(m), perm] = 1.0                 # (P B)[i] = B[perm[i]]
    B = rng.standard_normal((m, n)).astype(np.float32)
    out = orc.sgemm(1.0, P, B, 0.0, None)
    assert np.array_equal(out, B[perm].astype(np.float64))
    # and a permutation on the right permutes columns: (A Q)[:, j] = A[:, src[j]]
    q = rng.permutation(n)
    Q = np.zeros((n, n), dtype=np.float32)
    Q[q, np.arange(n)] = 1.0
    A = rng.standard_normal((m, n)).astype(np.float32)
    assert np.array_equal(orc.sgemm(1.0, A, Q, 0.0, None), A[:, q].astype(np.float64))


@pytest.mark.parametrize("M,N,K", [(5, 7, 11), (16, 9, 368), (3, 4, 1000)])
def test_rank1_closed_forms(M, N, K):
    i = np.arange(1, M + 1, dtype=np.float32)[:, None]
    j = np.arange(1, N + 1, dtype=np.float32)[None, :]
    k = np.arange(1, K + 1, dtype=np.float32)
    # A(i,k) = i+1, B(k,j) = j+1  =>  K (i+1)(j+1)
    A = np.repeat(i, K, axis=1)
    B = np.repeat(j, K, axis=0)
    assert np.array_equal(orc.sgemm(1.0, A, B, 0.0, None), K * (i.astype(np.float64) * j))
    # A(i,k) = k+1, B = 1  =>  K(K+1)/2
    A = np.repeat(k[None, :], M, axis=0)
    B = np.ones((K, N), dtype=np.float32)
    assert np.array_equal(orc.sgemm(1.0, A, B, 0.0, None), np.full((M, N), K * (K + 1) / 2))
    # A(i,k) = B(k,j) = k+1  =>  K(K+1)(2K+1)/6
    B = np.repeat(k[:, None], N, axis=1)
    assert np.array_equal(orc.sgemm(1.0, A, B, 0.0, None),
                          np.full((M, N), K * (K + 1) * (2 * K + 1) / 6))


def test_alpha_beta_edge_cases():
    rng = np.random.default_rng(13)
    A = rng.uniform(-1, 1, (9, 13)).astype(np.float32)
    B = rng.uniform(-1, 1, (13, 6)).astype(np.float32)
    C = rng.uniform(-1, 1, (9, 6)).astype(np.float32)
    # (alpha, beta) = (0, 1): C unchanged, even if A and B hold NaN (they are not read)
    An = A.copy(); An[2, 3] = np.nan
    assert np.array_equal(orc.sgemm(0.0, An, B, 1.0, C), C.astype(np.float64))
    # (0, 0): zeros even with NaN in C
    Cn = C.copy(); Cn[1, 1] = np.nan; Cn[0, 5] = np.inf
    assert np.array_equal(orc.sgemm(0.0, A, B, 0.0, Cn), np.zeros((9, 6)))
    # (1, 0) with NaN/Inf in C: C is not read
    out = orc.sgemm(1.0, A, B, 0.0, Cn)
    assert np.all(np.isfinite(out))
    assert np.array_equal(out, orc.sgemm(1.0, A, B, 0.0, None))
    # beta != 0 does read C: the NaN must propagate to exactly that element
    out = orc.sgemm(1.0, A, B, 1.0, Cn)
    assert np.isnan(out[1, 1]) and np.isinf(out[0, 5]) and np.isfinite(out).sum() == out.size - 2
    # (1, -1) with C_in = float32(A B): the residual is only the float rounding of C_in
    AB = orc.sgemm(1.0, A, B, 0.0, None)
    C32 = AB.astype(np.float32)
    res = orc.sgemm(1.0, A, B, -1.0, C32)
    assert np.max(np.abs(res)) <= 2.0 ** -24 * np.max(np.abs(AB)) * 1.01
    # K = 0: C = beta * C
    A0 = np.zeros((9, 0), dtype=np.float32); B0 = np.zeros((0, 6), dtype=np.float32)
    assert np.array_equal(orc.sgemm(3.0, A0, B0, 0.5, C), 0.5 * C.astype(np.float64))


def test_alpha_power_of_two_scales_exactly():
    rng = np.random.default_rng(14)
    A = rng.uniform(-1, 1, (12, 40)).astype(np.float32)
    B = rng.uniform(-1, 1, (40, 15)).astype(np.float32)
    one = orc.sgemm(1.0, A, B, 0.0, None)
    assert np.array_equal(orc.sgemm(2.0, A, B, 0.0, None), 2.0 * one)
    assert np.array_equal(orc.sgemm(-0.25, A, B, 0.0, None), -0.25 * one)


@pytest.mark.parametrize("layout", [0, 1, 2, 3])
def test_brute_force_tiny_integer_inputs_all_shapes(layout):
    """All M,N,K in 1..5 with small integers: sums are exact in any order, so the C code, a
    pure-Python loop in another loop order and integer numpy arithmetic must agree exactly."""
    rng = np.random.default_rng(15 + layout)
    for M, N, K in itertools.product(range(1, 6), repeat=3):
        Al = rng.integers(-3, 4, (M, K)); Bl = rng.integers(-3, 4, (K, N))
        Cl = rng.integers(-3, 4, (M, N))
        A = (Al.T if layout & 1 else Al).astype(np.float32)
        B = (Bl.T if layout & 2 else Bl).astype(np.float32)
        C = Cl.astype(np.float32)
        got = orc.sgemm(2.0, A, B, -3.0, C, layout)
        assert np.array_equal(got, (2 * (Al @ Bl) - 3 * Cl).astype(np.float64)), (M, N, K)
        assert np.array_equal(got, orc.sgemm_python(2.0, A, B, -3.0, C, layout)), (M, N, K)


@pytest.mark.parametrize("layout", [1, 2, 3])
def test_transposed_storage_equals_row_major_bit_for_bit(layout):
    rng = np.random.default_rng(16)
    A = rng.standard_normal((21, 34)).astype(np.float32)
    B = rng.standard_normal((34, 18)).astype(np.float32)
    C = rng.standard_normal((21, 18)).astype(np.float32)
    base = orc.sgemm(1.5, A, B, 0.75, C, 0)
    At = np.ascontiguousarray(A.T) if layout & 1 else A
    Bt = np.ascontiguousarray(B.T) if layout & 2 else B
    assert np.array_equal(orc.sgemm(1.5, At, Bt, 0.75, C, layout), base)


def test_non_square_random_against_numpy_fp64_matmul():
    """A transposed operand, a swapped index or a dropped term cannot survive this: numpy's
    double-precision matmul is an independent library routine; only rounding order differs."""
    rng = np.random.default_rng(17)
    for (M, N, K) in [(33, 65, 129), (100, 7, 257), (1, 50, 64), (64, 1, 50)]:
        A = rng.uniform(-1, 1, (M, K)).astype(np.float32)
        B = rng.uniform(-1, 1, (K, N)).astype(np.float32)
        C = rng.uniform(-1, 1, (M, N)).astype(np.float32)
        got = orc.sgemm(1.25, A, B, -0.5, C)
        ref = 1.25 * (A.astype(np.float64) @ B.astype(np.float64)) - 0.5 * C.astype(np.float64)
        assert np.max(np.abs(got - ref)) < 1e-12 * K


def test_leading_dimensions_are_honoured():
    rng = np.random.default_rng(18)
    M, N, K, lda, ldb, ldc = 7, 9, 11, 16, 13, 10
    Abuf = rng.uniform(-1, 1, (M, lda)).astype(np.float32)
    Bbuf = rng.uniform(-1, 1, (K, ldb)).astype(np.float32)
    Cbuf = rng.uniform(-1, 1, (M, ldc)).astype(np.float32)
    got = orc.sgemm_ld(M, N, K, 1.0, Abuf, lda, Bbuf, ldb, 2.0, Cbuf, ldc, 0)
    ref = orc.sgemm(1.0, Abuf[:, :K], Bbuf[:, :N], 2.0, Cbuf[:, :N], 0)
    assert np.array_equal(got, ref)


def test_sample_matches_full_oracle():
    A, B, C = synth.make_inputs(70, 90, 50, layout=1, seed=3)
    full = orc.sgemm(0.5, A, B, 2.0, C, 1)
    r, c = synth.sample_positions(70, 90, seed=3, rows=4, cols=4, scattered=64, edge=16)
    assert np.array_equal(orc.sgemm_sample(0.5, A, B, 2.0, C, r, c, 1), full[r, c])


def test_planted_mistakes_are_caught():
    """The pins are only worth something if plausible mistakes fail them: plant each mistake
    in a copy of the definition and check that a pin above would reject it."""
    rng = np.random.default_rng(19)
    M, N, K = 6, 5, 7
    A = rng.integers(-3, 4, (M, K)).astype(np.float32)
    B = rng.integers(-3, 4, (K, N)).astype(np.float32)
    C = rng.integers(-3, 4, (M, N)).astype(np.float32)
    good = orc.sgemm(2.0, A, B, -3.0, C)
    A64, B64, C64 = (x.astype(np.float64) for x in (A, B, C))
    wrong = {
        "dropped last k term": 2 * (A64[:, :-1] @ B64[:-1]) - 3 * C64,
        "beta sign": 2 * (A64 @ B64) + 3 * C64,
        "alpha applied to C": 2 * (A64 @ B64 - 3 * C64),
    }
    for name, w in wrong.items():
        assert not np.array_equal(good, w), name
    # operands swapped (B A instead of A B) on square inputs
    sq = rng.integers(-3, 4, (5, 5)).astype(np.float32)
    sq2 = rng.integers(-3, 4, (5, 5)).astype(np.float32)
    assert not np.array_equal(orc.sgemm(1.0, sq, sq2, 0.0, None),
                              (sq2.astype(np.float64) @ sq.astype(np.float64)))


def test_tolerance_formula():
    C = np.array([[0.0, -2.0], [1e6, 3.0]])
    tol = orc.tolerance(100, 0.5, 2.0, C)
    assert np.allclose(tol, 1e-5 * 100 * 1.0 + 1e-6 * np.abs(C), rtol=0, atol=1e-18)
