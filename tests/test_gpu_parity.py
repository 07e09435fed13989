"""GPU parity: every tested variant of the kernel family, driven through the C ABI, against
the CPU oracle, element by element.  Sizes span several workgroup tiles and ragged tails."""
import numpy as np
import pytest

from oracle import sgemm_oracle as orc
from paper_1703_06503_amd import binding as b
from paper_1703_06503_amd import synth
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu

# The fixed samples of the spaces, the shapes and the hand-picked configurations live in
# tests/variants.py (also read by tests/precompile_test_variants.py).
from tests.variants import (FULL_SAMPLE, MFMA_SAMPLE, EXT_SAMPLE, DIRECT_SAMPLE, KSPLIT_SAMPLE, EXACT_EXT, RAGGED_EXT,  # noqa: E402
                            EXACT_SHAPE, RAGGED_SHAPE, NARROW_SHAPE, RAGGED_BIG, ODD_SHAPE, BENCH_CONFIGS,
                            SKINNY_CONFIGS, sample_configs)
from tests.variants import some_configs as _some_configs  # noqa: E402


def _sweep(space, indices, shape, alpha, beta, layout, seed, dist="uniform"):
    M, N, K = shape
    A, B, C = synth.make_inputs(M, N, K, layout, seed, dist)
    ref = orc.sgemm(alpha, A, B, beta, C, layout)
    worst = 0.0
    for i in indices:
        cfg = b.sgemm_space_get(space, i)
        print(f"case space={space} index={i} {cfg} shape={shape} layout={layout}", flush=True)
        got = gu.run_gpu(cfg, A, B, C, alpha, beta, layout)
        worst = max(worst, gu.check_against_oracle(got, A, B, C, alpha, beta, layout, ref,
                                                   what=f"space {space} index {i} {cfg}"))
    return worst


def test_small_space_all_16_configs_at_256_cubed():
    """Benchmark configuration 1: 256^3, alpha=1, beta=0, uniform[-1,1] seed 0."""
    w = synth.WORKLOADS["cfg1_256"]
    assert b.sgemm_space_size(b.SPACE_SMALL) == 16
    worst = _sweep(b.SPACE_SMALL, range(16), (w.M, w.N, w.K), w.alpha, w.beta, w.layout, w.seed)
    assert worst <= 1.0


def test_full_space_sample_exact_tiles():
    _sweep(b.SPACE_FULL, sample_configs(**FULL_SAMPLE), EXACT_SHAPE, 2.0, 0.5, 0, seed=21)


def test_full_space_sample_ragged():
    _sweep(b.SPACE_FULL, sample_configs(**FULL_SAMPLE), RAGGED_SHAPE, 1.0, 1.0, 0, seed=22)


def test_mfma_space_sample_exact_tiles():
    _sweep(b.SPACE_MFMA, sample_configs(**MFMA_SAMPLE), EXACT_SHAPE, 1.0, 0.0, 0, seed=23,
           dist="normal")


def test_mfma_space_sample_ragged():
    _sweep(b.SPACE_MFMA, sample_configs(**MFMA_SAMPLE), RAGGED_BIG, -1.5, 0.25, 0, seed=24)


def test_ext_space_sample_exact_tiles():
    _sweep(b.SPACE_EXT, sample_configs(**EXT_SAMPLE), EXACT_EXT, 1.5, -0.5, 0, seed=25)


def test_ext_space_sample_ragged():
    _sweep(b.SPACE_EXT, sample_configs(**EXT_SAMPLE), RAGGED_EXT, 1.0, 1.0, 0, seed=26,
           dist="normal")


def test_direct_space_sample_exact_tiles():
    _sweep(b.SPACE_DIRECT, sample_configs(**DIRECT_SAMPLE), EXACT_EXT, 1.0, 0.0, 0, seed=27,
           dist="normal")


def test_direct_space_sample_ragged():
    idx = sample_configs(**DIRECT_SAMPLE)
    _sweep(b.SPACE_DIRECT, idx, RAGGED_EXT, 2.0, 0.5, 0, seed=28)
    # odd sizes: the stored rows end inside a 16-byte vector, so the loads are narrowed
    _sweep(b.SPACE_DIRECT, idx[::4], ODD_SHAPE, 1.0, 1.0, 0, seed=29)


def test_ksplit_space_sample():
    """Variants whose waves share out the K slab (KSW 2 and 4): exact tiles, ragged sizes, and
    odd sizes whose stored rows end inside a load vector."""
    idx = sample_configs(**KSPLIT_SAMPLE)
    _sweep(b.SPACE_KSPLIT, idx, EXACT_EXT, 1.0, 0.0, 0, seed=31, dist="normal")
    _sweep(b.SPACE_KSPLIT, idx, RAGGED_EXT, -0.5, 2.0, 0, seed=32)
    _sweep(b.SPACE_KSPLIT, idx[::4], ODD_SHAPE, 1.0, 1.0, 0, seed=33)


@pytest.mark.parametrize("layout", [1, 2, 3])
def test_ksplit_space_transposed_storage(layout):
    idx = sample_configs(b.SPACE_KSPLIT, 16, seed=400 + layout)
    _sweep(b.SPACE_KSPLIT, idx, EXACT_EXT, 1.0, 0.0, layout, seed=34 + layout)
    _sweep(b.SPACE_KSPLIT, idx, RAGGED_EXT, 1.5, -0.5, layout, seed=37 + layout)


@pytest.mark.parametrize("layout", [1, 2, 3])
def test_direct_space_transposed_storage(layout):
    idx = sample_configs(b.SPACE_DIRECT, 24, seed=300 + layout)
    _sweep(b.SPACE_DIRECT, idx, EXACT_EXT, 1.0, 0.0, layout, seed=80 + layout)
    _sweep(b.SPACE_DIRECT, idx, RAGGED_EXT, -1.0, 0.5, layout, seed=90 + layout)


@pytest.mark.parametrize("layout", [1, 2, 3])
def test_ext_space_transposed_storage(layout):
    idx = sample_configs(b.SPACE_EXT, 24, seed=200 + layout)
    _sweep(b.SPACE_EXT, idx, RAGGED_EXT, 0.75, 0.0, layout, seed=70 + layout)


@pytest.mark.parametrize("layout", [1, 2, 3])
def test_transposed_storage(layout):
    idx = sample_configs(b.SPACE_FULL, 40, seed=100 + layout)
    _sweep(b.SPACE_FULL, idx, EXACT_SHAPE, 1.0, 0.0, layout, seed=30 + layout)
    _sweep(b.SPACE_FULL, idx, RAGGED_SHAPE, 0.5, 2.0, layout, seed=40 + layout)


WHICH = list(range(12))


@pytest.mark.parametrize("layout", [0, 1, 2, 3])
def test_tile_edges_of_five_and_seven_times_a_power_of_two(layout):
    """Tiles of 160, 224, 80 x 112 and 112 x 80: on a shape that all of them divide and on a
    ragged one, beta != 0, every storage layout."""
    from tests.variants import ODD_EDGE_CONFIGS, ODD_EDGE_SHAPES
    for shape in ODD_EDGE_SHAPES:
        A, B, C = synth.make_inputs(*shape, layout, seed=61 + layout)
        ref = orc.sgemm(0.75, A, B, -1.25, C, layout)
        for cfg in ODD_EDGE_CONFIGS:
            print(f"case {cfg} shape={shape} layout={layout}", flush=True)
            got = gu.run_gpu(cfg, A, B, C, 0.75, -1.25, layout)
            gu.check_against_oracle(got, A, B, C, 0.75, -1.25, layout, ref, what=f"{cfg} {shape} layout {layout}")


def test_dispatch_picks_odd_tile_edges_where_they_fill_the_cus():
    """2560 = 16 x 160 and 3584 = 16 x 224: the built-in rule takes those tiles (no entry in the
    table is near enough in K), and the calls are right."""
    for (M, N, K, layout), edge in [((2560, 2560, 1536, 0), 160), ((3584, 3584, 1024, 3), 224)]:
        cfg = b.sgemm_config_select(M, N, K, layout)
        assert (cfg.mwg, cfg.nwg) == (edge, edge), cfg
        A, B, C = synth.make_inputs(M, N, K, layout, seed=62)
        got = gu.run_gpu(None, A, B, C, 1.0, 0.5, layout, entry="tuned")
        gu.check_against_oracle(got, A, B, C, 1.0, 0.5, layout, what=f"{(M, N, K)} layout {layout} {cfg}")


@pytest.mark.parametrize("which", WHICH)
def test_integer_inputs_are_bit_exact(which):
    """Small-integer operands: every summation order gives the same float, so the GPU must
    equal the oracle exactly, whatever the tiling or MFMA blocking."""
    cfg = _some_configs()[which]
    assert b.sgemm_config_check(cfg) == 0
    for shape in [(256, 256, 64), (130, 70, 33), (1, 1, 1), (5, 300, 2), (200, 100, 300)]:
        M, N, K = shape
        A, B, C = synth.make_inputs(M, N, K, 0, seed=50, dist="smallint")
        got = gu.run_gpu(cfg, A, B, C, 2.0, -3.0)
        assert np.array_equal(got.astype(np.float64), orc.sgemm(2.0, A, B, -3.0, C)), shape


@pytest.mark.parametrize("which", WHICH)
def test_permutation_matrix_is_bit_exact(which):
    cfg = _some_configs()[which]
    rng = np.random.default_rng(51)
    m, n = 192, 160
    perm = rng.permutation(m)
    P = np.zeros((m, m), dtype=np.float32)
    P[np.arange(m), perm] = 1.0
    B = rng.standard_normal((m, n)).astype(np.float32)
    got = gu.run_gpu(cfg, P, B, np.zeros((m, n), np.float32), 1.0, 0.0)
    assert np.array_equal(got, B[perm])


@pytest.mark.parametrize("which", WHICH)
def test_alpha_beta_edge_cases(which):
    cfg = _some_configs()[which]
    A, B, C = synth.make_inputs(150, 140, 60, 0, seed=52)
    Cn = C.copy()
    Cn[3, 5] = np.nan
    Cn[149, 139] = np.inf
    # beta == 0: NaN/Inf in C must not reach the result
    got = gu.run_gpu(cfg, A, B, Cn, 1.0, 0.0)
    assert np.all(np.isfinite(got))
    gu.check_against_oracle(got, A, B, Cn, 1.0, 0.0)
    # alpha == 0: A and B are not read (NaN there is harmless); C = beta*C exactly
    An = A.copy()
    An[0, 0] = np.nan
    got = gu.run_gpu(cfg, An, B, C, 0.0, 1.0)
    assert np.array_equal(got, C)
    got = gu.run_gpu(cfg, An, B, Cn, 0.0, 0.0)
    assert np.array_equal(got, np.zeros_like(C))
    got = gu.run_gpu(cfg, A, B, C, 0.0, 0.5)
    assert np.array_equal(got, (0.5 * C).astype(np.float32))
    # beta != 0 reads C: NaN and Inf land exactly where they were
    got = gu.run_gpu(cfg, A, B, Cn, 1.0, 1.0)
    assert np.isnan(got[3, 5]) and np.isinf(got[149, 139])
    assert np.isfinite(got).sum() == got.size - 2
    # (1, -1) with C_in = A B: residual within the bound around zero
    AB = orc.sgemm(1.0, A, B, 0.0, None).astype(np.float32)
    got = gu.run_gpu(cfg, A, B, AB, 1.0, -1.0)
    gu.check_against_oracle(got, A, B, AB, 1.0, -1.0)


@pytest.mark.parametrize("which", WHICH)
def test_leading_dimensions_and_untouched_padding(which):
    """ld > row length, unaligned for vector access; elements of C outside M x N stay
    bit-identical, including guard rows after the matrix."""
    import torch
    cfg = _some_configs()[which]
    _check_leading_dimensions(cfg, 97, 83, 45, 51, 90, 89)
    # aligned leading dimensions, but rows that end inside a 16-byte vector
    _check_leading_dimensions(cfg, 97, 83, 45, 48, 84, 84)


@pytest.mark.parametrize("layout", [0, 1, 2, 3])
@pytest.mark.parametrize("which", [0, 1, 3, 4, 6, 10])
def test_what_lies_beside_the_matrices_is_never_summed(which, layout):
    """Guarded builds read through windows that end with the matrix and clamp nothing: whatever
    a lane picks up beyond M, N or K - here NaN in the padding of every stored row and in guard
    rows behind A and B - must not reach C.  Sizes are ragged in all three dimensions."""
    import torch
    cfg = _some_configs()[which]
    for (M, N, K), pad in [((97, 83, 45), 3), ((150, 140, 60), 4), ((64, 64, 64), 8)]:
        A, B, C = synth.make_inputs(M, N, K, layout, seed=91 + layout)
        def framed(X):      # the matrix with `pad` NaN columns on the right and two NaN rows below
            out = np.full((X.shape[0] + 2, X.shape[1] + pad), np.nan, dtype=np.float32)
            out[:X.shape[0], :X.shape[1]] = X
            return out
        dA, dB, dC = (torch.from_numpy(x).cuda() for x in (framed(A), framed(B), C.copy()))
        b.sgemm_run_config(None, cfg, M, N, K, 1.5, dA, A.shape[1] + pad, dB, B.shape[1] + pad, 0.25, dC, N, layout)
        torch.cuda.synchronize()
        gu.check_against_oracle(dC.cpu().numpy(), A, B, C, 1.5, 0.25, layout, what=f"NaN frame {cfg} {(M, N, K)} layout {layout}")


def test_leading_dimensions_up_to_the_documented_limit():
    """Rows 4 MiB apart (the largest leading dimension the header allows): the kernels' 32-bit
    offsets reach every row of a tile; one element more is refused."""
    import torch
    ld = 1 << 20
    M, N, K = 200, 72, 40
    rng = np.random.default_rng(17)
    A = rng.uniform(-1, 1, (M, K)).astype(np.float32)
    B = rng.uniform(-1, 1, (K, N)).astype(np.float32)
    C = rng.uniform(-1, 1, (M, N)).astype(np.float32)
    dA = torch.zeros((M, ld), dtype=torch.float32, device="cuda")
    dB = torch.zeros((K, ld), dtype=torch.float32, device="cuda")
    dA[:, :K] = torch.from_numpy(A).cuda()
    dB[:, :N] = torch.from_numpy(B).cuda()
    for cfg in (_some_configs()[1], _some_configs()[4], b.make_config(256, 256, 32, 32, 8, 4, 4, 1, 1, 0, 8, 1, 0, 1, 2)):
        dC = torch.from_numpy(C.copy()).cuda()
        b.sgemm_run_config(None, cfg, M, N, K, 1.0, dA, ld, dB, ld, 1.0, dC, N, 0)
        torch.cuda.synchronize()
        gu.check_against_oracle(dC.cpu().numpy(), A, B, C, 1.0, 1.0, 0, what=f"ld 2^20 {cfg}")
        with pytest.raises(b.SgemmError) as e:
            b.sgemm_run_config(None, cfg, M, N, K, 1.0, dA, ld + 1, dB, ld, 1.0, dC, N, 0)
        assert e.value.status == b.E_BADARG
    del dA, dB


def _check_leading_dimensions(cfg, M, N, K, lda, ldb, ldc):
    import torch
    rng = np.random.default_rng(53)
    Abuf = rng.uniform(-1, 1, (M, lda)).astype(np.float32)
    Bbuf = rng.uniform(-1, 1, (K, ldb)).astype(np.float32)
    Cbuf = rng.uniform(-1, 1, (M + 3, ldc)).astype(np.float32)   # 3 guard rows
    dA, dB, dC = (torch.from_numpy(x).cuda() for x in (Abuf, Bbuf, Cbuf.copy()))
    b.sgemm_run_config(None, cfg, M, N, K, 1.25, dA, lda, dB, ldb, 0.5, dC, ldc, 0)
    torch.cuda.synchronize()
    out = dC.cpu().numpy()
    assert np.array_equal(out[:M, N:], Cbuf[:M, N:]) and np.array_equal(out[M:], Cbuf[M:])
    A, B, C = Abuf[:, :K].copy(), Bbuf[:, :N].copy(), Cbuf[:M, :N].copy()
    gu.check_against_oracle(out[:M, :N], A, B, C, 1.25, 0.5)


@pytest.mark.parametrize("layout", [0, 1, 2, 3])
@pytest.mark.parametrize("which", [0, 1, 4, 6, 10])
def test_padded_path_matches_the_oracle_and_leaves_padding_untouched(which, layout):
    """Pre-processing instead of guards: zero-padded copies, the unguarded build, copy back."""
    import torch
    cfg = _some_configs()[which]
    for shape, (alpha, beta) in [((203, 137, 67), (1.0, 0.0)), ((300, 520, 44), (-1.5, 0.25)),
                                 ((256, 256, 64), (1.0, 1.0))]:
        M, N, K = shape
        A, B, C = synth.make_inputs(M, N, K, layout, seed=76 + layout)
        got = gu.run_gpu(cfg, A, B, C, alpha, beta, layout, entry="padded")
        gu.check_against_oracle(got, A, B, C, alpha, beta, layout, what=f"padded {cfg} {shape}")
    # ld > N: what lies outside M x N is not written
    M, N, K, ldc = 97, 83, 45, 89
    A, B, _ = synth.make_inputs(M, N, K, layout, seed=77)
    Cbuf = np.random.default_rng(78).uniform(-1, 1, (M + 2, ldc)).astype(np.float32)
    dA, dB, dC = (torch.from_numpy(x).cuda() for x in (A, B, Cbuf.copy()))
    b.sgemm_run_config_padded(None, cfg, M, N, K, 1.0, dA, A.shape[1], dB, B.shape[1], 0.5, dC, ldc, layout)
    torch.cuda.synchronize()
    out = dC.cpu().numpy()
    assert np.array_equal(out[:M, N:], Cbuf[:M, N:]) and np.array_equal(out[M:], Cbuf[M:])
    gu.check_against_oracle(out[:M, :N], A, B, Cbuf[:M, :N].copy(), 1.0, 0.5, layout)


def test_dispatch_pads_a_large_problem_with_odd_rows_and_stays_within_the_bound():
    """4091^3 through sgemm_tuned_on(): the committed 4096^3 winner serves it, its guarded build
    would load single floats, so dispatch goes through zero-padded copies; sampled rows, columns
    and scattered elements against the oracle, and the whole result against the reference kernel."""
    import torch
    _restore_cache()
    M = N = K = 4091
    cfg = b.sgemm_config_select(M, N, K, 0)
    assert b.sgemm_config_prefers_padding(cfg, M, N, K, K, N, N, 0, 0.0) == 1
    A, B, C = synth.make_inputs(M, N, K, 0, seed=91, dist="normal")
    dA, dB, dC = (torch.from_numpy(x).cuda() for x in (A, B, C))
    dR = dC.clone()
    b.sgemm_tuned_on(None, M, N, K, 1.0, dA, K, dB, N, 0.0, dC, N, 0)
    b.sgemm_reference(None, M, N, K, 1.0, dA, K, dB, N, 0.0, dR, N, 0)
    torch.cuda.synchronize()
    r, c = synth.sample_positions(M, N, 91, rows=2, cols=2, scattered=512)
    ref = orc.sgemm_sample(1.0, A, B, 0.0, C, r, c, 0)
    tol = orc.tolerance(K, np.abs(A).max(), np.abs(B).max(), ref)
    got = dC.cpu().numpy()
    assert np.all(np.abs(got[r, c] - ref) <= tol)
    bound = 1e-5 * K * float(dA.abs().max()) * float(dB.abs().max()) + 1e-6 * dR.abs()
    assert bool(((dC - dR).abs() <= 2 * bound).all())


@pytest.mark.parametrize("which", WHICH)
def test_even_sizes_that_are_not_multiples_of_four_keep_two_float_loads(which):
    """Row lengths 138 and 66 (202 when A is stored transposed): 4-float loads are narrowed to 2."""
    cfg = _some_configs()[which]
    for layout in (0, 3):
        A, B, C = synth.make_inputs(*NARROW_SHAPE, layout, seed=95 + layout)
        got = gu.run_gpu(cfg, A, B, C, 1.25, -0.5, layout)
        gu.check_against_oracle(got, A, B, C, 1.25, -0.5, layout, what=f"{cfg} {NARROW_SHAPE} layout {layout}")


def test_degenerate_sizes():
    import torch
    cfg = _some_configs()[1]
    dA = torch.zeros(16, device="cuda"); dB = torch.zeros(16, device="cuda")
    dC = torch.full((4, 4), 7.0, device="cuda")
    # M == 0 or N == 0: no-op; K == 0: C = beta*C
    b.sgemm_run_config(None, cfg, 0, 4, 4, 1.0, dA, 4, dB, 4, 0.0, dC, 4, 0)
    b.sgemm_run_config(None, cfg, 4, 0, 4, 1.0, dA, 4, dB, 4, 0.0, dC, 4, 0)
    torch.cuda.synchronize()
    assert torch.all(dC == 7.0)
    b.sgemm_run_config(None, cfg, 4, 4, 0, 1.0, dA, 4, dB, 4, 0.5, dC, 4, 0)
    torch.cuda.synchronize()
    assert torch.all(dC == 3.5)
    # bad arguments are errors, not launches
    for args in [(-1, 4, 4, 4, 4, 4), (4, 4, 4, 3, 4, 4), (4, 4, 4, 4, 3, 4), (4, 4, 4, 4, 4, 3)]:
        M, N, K, lda, ldb, ldc = args
        with pytest.raises(b.SgemmError) as e:
            b.sgemm_run_config(None, cfg, M, N, K, 1.0, dA, lda, dB, ldb, 0.0, dC, ldc, 0)
        assert e.value.status == b.E_BADARG
    with pytest.raises(b.SgemmError):
        b.sgemm_run_config(None, cfg, 4, 4, 4, 1.0, dA, 4, dB, 4, 0.0, dC, 4, 7)
    bad = b.make_config(100, 64, 16, 8, 8, 1, 1, 1, 1, 0, 2, 0, 0)
    with pytest.raises(b.SgemmError) as e:
        b.sgemm_run_config(None, bad, 4, 4, 4, 1.0, dA, 4, dB, 4, 0.0, dC, 4, 0)
    assert e.value.status == b.E_INVALID


def test_more_rows_than_one_grid_dimension_holds():
    """300 000 rows: the reference kernel and the scaling kernel put rows into the grid's second
    dimension (at most 65 535 workgroups there) and stride over what does not fit; the tuned
    variants number their tiles along the first."""
    import torch
    M, N, K = 300000, 24, 40
    A, B, C = synth.make_inputs(M, N, K, 0, seed=64)
    ref = orc.sgemm(1.5, A, B, 0.5, C, 0)
    for entry in ("reference", "tuned"):
        got = gu.run_gpu(None, A, B, C, 1.5, 0.5, 0, entry=entry)
        gu.check_against_oracle(got, A, B, C, 1.5, 0.5, 0, ref, what=f"{entry} {M}x{N}x{K}")
    # alpha = 0: C = beta * C, every row of it
    dC = torch.from_numpy(C.copy()).cuda()
    b.sgemm_tuned_on(None, M, N, K, 0.0, None, K, None, N, 0.5, dC, N, 0)
    torch.cuda.synchronize()
    assert np.array_equal(dC.cpu().numpy(), np.float32(0.5) * C)


def test_reference_kernel_against_oracle():
    """The device reference kernel that tune() verifies against is itself held to the oracle."""
    for layout in range(4):
        A, B, C = synth.make_inputs(77, 131, 200, layout, seed=60 + layout)
        got = gu.run_gpu(None, A, B, C, 1.5, -0.5, layout, entry="reference")
        ref = orc.sgemm(1.5, A, B, -0.5, C, layout)
        assert np.max(np.abs(got - ref)) <= 2.0 ** -23 * np.max(np.abs(ref))


@pytest.mark.parametrize("which", [1, 4, 5, 7, 9, 10])
def test_run_to_run_determinism(which):
    """No atomics anywhere: split-K planes are added in index order by the reduction kernel."""
    cfg = _some_configs()[which]
    A, B, C = synth.make_inputs(384, 256, 512, 0, seed=61)
    first = gu.run_gpu(cfg, A, B, C, 1.0, 0.0)
    for _ in range(3):
        assert np.array_equal(gu.run_gpu(cfg, A, B, C, 1.0, 0.0), first)


# ---- full benchmark sizes: sampled outputs ------------------------------------------------
# At 4096^3 the oracle cannot produce the whole matrix in test time, but every element is an
# independent dot product: whole rows, whole columns, edge tiles and scattered elements are
# computed one by one and compared under the same bound.

_SAMPLED_REFERENCE = {}


def _sampled_check(workload, cfg, entry="config", rows=64, cols=64, scattered=4096):
    import torch
    w = synth.WORKLOADS[workload]
    A, B, C = synth.make_workload(w)
    dA, dB, dC = (torch.from_numpy(x).cuda() for x in (A, B, C))
    lda, ldb, ldc = A.shape[1], B.shape[1], w.N
    if entry == "config":
        b.sgemm_run_config(None, cfg, w.M, w.N, w.K, w.alpha, dA, lda, dB, ldb, w.beta, dC, ldc, w.layout)
    else:
        b.sgemm_tuned_on(None, w.M, w.N, w.K, w.alpha, dA, lda, dB, ldb, w.beta, dC, ldc, w.layout)
    torch.cuda.synchronize()
    got = dC.cpu().numpy()
    key = (workload, rows, cols, scattered)
    if key not in _SAMPLED_REFERENCE:   # the oracle's values depend on the workload only
        r, c = synth.sample_positions(w.M, w.N, w.seed, rows=rows, cols=cols, scattered=scattered)
        _SAMPLED_REFERENCE.clear()      # one workload's sample at a time is kept
        _SAMPLED_REFERENCE[key] = (r, c, orc.sgemm_sample(w.alpha, A, B, w.beta, C, r, c, w.layout))
    r, c, ref = _SAMPLED_REFERENCE[key]
    tol = orc.tolerance(w.K, np.max(np.abs(A)), np.max(np.abs(B)), ref)
    err = np.abs(got[r, c].astype(np.float64) - ref)
    assert np.all(err <= tol), (workload, cfg, float(np.max(err / tol)))
    # property that holds at any size: nothing non-finite, nothing left unwritten
    assert np.all(np.isfinite(got))
    return float(np.max(err / tol))


@pytest.mark.parametrize("which", range(len(BENCH_CONFIGS)))
def test_headline_size_4096_sampled(which):
    _sampled_check("cfg4_4096", BENCH_CONFIGS[which])


def test_dispatch_entry_point_at_headline_size():
    _sampled_check("cfg4_4096", None, entry="tuned")


@pytest.mark.parametrize("workload", ["cfg5_128x4096x4096", "cfg5_4096x64x9216"])
def test_deep_learning_shapes_a_transposed(workload):
    for cfg in SKINNY_CONFIGS:
        _sampled_check(workload, cfg, rows=16, cols=16)
    _sampled_check(workload, None, entry="tuned", rows=16, cols=16)


@pytest.mark.parametrize("workload", ["cfg3_1000", "cfg3_1536"])
def test_non_tile_multiple_sizes_full_compare(workload):
    w = synth.WORKLOADS[workload]
    A, B, C = synth.make_workload(w)
    ref = orc.sgemm(w.alpha, A, B, w.beta, C, w.layout)
    for cfg in BENCH_CONFIGS:
        got = gu.run_gpu(cfg, A, B, C, w.alpha, w.beta, w.layout)
        gu.check_against_oracle(got, A, B, C, w.alpha, w.beta, w.layout, ref, what=f"{workload} {cfg}")
    got = gu.run_gpu(None, A, B, C, w.alpha, w.beta, w.layout, entry="tuned")
    gu.check_against_oracle(got, A, B, C, w.alpha, w.beta, w.layout, ref, what=f"{workload} tuned")


def test_paper_workload_2048_cubed_full_compare():
    """Benchmark configuration 2, the paper's own search-strategy workload (2048^3, alpha = 2,
    beta = 0.5; first equation of the matrix-multiplication case study): every element of C
    against the oracle, for the committed winner run explicitly and through the dispatch."""
    w = synth.WORKLOADS["cfg2_2048"]
    A, B, C = synth.make_workload(w)
    ref = orc.sgemm(w.alpha, A, B, w.beta, C, w.layout)
    _restore_cache()
    winner = b.sgemm_config_get(w.M, w.N, w.K, w.layout)
    assert winner is not None
    for cfg, entry in [(winner, "config"), (None, "tuned"), (BENCH_CONFIGS[0], "config")]:
        got = gu.run_gpu(cfg, A, B, C, w.alpha, w.beta, w.layout, entry=entry)
        gu.check_against_oracle(got, A, B, C, w.alpha, w.beta, w.layout, ref, what=f"cfg2_2048 {entry} {cfg}")


@pytest.mark.parametrize("workload,rows,cols", [("cfg3_3000", 64, 64), ("cfg4_8192", 64, 64)])
def test_largest_benchmark_sizes_sampled(workload, rows, cols):
    """3000^3 (192 x 192 tiles with a ragged edge on every side, alpha = beta = 1) and 8192^3:
    whole rows, whole columns, the edge tiles and scattered elements against the oracle, for the
    committed winner run explicitly and through the dispatch."""
    w = synth.WORKLOADS[workload]
    _restore_cache()
    winner = b.sgemm_config_get(w.M, w.N, w.K, w.layout)
    assert winner is not None
    _sampled_check(workload, winner, rows=rows, cols=cols)
    _sampled_check(workload, None, entry="tuned", rows=rows, cols=cols)


@pytest.mark.parametrize("size", [512, 1024])
def test_power_of_two_sizes_of_the_committed_table(size):
    """512^3 and 1024^3 have entries of their own (winners of focused full searches): the
    dispatch takes them, and the result holds against the oracle with and without the old C."""
    tuned = b.sgemm_config_get(size, size, size, 0)
    assert tuned is not None and b.sgemm_config_select(size, size, size, 0).as_tuple() == tuned.as_tuple()
    A, B, C = synth.make_inputs(size, size, size, 0, seed=63)
    for alpha, beta in [(1.0, 0.0), (-1.5, 0.75)]:
        got = gu.run_gpu(None, A, B, C, alpha, beta, 0, entry="tuned")
        gu.check_against_oracle(got, A, B, C, alpha, beta, 0, what=f"{size}^3 {tuned} beta {beta}")


# ---- the tuner and the dispatch entry points on the device ---------------------------------

def _restore_cache():
    """Back to what a fresh process starts with: the committed table of tuned configurations."""
    import os
    b.sgemm_cache_clear()
    table = os.path.join(os.path.dirname(b.LIB_PATH), "..", "tuned_configs.txt")
    if os.path.exists(table):
        b.sgemm_cache_load(table)


def _device_operands(workload):
    import torch
    w = synth.WORKLOADS[workload]
    A, B, C = synth.make_workload(w)
    dA, dB, dC0 = (torch.from_numpy(x).cuda() for x in (A, B, C))
    return w, (A, B, C), dA, dB, dC0.clone(), dC0


def test_tune_ex_full_search_of_the_small_space(tmp_path):
    """Benchmark configuration 1 end to end: 16 variants compiled, verified against the device
    reference kernel, timed; the winner lands in the per-shape cache and sgemm_tuned() then
    agrees with the oracle."""
    import json
    import torch
    w, (A, B, C), dA, dB, dC, dC0 = _device_operands("cfg1_256")
    log = tmp_path / "evals.jsonl"
    opts = b.tune_opts()
    opts.space = b.SPACE_SMALL
    opts.A, opts.B, opts.C, opts.C0 = dA.data_ptr(), dB.data_ptr(), dC.data_ptr(), dC0.data_ptr()
    opts.lda, opts.ldb, opts.ldc = w.K, w.N, w.N
    opts.log_path = str(log).encode()
    b.sgemm_cache_clear()
    try:
        evals, res = b.tune_ex(w.M, w.N, w.K, w.layout, w.alpha, w.beta, b.STRATEGY_FULL, 0, 0, opts)
        assert evals == 16 and res.space_size == 16 and res.failed == 0
        assert 0 <= res.best_index < 16 and res.best_ms > 0 and res.best_gflops > 0
        assert res.best.as_tuple() == b.sgemm_space_get(b.SPACE_SMALL, res.best_index).as_tuple()
        rows = [json.loads(line) for line in log.read_text().splitlines()]
        assert [r["index"] for r in rows] == list(range(16))
        assert all(r["status"].startswith("ok") and r["scratch"] == 0 for r in rows)
        assert min(r["ms"] for r in rows) == pytest.approx(res.best_ms, rel=1e-4)   # log prints 6 digits
        assert b.sgemm_config_get(w.M, w.N, w.K, w.layout).as_tuple() == res.best.as_tuple()
        dC.copy_(dC0)
        b.sgemm_tuned_on(None, w.M, w.N, w.K, w.alpha, dA, w.K, dB, w.N, w.beta, dC, w.N, w.layout)
        torch.cuda.synchronize()
        gu.check_against_oracle(dC.cpu().numpy(), A, B, C, w.alpha, w.beta, w.layout)
    finally:
        _restore_cache()


def test_verification_catches_a_variant_that_leaves_a_tile_unwritten(tmp_path, monkeypatch):
    """The paper's verification of every tested configuration ("Advanced usage") must not be
    fooled by stale output: with beta = 0, C still holds the previous candidate's correct result
    when the next candidate runs.  Variants built with a planted bug (one workgroup returns
    without writing its tile) are all rejected, in a search that follows an honest one on the
    same C."""
    import json
    w, (A, B, C), dA, dB, dC, dC0 = _device_operands("cfg1_256")
    assert w.beta == 0.0
    log = tmp_path / "evals.jsonl"
    opts = b.tune_opts()
    opts.space = b.SPACE_SMALL
    opts.A, opts.B, opts.C, opts.C0 = dA.data_ptr(), dB.data_ptr(), dC.data_ptr(), dC0.data_ptr()
    opts.lda, opts.ldb, opts.ldc = w.K, w.N, w.N
    opts.reps, opts.warmup_ms = 3, -1.0
    opts.log_path = str(log).encode()
    b.sgemm_cache_clear()
    try:
        evals, res = b.tune_ex(w.M, w.N, w.K, w.layout, w.alpha, w.beta, b.STRATEGY_FULL, 0, 0, opts)
        assert evals == 16 and res.failed == 0          # C now holds a correct result
        gu.check_against_oracle(dC.cpu().numpy(), A, B, C, w.alpha, w.beta, w.layout)
        log.write_text("")
        monkeypatch.setenv("SGEMM_TUNED_EXTRA_DEFINES", "-DPLANT_SKIP_TILE=1")
        with pytest.raises(b.SgemmError) as e:
            b.tune_ex(w.M, w.N, w.K, w.layout, w.alpha, w.beta, b.STRATEGY_FULL, 0, 0, opts)
        assert e.value.status == b.E_NOCONFIG
        rows = [json.loads(line) for line in log.read_text().splitlines()]
        assert len(rows) == 16 and all(r["status"] == "verify" for r in rows), [r["status"] for r in rows]
    finally:
        monkeypatch.delenv("SGEMM_TUNED_EXTRA_DEFINES", raising=False)
        _restore_cache()


@pytest.mark.parametrize("strategy", [b.STRATEGY_RANDOM, b.STRATEGY_ANNEALING, b.STRATEGY_PSO])
def test_tune_ex_budgeted_strategies(strategy):
    """A budget counts distinct configurations; every one of them is verified on a C restored
    from C0 (with beta != 0 the timed repetitions then keep updating C); the caller's C0 is
    never touched."""
    import torch
    M, N, K = 192, 160, 96
    A, B, C = synth.make_inputs(M, N, K, 0, seed=71)
    dA, dB, dC0 = (torch.from_numpy(x).cuda() for x in (A, B, C))
    dC = dC0.clone()
    opts = b.tune_opts()
    opts.space = b.SPACE_SMALL
    opts.A, opts.B, opts.C, opts.C0 = dA.data_ptr(), dB.data_ptr(), dC.data_ptr(), dC0.data_ptr()
    opts.lda, opts.ldb, opts.ldc = K, N, N
    opts.reps, opts.warmup_ms = 3, -1.0
    b.sgemm_cache_clear()
    try:
        evals, res = b.tune_ex(M, N, K, 0, 1.5, 0.5, strategy, 6, 3, opts)
        assert 1 <= evals <= 6 and res.failed == 0 and res.best_index >= 0
        assert torch.equal(dC0.cpu(), torch.from_numpy(C))
    finally:
        _restore_cache()


def test_tune_simple_entry_point_and_dispatch_fallback():
    """tune(M,N,K,strategy,budget) on library-owned synthetic operands; afterwards a nearby
    untuned shape is served by the tuned shape's configuration."""
    import torch
    b.sgemm_cache_clear()
    try:
        evals = b.tune(256, 256, 128, b.STRATEGY_RANDOM, 3)
        assert 1 <= evals <= 3
        tuned = b.sgemm_config_get(256, 256, 128, 0)
        assert tuned is not None and b.sgemm_config_check(tuned) == 0
        assert b.sgemm_config_select(250, 250, 128, 0).as_tuple() == tuned.as_tuple()    # the same grid of tiles
        A, B, C = synth.make_inputs(250, 250, 128, 0, seed=72)
        got = gu.run_gpu(None, A, B, C, 1.0, 0.0, 0, entry="tuned")
        gu.check_against_oracle(got, A, B, C, 1.0, 0.0, 0)
    finally:
        _restore_cache()


@pytest.mark.parametrize("layout", [2, 3])
def test_dispatch_without_a_tuned_shape_uses_the_built_in_default(layout):
    """No shape is tuned for these storage layouts, so sgemm_tuned() runs the built-in default
    configuration (with split K on the long-K shape)."""
    for shape in [(300, 200, 150), (96, 1000, 4100), (1536, 1536, 64)]:
        M, N, K = shape
        A, B, C = synth.make_inputs(M, N, K, layout, seed=74 + layout)
        assert b.sgemm_config_get(M, N, K, layout) is None
        cfg = b.sgemm_config_select(M, N, K, layout)
        assert cfg.as_tuple() == b.sgemm_config_default(M, N, K, layout).as_tuple()
        got = gu.run_gpu(None, A, B, C, 1.0, 0.5, layout, entry="tuned")
        gu.check_against_oracle(got, A, B, C, 1.0, 0.5, layout, what=f"{shape} layout {layout} {cfg}")


@pytest.mark.parametrize("strategy", [b.STRATEGY_ANNEALING, b.STRATEGY_PSO, b.STRATEGY_FULL])
def test_online_tuning_settles_on_a_configuration_and_every_call_is_correct(strategy):
    """Tuning in the first calls: each call computes its GEMM with the configuration the search
    wants timed next; after the budget the winner is in the per-shape cache."""
    import torch
    M, N, K = 320, 256, 192
    A, B, C = synth.make_inputs(M, N, K, 0, seed=75)
    dA, dB, dC0 = (torch.from_numpy(x).cuda() for x in (A, B, C))
    dC = dC0.clone()
    ref = orc.sgemm(1.25, A, B, 0.5, C, 0)
    budget = 6 if strategy != b.STRATEGY_FULL else 0      # full search ignores the budget
    b.sgemm_cache_clear()
    try:
        settled_after = None
        for call in range(24):
            dC.copy_(dC0)
            b.sgemm_tuned_online(None, M, N, K, 1.25, dA, K, dB, N, 0.5, dC, N, 0,
                                 space=b.SPACE_SMALL, strategy=strategy, budget=max(budget, 1))
            torch.cuda.synchronize()
            gu.check_against_oracle(dC.cpu().numpy(), A, B, C, 1.25, 0.5, 0, ref, what=f"call {call}")
            if settled_after is None and b.sgemm_config_get(M, N, K, 0) is not None:
                settled_after = call
        assert settled_after is not None
        # the search times one configuration per call; the call after the last one settles
        assert settled_after <= (16 if strategy == b.STRATEGY_FULL else budget)
        winner = b.sgemm_config_get(M, N, K, 0)
        assert b.sgemm_space_find(b.SPACE_SMALL, winner) >= 0
    finally:
        _restore_cache()


def test_online_tuning_with_concurrent_callers_of_one_shape():
    """Several host threads make their first calls of the same shape at once: each candidate of
    the search is handed to exactly one of them, every call still computes its own GEMM, and the
    threads that are still waiting when the search ends are served by the winner."""
    import threading
    import torch
    M, N, K = 320, 256, 192
    A, B, C = synth.make_inputs(M, N, K, 0, seed=75)
    dA, dB, dC0 = (torch.from_numpy(x).cuda() for x in (A, B, C))
    ref = orc.sgemm(1.25, A, B, 0.5, C, 0)
    torch.cuda.synchronize()
    b.sgemm_cache_clear()
    failures = []

    def caller(who):
        try:
            torch.cuda.set_device(0)
            dC = dC0.clone()
            for call in range(10):
                dC.copy_(dC0)
                torch.cuda.synchronize()
                b.sgemm_tuned_online(None, M, N, K, 1.25, dA, K, dB, N, 0.5, dC, N, 0,
                                     space=b.SPACE_SMALL, strategy=b.STRATEGY_FULL, budget=1)
                torch.cuda.synchronize()
                gu.check_against_oracle(dC.cpu().numpy(), A, B, C, 1.25, 0.5, 0, ref,
                                        what=f"thread {who} call {call}")
        except BaseException as e:  # noqa: BLE001 - reported by the test's own thread below
            failures.append((who, repr(e)))

    try:
        threads = [threading.Thread(target=caller, args=(i,)) for i in range(3)]
        for t in threads:
            t.start()
        for t in threads:
            t.join(120)
        assert not any(t.is_alive() for t in threads), "a caller never returned"
        assert not failures, failures
        # 30 calls for 16 candidates: the search has ended and its winner is in the table
        winner = b.sgemm_config_get(M, N, K, 0)
        assert winner is not None and b.sgemm_space_find(b.SPACE_SMALL, winner) >= 0
    finally:
        _restore_cache()


def test_prepared_call_repeats_the_ordinary_one():
    """The binding's prepared call (arguments marshalled once) launches what sgemm_tuned_on()
    launches: same bits, call after call, also after the output was overwritten in between."""
    import torch
    M, N, K = 300, 200, 150
    A, B, C = synth.make_inputs(M, N, K, 0, seed=76)
    dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
    want = gu.run_gpu(None, A, B, C, 1.25, 0.0, 0, entry="tuned")
    gu.check_against_oracle(want, A, B, C, 1.25, 0.0, 0)
    dC = torch.empty((M, N), dtype=torch.float32, device="cuda")
    call = b.sgemm_tuned_prepare(None, M, N, K, 1.25, dA, K, dB, N, 0.0, dC, N, 0)
    for _ in range(3):
        dC.fill_(float("nan"))
        assert call() == 0
        torch.cuda.synchronize()
        assert np.array_equal(dC.cpu().numpy(), want)


def test_launch_on_a_side_stream_and_on_the_set_stream():
    import torch
    cfg = _some_configs()[1]
    A, B, C = synth.make_inputs(300, 200, 150, 0, seed=73)
    dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    dC = torch.from_numpy(C).cuda()
    torch.cuda.synchronize()
    b.sgemm_run_config(side, cfg, 300, 200, 150, 1.0, dA, 150, dB, 200, 1.0, dC, 200, 0)
    side.synchronize()
    gu.check_against_oracle(dC.cpu().numpy(), A, B, C, 1.0, 1.0, 0)
    # sgemm_tuned() launches on the stream given to sgemm_set_stream()
    dC2 = torch.from_numpy(C).cuda()
    torch.cuda.synchronize()
    b.sgemm_set_stream(side)
    try:
        b.sgemm_tuned(300, 200, 150, 2.0, dA, 150, dB, 200, 0.0, dC2, 200, 0)
        side.synchronize()
    finally:
        b.sgemm_set_stream(0)
    gu.check_against_oracle(dC2.cpu().numpy(), A, B, C, 2.0, 0.0, 0)
