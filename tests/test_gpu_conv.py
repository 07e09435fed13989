"""GPU parity of the tunable 2D convolution (second kernel family) against the CPU oracle,
through the C ABI.  Bound per element:
    |B_gpu - B_ref| <= 1e-5 * Xf * Yf * |w| * max|F| * max|A| + 1e-6 * |B_ref|."""
import numpy as np
import pytest

from oracle import conv_oracle as co
from paper_1703_06503_amd import binding as b
from paper_1703_06503_amd import synth

pytestmark = pytest.mark.gpu

from tests.variants import CONV_SAMPLES as SAMPLES, CONV_CONFIGS as CONFIGS, conv_sample as sample  # noqa: E402


def run(cfg, A, F, w, X, Y, entry="config", ldb=None, a_offset=0):
    """One call through the C ABI; returns B (Y x ldb, float32).  a_offset shifts the image by
    that many floats inside its buffer (a misaligned pointer)."""
    import torch
    Yf, Xf = F.shape
    ldb = ldb or max(X, 1)
    buf = torch.zeros(A.size + a_offset, dtype=torch.float32, device="cuda")
    buf[a_offset:] = torch.from_numpy(A).cuda().reshape(-1)
    dA = buf[a_offset:]
    dF = torch.from_numpy(np.ascontiguousarray(F)).cuda()
    dB = torch.full((max(Y, 1), ldb), -777.0, dtype=torch.float32, device="cuda")
    lda = A.shape[1]
    if entry == "config":
        b.conv2d_run_config(None, cfg, X, Y, Xf, Yf, w, dF, dA, lda, dB, ldb)
    elif entry == "tuned":
        b.conv2d_tuned(X, Y, Xf, Yf, w, dF, dA, lda, dB, ldb)
    else:
        b.conv2d_reference(None, X, Y, Xf, Yf, w, dF, dA, lda, dB, ldb)
    torch.cuda.synchronize()
    return dB.cpu().numpy()


def check(got, A, F, w, X, Y, what=""):
    Yf, Xf = F.shape
    ref = co.conv2d(A, F, w, X, Y)
    tol = co.tolerance(ref, F, A[:Y + Yf - 1, :X + Xf - 1], w)
    err = np.abs(got[:Y, :X].astype(np.float64) - ref)
    bad = ~(err <= tol)
    if bad.any():
        y, x = np.unravel_index(np.argmax(np.where(bad, err, 0)), err.shape)
        raise AssertionError(f"{what}: {int(bad.sum())} outputs outside the bound; worst at (y={y}, x={x}): "
                             f"got {got[y, x]!r}, oracle {ref[y, x]!r}, bound {tol[y, x]:.3e}")


@pytest.mark.parametrize("Xf,Yf", list(SAMPLES))
def test_sampled_configurations_match_the_oracle(Xf, Yf):
    """A sample of the space on an image that is a multiple of every tile (unguarded builds,
    several workgroups) and on a ragged one (guarded builds, a partial tile on both edges)."""
    for (X, Y), seed in [((1024, 512), 20), ((300, 201), 21)]:
        A, F = synth.make_conv_inputs(X, Y, Xf, Yf, seed=seed + Xf)
        for i in sample(Xf, Yf):
            cfg = b.conv2d_space_get(Xf, Yf, i)
            got = run(cfg, A, F, 0.37, X, Y)
            check(got, A, F, 0.37, X, Y, what=f"{cfg} {Xf}x{Yf} on {X}x{Y}")


@pytest.mark.parametrize("which", range(len(CONFIGS)))
def test_integer_inputs_are_bit_exact_and_all_variants_agree_bit_for_bit(which):
    """Small integers: every order of summation is exact, so the result equals the oracle's
    exactly; and on ordinary inputs every variant adds its taps in the same order as the
    reference kernel, so all of them give the same bits."""
    import torch
    cfg = b.make_conv_config(*CONFIGS[which])
    X, Y, Xf, Yf = 520, 130, 7, 5
    A, F = synth.make_conv_inputs(X, Y, Xf, Yf, seed=30, dist="smallint")
    got = run(cfg, A, F, 2.0, X, Y)
    assert np.array_equal(got.astype(np.float64), co.conv2d(A, F, 2.0, X, Y))
    A, F = synth.make_conv_inputs(X, Y, Xf, Yf, seed=31)
    assert np.array_equal(run(cfg, A, F, 0.1, X, Y), run(None, A, F, 0.1, X, Y, entry="reference"))


@pytest.mark.parametrize("which", range(len(CONFIGS)))
def test_leading_dimensions_misaligned_pointers_and_untouched_padding(which):
    cfg = b.make_conv_config(*CONFIGS[which])
    X, Y, Xf, Yf = 256, 64, 3, 3
    for lda, ldb, off in [(X + Xf - 1 + 6, X + 8, 0), (X + Xf - 1 + 3, X + 5, 0), (X + Xf - 1 + 2, X, 1)]:
        A, F = synth.make_conv_inputs(X, Y, Xf, Yf, seed=40, lda=lda)
        got = run(cfg, A, F, 1.0, X, Y, ldb=ldb, a_offset=off)
        check(got, A, F, 1.0, X, Y, what=f"{cfg} lda={lda} ldb={ldb} offset={off}")
        assert np.all(got[:, X:] == -777.0)


def test_reference_kernel_matches_the_oracle():
    for (X, Y, Xf, Yf) in [(300, 201, 7, 7), (65, 5, 3, 11), (1, 1, 1, 1)]:
        A, F = synth.make_conv_inputs(X, Y, Xf, Yf, seed=50)
        check(run(None, A, F, -0.5, X, Y, entry="reference"), A, F, -0.5, X, Y, what="reference")


def test_more_image_rows_than_one_grid_dimension_holds():
    """270 000 image rows: the reference kernel strides over the rows that its grid's second
    dimension (at most 65 535 workgroups) does not hold; the tuned variant's tile rows fit."""
    X, Y, Xf, Yf = 16, 270000, 3, 3
    A, F = synth.make_conv_inputs(X, Y, Xf, Yf, seed=51)
    for entry in ("reference", "tuned"):
        check(run(None, A, F, 0.25, X, Y, entry=entry), A, F, 0.25, X, Y, what=f"{entry}, {Y} rows")


def test_default_dispatch_for_filter_sizes_that_were_never_tuned():
    """conv2d_tuned with nothing in its table: the built-in defaults for small, medium, large and
    very large filters, square and not, on a ragged image."""
    b.conv2d_cache_clear()
    for Xf, Yf in [(1, 1), (2, 5), (9, 9), (11, 3), (13, 13), (31, 5), (17, 17)]:
        X, Y = 333, 77
        A, F = synth.make_conv_inputs(X, Y, Xf, Yf, seed=90 + Xf)
        check(run(None, A, F, 0.5, X, Y, entry="tuned"), A, F, 0.5, X, Y, what=f"default for {Xf}x{Yf}")


def test_degenerate_sizes_and_error_returns():
    import torch
    cfg = b.make_conv_config(32, 8, 2, 4, 1, 2, 0, 1)
    A, F = synth.make_conv_inputs(8, 8, 3, 3, seed=60)
    dA, dF = torch.from_numpy(A).cuda(), torch.from_numpy(F).cuda()
    dB = torch.full((8, 8), 5.0, device="cuda")
    assert b.conv2d_run_config(None, cfg, 0, 8, 3, 3, 1.0, dF, dA, 10, dB, 8) == b.OK
    assert b.conv2d_run_config(None, cfg, 8, 0, 3, 3, 1.0, dF, dA, 10, dB, 8) == b.OK
    torch.cuda.synchronize()
    assert bool((dB == 5.0).all())
    for args in [(8, 8, 3, 3, 1.0, dF, dA, 9, dB, 8),      # lda < X + Xf - 1
                 (8, 8, 3, 3, 1.0, dF, dA, 10, dB, 7),     # ldb < X
                 (8, 8, 0, 3, 1.0, dF, dA, 10, dB, 8),     # filter size
                 (-1, 8, 3, 3, 1.0, dF, dA, 10, dB, 8),
                 (8, 8, 3, 3, 1.0, None, dA, 10, dB, 8)]:
        with pytest.raises(b.SgemmError) as e:
            b.conv2d_run_config(None, cfg, *args)
        assert e.value.status == b.E_BADARG
    with pytest.raises(b.SgemmError) as e:
        b.conv2d_run_config(None, b.make_conv_config(64, 64, 1, 1, 0, 1, 0, 1), 8, 8, 3, 3, 1.0, dF, dA, 10, dB, 8)
    assert e.value.status == b.E_INVALID
    # a tiny image with a tile much larger than it
    got = run(b.make_conv_config(32, 16, 8, 8, 2, 8, 0, 1), A, F, 1.0, 8, 8)
    check(got, A, F, 1.0, 8, 8, what="tile larger than the image")


def test_tuner_on_the_device_and_tuned_dispatch(tmp_path):
    """A budgeted search of each strategy on a small image: every evaluated configuration is
    verified by the library against its reference kernel; the winner then serves conv2d_tuned,
    whose output is held to the oracle."""
    import json
    X, Y, Xf, Yf, w = 1024, 512, 7, 7, 1.0 / 49
    log = tmp_path / "conv.jsonl"
    o = b.tune_opts()
    o.reps, o.warmup_ms, o.log_path = 3, 1.0, str(log).encode()
    total = 0
    for strategy in (b.STRATEGY_RANDOM, b.STRATEGY_ANNEALING, b.STRATEGY_PSO):
        n, res = b.conv2d_tune(X, Y, Xf, Yf, w, strategy, 12, seed=3, opts=o)
        total += n
        assert 1 <= n <= 12 and res.best_ms > 0 and res.space_size == b.conv2d_space_size(Xf, Yf)
        assert b.conv2d_config_check(res.best, Xf, Yf) == b.OK
    lines = [json.loads(l) for l in log.read_text().splitlines()]
    assert len(lines) == total and all(l["status"] in ("ok", "ok-cut") for l in lines)
    exact, cfg = b.conv2d_config_select(X, Y, Xf, Yf)
    best = min(l["ms"] for l in lines if l["status"] == "ok")
    assert exact == 1 and list(cfg.as_tuple()) == next(l["config"] for l in lines if l["ms"] == best)
    A, F = synth.make_conv_inputs(X, Y, Xf, Yf, seed=70)
    check(run(None, A, F, w, X, Y, entry="tuned"), A, F, w, X, Y, what="conv2d_tuned after tuning")
    # another image size with the same filter takes the nearest entry; an unseen filter the default
    exact, near = b.conv2d_config_select(999, 333, Xf, Yf)
    assert exact == 0 and near.as_tuple() == cfg.as_tuple()
    A, F = synth.make_conv_inputs(333, 99, 5, 5, seed=71)
    check(run(None, A, F, 1.0, 333, 99, entry="tuned"), A, F, 1.0, 333, 99, what="conv2d_tuned default")


@pytest.mark.parametrize("name", ["conv_3x3", "conv_7x7", "conv_11x11", "conv_7x7_ragged"])
def test_full_size_image_on_sampled_outputs(name):
    """The paper's 8192 x 4096 image (and one just short of it, so that interior workgroups take
    the plain path and border workgroups the guarded one): outputs sampled over the whole image
    (corners, tile seams and random points) against the oracle, and the whole result against
    the reference kernel."""
    b.conv2d_cache_clear()
    import torch
    wl = synth.CONV_WORKLOADS[name]
    A, F = synth.make_conv_workload(wl)
    dA, dF = torch.from_numpy(A).cuda(), torch.from_numpy(F).cuda()
    dB = torch.empty((wl.Y, wl.X), dtype=torch.float32, device="cuda")
    dR = torch.empty_like(dB)
    b.conv2d_tuned(wl.X, wl.Y, wl.Xf, wl.Yf, wl.w, dF, dA, A.shape[1], dB, wl.X)
    b.conv2d_reference(None, wl.X, wl.Y, wl.Xf, wl.Yf, wl.w, dF, dA, A.shape[1], dR, wl.X)
    torch.cuda.synchronize()
    assert bool((dB == dR).all())                      # same order of summation: same bits
    rng = np.random.default_rng(80)
    ys = np.concatenate([[0, 0, wl.Y - 1, wl.Y - 1, 31, 32, 255, 256], rng.integers(0, wl.Y, 2000)])
    xs = np.concatenate([[0, wl.X - 1, 0, wl.X - 1, 63, 64, 511, 512], rng.integers(0, wl.X, 2000)])
    ref = co.conv2d_sample(A, F, wl.w, ys, xs)
    got = dB.cpu().numpy()[ys, xs].astype(np.float64)
    tol = co.tolerance(ref, F, A, wl.w)
    assert np.all(np.abs(got - ref) <= tol)
