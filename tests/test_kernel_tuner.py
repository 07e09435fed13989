"""The generic tuner (include/kernel_tuner.h): the paper's user-facing method for any HIP
kernel.  Host part: the space it builds from parameters, thread-count modifiers and constraints
is checked against a brute-force enumeration written here; GPU part: the paper's copy example,
a kernel with a parameter-dependent bug that verification must catch, and a constrained 2-D
kernel whose result is checked against numpy."""
import itertools
import json

import numpy as np
import pytest

from paper_1703_06503_amd import binding as b

COPY = r"""
extern "C" __global__ void copy(const float* in, float* out) {
    const int tid = blockIdx.x * blockDim.x + threadIdx.x;
    for (int w = 0; w < WPT; ++w) out[tid * WPT + w] = in[tid * WPT + w];
}
"""
COPY_REF = r"""
extern "C" __global__ void copy_ref(const float* in, float* out) {
    const int tid = blockIdx.x * blockDim.x + threadIdx.x;
    out[tid] = in[tid];
}
"""
# wrong for WPT == 4: the last element of each thread's run is doubled
COPY_BUG = COPY.replace("out[tid * WPT + w] = in[tid * WPT + w];",
                        "out[tid * WPT + w] = (WPT == 4 && w == 3 ? 2.0f : 1.0f) * in[tid * WPT + w];")
N = 1 << 20


def copy_tuner(source=COPY):
    """The paper's example ("Basic example of using CLTune on a kernel to copy ... elements")
    with its extension from "Advanced usage": work per thread WPT and workgroup size WG."""
    t = b.ktuner_create(source, "copy", (N, 1, 1), (1, 1, 1))
    b.ktuner_add_parameter(t, "WPT", [1, 2, 4])
    b.ktuner_add_parameter(t, "WG", [32, 64, 128, 256])
    b.ktuner_div_global_size(t, ["WPT", None, None])
    b.ktuner_mul_local_size(t, ["WG", None, None])
    return t


def test_space_is_the_constrained_product_with_thread_rules():
    t = b.ktuner_create(COPY, "copy", (4096, 64, 1), (1, 1, 1))
    vals = {"WPT": [1, 2, 3, 4], "XWG": [8, 16, 32, 64, 128], "YWG": [1, 4, 16, 128], "U": [0, 1]}
    for k, v in vals.items():
        b.ktuner_add_parameter(t, k, v)
    b.ktuner_div_global_size(t, ["WPT", None, None])
    b.ktuner_mul_local_size(t, ["XWG", "YWG", None])
    b.ktuner_add_constraint(t, lambda v: v[0] * v[1] >= 64, ["XWG", "YWG"])
    b.ktuner_add_constraint(t, lambda v: not (v[0] == 1 and v[1] == 3), ["U", "WPT"])
    want = []
    for wpt, xwg, ywg, u in itertools.product(*vals.values()):
        if xwg * ywg < 64 or (u == 1 and wpt == 3):
            continue
        if 4096 % wpt or (4096 // wpt) % xwg or 64 % ywg or xwg * ywg > 1024:
            continue                       # division with remainder, partial workgroups, device limit
        want.append((wpt, xwg, ywg, u))
    n = b.ktuner_space_size(t)
    assert [b.ktuner_space_get(t, i, 4) for i in range(n)] == want and n > 20
    i = want.index((2, 32, 4, 0))
    assert b.ktuner_launch_shape(t, i) == ((2048 // 32, 64 // 4, 1), (32, 4, 1))
    # modifiers apply in the order given: (N / WPT) * U' etc. -- a second modifier on the same size
    b.ktuner_mul_global_size(t, ["WPT", None, None])
    assert b.ktuner_launch_shape(t, i) == ((4096 // 32, 16, 1), (32, 4, 1))
    b.ktuner_destroy(t)


def test_bad_arguments_and_compilation_without_a_gpu():
    with pytest.raises(b.SgemmError):
        b.ktuner_create(COPY, "not an identifier", (1, 1, 1), (1, 1, 1))
    with pytest.raises(b.SgemmError):
        b.ktuner_create(COPY, "copy", (0, 1, 1), (1, 1, 1))
    t = copy_tuner()
    with pytest.raises(b.SgemmError):
        b.ktuner_add_parameter(t, "WPT", [8])                  # named twice
    with pytest.raises(b.SgemmError):
        b.ktuner_div_global_size(t, ["NOPE", None, None])
    with pytest.raises(b.SgemmError):
        b.ktuner_add_constraint(t, lambda v: True, ["NOPE"])
    assert b.ktuner_space_size(t) == 12
    info = b.ktuner_compile(t, 5)
    assert info.code_bytes > 0 and info.scratch_bytes == 0
    assert b.ktuner_compile(t, 5).from_cache == 1
    bad = b.ktuner_create("extern \"C\" __global__ void k(float* x) { x[0] = UNDECLARED; }", "k", (64, 1, 1), (64, 1, 1))
    b.ktuner_add_parameter(bad, "P", [1])
    with pytest.raises(b.SgemmError) as e:
        b.ktuner_compile(bad, 0)
    assert e.value.status == b.E_COMPILE and "UNDECLARED" in str(e.value)
    b.ktuner_destroy(bad)
    b.ktuner_destroy(t)


@pytest.mark.gpu
def test_copy_example_every_configuration_verified_and_timed(tmp_path):
    rng = np.random.default_rng(0)
    src, dst = rng.standard_normal(N).astype(np.float32), np.zeros(N, np.float32)
    t = copy_tuner()
    b.ktuner_add_argument_input(t, src)
    b.ktuner_add_argument_output(t, dst)
    b.ktuner_set_reference(t, COPY_REF, "copy_ref", (N, 1, 1), (256, 1, 1))
    o = b.tune_opts()
    o.reps, o.warmup_ms, o.log_path = 3, 1.0, str(tmp_path / "log.jsonl").encode()
    n, res = b.ktuner_tune(t, b.STRATEGY_FULL, 0, 0, o)
    assert (n, res.space_size, res.failed, res.failed_verify) == (12, 12, 0, 0)
    times = [b.ktuner_time_of(t, i) for i in range(12)]
    assert all(x > 0 for x in times) and res.best_ms == pytest.approx(min(times))
    lines = [json.loads(l) for l in open(tmp_path / "log.jsonl")]
    assert [l["config"] for l in lines] == [{"WPT": w, "WG": g} for w in (1, 2, 4) for g in (32, 64, 128, 256)]
    out = np.empty_like(dst)
    b.ktuner_read_output(t, 0, out)
    assert np.array_equal(out, src)
    # a budgeted heuristic search on the same tuner
    n, res = b.ktuner_tune(t, b.STRATEGY_ANNEALING, 5, 1, o)
    assert 1 <= n <= 5 and res.best_index >= 0
    b.ktuner_destroy(t)


@pytest.mark.gpu
def test_verification_catches_a_parameter_dependent_bug():
    rng = np.random.default_rng(1)
    src, dst = rng.uniform(1, 2, N).astype(np.float32), np.zeros(N, np.float32)
    t = copy_tuner(COPY_BUG)
    b.ktuner_add_argument_input(t, src)
    b.ktuner_add_argument_output(t, dst)
    b.ktuner_set_reference(t, COPY_REF, "copy_ref", (N, 1, 1), (256, 1, 1))
    o = b.tune_opts()
    o.reps, o.warmup_ms = 3, 1.0
    n, res = b.ktuner_tune(t, b.STRATEGY_FULL, 0, 0, o)
    assert (n, res.failed, res.failed_verify) == (12, 4, 4)
    for i in range(12):
        wpt, _ = b.ktuner_space_get(t, i, 2)
        assert (b.ktuner_time_of(t, i) < 0) == (wpt == 4)
    assert b.ktuner_space_get(t, res.best_index, 2)[0] != 4
    # without verification the wrong configurations are timed like the others
    o.verify_off = 1
    n, res = b.ktuner_tune(t, b.STRATEGY_FULL, 0, 0, o)
    assert res.failed == 0
    b.ktuner_destroy(t)


SCALE2D = r"""
extern "C" __global__ void scale2d(const float* in, float* out, int width, float factor) {
    const int x0 = (blockIdx.x * blockDim.x + threadIdx.x) * XW;
    const int y0 = (blockIdx.y * blockDim.y + threadIdx.y) * YW;
    for (int j = 0; j < YW; ++j)
        for (int i = 0; i < XW; ++i) out[(y0 + j) * width + x0 + i] = factor * in[(y0 + j) * width + x0 + i];
}
"""


@pytest.mark.gpu
def test_two_dimensional_kernel_with_scalars_and_a_constraint():
    W, H = 1024, 512
    rng = np.random.default_rng(2)
    src, dst = rng.standard_normal((H, W)).astype(np.float32), np.zeros((H, W), np.float32)
    t = b.ktuner_create(SCALE2D, "scale2d", (W, H, 1), (1, 1, 1))
    for name, vals in [("XW", [1, 2, 4]), ("YW", [1, 2]), ("XT", [16, 64, 256]), ("YT", [1, 4, 16])]:
        b.ktuner_add_parameter(t, name, vals)
    b.ktuner_div_global_size(t, ["XW", "YW", None])
    b.ktuner_mul_local_size(t, ["XT", "YT", None])
    b.ktuner_add_constraint(t, lambda v: 64 <= v[0] * v[1] <= 1024, ["XT", "YT"])
    b.ktuner_add_argument_input(t, src)
    b.ktuner_add_argument_output(t, dst)
    b.ktuner_add_argument_int(t, W)
    b.ktuner_add_argument_float(t, 2.5)
    size = b.ktuner_space_size(t)
    assert size == 3 * 2 * sum(1 for x in (16, 64, 256) for y in (1, 4, 16) if 64 <= x * y <= 1024)
    o = b.tune_opts()
    o.reps, o.warmup_ms = 3, 1.0
    n, res = b.ktuner_tune(t, b.STRATEGY_PSO, 12, 3, o)        # no reference kernel: timed only
    assert 1 <= n <= 12 and res.failed == 0
    out = np.empty_like(dst)
    b.ktuner_read_output(t, 0, out)
    assert np.array_equal(out, np.float32(2.5) * src)
    b.ktuner_destroy(t)
