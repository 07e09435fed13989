"""The convolution family's search space and the tuner's strategies on it (no GPU): the library
must enumerate exactly the oracle's space for every filter size, agree with it on the derived
quantities, and walk the oracle's searches step by step on the same cost tables and seeds --
the strategies are the GEMM tuner's, used unchanged on a space of 8 parameters."""
import math

import numpy as np
import pytest

from oracle import conv_space_oracle as cs
from oracle import search_oracle as so
from paper_1703_06503_amd import binding as b


@pytest.mark.parametrize("Xf,Yf", [(1, 1), (3, 3), (7, 7), (11, 11), (5, 3), (2, 4), (31, 31)])
def test_library_space_is_the_oracles(Xf, Yf):
    want = cs.enumerate_space(Xf, Yf)
    n = b.conv2d_space_size(Xf, Yf)
    assert n == len(want)
    got = [b.conv2d_space_get(Xf, Yf, i) for i in range(n)]
    assert [c.as_tuple() for c in got] == want
    for i in range(0, n, 53):
        assert b.conv2d_space_find(Xf, Yf, got[i]) == i
        assert b.conv2d_config_lds_bytes(got[i], Xf, Yf) == cs.lds_bytes(want[i], Xf, Yf)
        assert b.conv2d_config_threads(got[i], Xf, Yf) == cs.threads(want[i], Xf, Yf)


def test_config_check_agrees_with_the_oracle_on_the_whole_product():
    import itertools
    for Xf, Yf in [(7, 7), (11, 3)]:
        for c in itertools.product(*cs.VALUES):
            ok = b.conv2d_config_check(b.make_conv_config(*c), Xf, Yf) == b.OK
            assert ok == cs.valid(c, Xf, Yf), c
    # values outside the lists, filters outside 1..31
    assert b.conv2d_config_check(b.make_conv_config(24, 8, 1, 1, 0, 1, 0, 1), 3, 3) == b.E_INVALID
    assert b.conv2d_config_check(b.make_conv_config(32, 8, 2, 1, 0, 4, 0, 1), 3, 3) == b.E_INVALID
    assert b.conv2d_config_check(b.make_conv_config(32, 8, 1, 1, 0, 1, 0, 1), 0, 3) == b.E_BADARG
    with pytest.raises(b.SgemmError):
        b.conv2d_space_size(32, 3)


def _costs(configs, seed, fail_fraction=0.03):
    rng = np.random.default_rng(seed)
    factors = []
    for d in range(8):
        vals = sorted({c[d] for c in configs})
        factors.append({v: float(f) for v, f in zip(vals, rng.uniform(0.6, 1.8, len(vals)))})
    t = np.array([math.prod(factors[d][c[d]] for d in range(8)) for c in configs])
    t *= rng.uniform(0.9, 1.1, len(configs))
    t[rng.random(len(configs)) < fail_fraction] = -1.0
    return t.astype(np.float32)


def _opts(**kw):
    o = b.tune_opts()
    for k, v in kw.items():
        setattr(o, k, v)
    return o


def test_strategies_walk_the_oracles_searches_on_the_convolution_space():
    cfgs = cs.enumerate_space(7, 7)
    vals = cs.VALUES
    budget = len(cfgs) // 32                       # the paper explores 1/32 of its space
    for seed in (0, 5):
        t = _costs(cfgs, 70 + seed)
        ev, res, v = b.conv2d_tune_replay(7, 7, t, b.STRATEGY_FULL, 0, seed)
        want = so.full_search(cfgs, t)
        assert (ev, res.best_index, v) == (want["evaluations"], want["best_index"], want["visited"])
        assert res.best.as_tuple() == cfgs[want["best_index"]] and res.space_size == len(cfgs)
        ev, res, v = b.conv2d_tune_replay(7, 7, t, b.STRATEGY_RANDOM, budget, seed)
        assert v == so.random_search(cfgs, t, budget, seed)["visited"]
        for T in (2.0, 4.0, 6.0):
            ev, res, v = b.conv2d_tune_replay(7, 7, t, b.STRATEGY_ANNEALING, budget, seed, _opts(sa_T=T))
            want = so.simulated_annealing(cfgs, vals, t, budget, seed, T=T)
            assert v == want["visited"] and res.best_index == want["best_index"]
        for S in (3, 6):
            ev, res, v = b.conv2d_tune_replay(7, 7, t, b.STRATEGY_PSO, budget, seed, _opts(pso_S=S))
            want = so.particle_swarm(cfgs, vals, t, budget, seed, S=S)
            assert v == want["visited"] and res.best_index == want["best_index"]
            assert res.evals_to_best == want["evals_to_best"]
    with pytest.raises(b.SgemmError):
        b.conv2d_tune_replay(7, 7, t[:10], b.STRATEGY_FULL, 0, 0)


def test_variants_compile_without_a_gpu_and_report_their_resources(tmp_path):
    for cfg, f in [((32, 8, 2, 4, 2, 2, 1, 1), 7), ((16, 16, 1, 1, 1, 1, 0, 0), 3), ((64, 8, 1, 8, 0, 1, 0, 1), 11)]:
        c = b.make_conv_config(*cfg)
        for edge in (0, 1):
            info = b.conv2d_kernel_compile(c, f, f, edge, 1)
            assert info.scratch_bytes == 0 and info.vgprs > 0
            assert info.lds_bytes == cs.lds_bytes(cfg, f, f)
    with pytest.raises(b.SgemmError):
        b.conv2d_kernel_compile(b.make_conv_config(64, 64, 1, 1, 0, 1, 0, 1), 3, 3)


def test_table_of_best_configurations_round_trips_and_selects_the_nearest(tmp_path):
    b.conv2d_cache_clear()
    a7 = b.make_conv_config(32, 8, 8, 2, 0, 8, 0, 1)
    b7 = b.make_conv_config(16, 16, 4, 4, 2, 4, 1, 1)
    b.conv2d_config_set(8192, 4096, 7, 7, a7, 0.06)
    b.conv2d_config_set(512, 512, 7, 7, b7, 0.002)
    assert b.conv2d_config_select(8192, 4096, 7, 7)[0] == 1
    exact, near = b.conv2d_config_select(600, 400, 7, 7)             # nearest image, same filter
    assert exact == 0 and near.as_tuple() == b7.as_tuple()
    exact, other = b.conv2d_config_select(600, 400, 3, 3)            # unseen filter: built-in default
    assert exact == 0 and other.lmem == 0 and b.conv2d_config_check(other, 3, 3) == b.OK
    path = str(tmp_path / "conv.txt")
    assert b.conv2d_cache_save(path) == 2
    with open(path, "a") as f:
        f.write("100 100 7 7 0.5 64 64 1 1 0 1 0 1\n")                # too many threads: skipped
        f.write("8192 4096 7 7 0.5 8 8 1 1 0 1 0 1\n")                # slower than the entry held
        f.write("not a line\n")
    b.conv2d_cache_clear()
    assert b.conv2d_config_select(8192, 4096, 7, 7)[0] == 0
    assert b.conv2d_cache_load(path) == 3
    exact, got = b.conv2d_config_select(8192, 4096, 7, 7)
    assert exact == 1 and got.as_tuple() == a7.as_tuple()
    assert b.conv2d_config_select(100, 100, 7, 7)[0] == 0
    with pytest.raises(b.SgemmError):
        b.conv2d_cache_load(str(tmp_path / "missing.txt"))
    with pytest.raises(b.SgemmError):
        b.conv2d_config_set(8, 8, 7, 7, b.make_conv_config(64, 64, 1, 1, 0, 1, 0, 1))
    b.conv2d_cache_clear()
