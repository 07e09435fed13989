"""The enumerated search space of the library against an independent enumeration
(oracle/space_oracle.py), plus brute-force checks of the constraints themselves."""
import os

import numpy as np
import pytest

from oracle import space_oracle as so
from paper_1703_06503_amd import binding as b


@pytest.mark.parametrize("preset", [b.SPACE_FULL, b.SPACE_SMALL, b.SPACE_MFMA, b.SPACE_EXT,
                                    b.SPACE_DIRECT, b.SPACE_KSPLIT])
def test_space_equals_oracle_enumeration(preset):
    want = so.enumerate_space(preset)
    n = b.sgemm_space_size(preset)
    assert n == len(want)
    assert b.sgemm_space_raw_size(preset) == so.raw_size(preset)
    assert b.sgemm_space_dims(preset) == len(so.NAMES) == 16
    for d in range(16):
        assert b.sgemm_space_values(preset, d) == list(so.VALUES[preset][d])
    step = 1 if n < 2000 else (7 if n < 50000 else 101)
    for i in list(range(0, n, step)) + [n - 1]:
        assert b.sgemm_space_get(preset, i).as_tuple() == want[i], i
    # find() is the inverse of get()
    for i in np.random.default_rng(0).choice(n, size=min(n, 200), replace=False):
        assert b.sgemm_space_find(preset, b.make_config(*want[int(i)])) == int(i)


def test_sizes():
    assert b.sgemm_space_size(b.SPACE_SMALL) == 16          # benchmark configuration 1
    assert 5000 <= b.sgemm_space_size(b.SPACE_FULL) <= 30000  # "about 10^4"
    assert b.sgemm_space_raw_size(b.SPACE_FULL) == 4 * 4 * 3 * 2 * 2 * 2 * 2 * 2 * 2 * 2 * 2 * 2 * 2


def test_config_check_agrees_with_oracle_on_the_raw_product():
    """Every point of the raw cartesian product of a preset, valid or not."""
    import itertools
    for preset in (b.SPACE_SMALL, b.SPACE_MFMA, b.SPACE_EXT, b.SPACE_DIRECT, b.SPACE_KSPLIT):
        lists = so.VALUES[preset]
        rng = np.random.default_rng(preset)
        for _ in range(1500):
            cfg = tuple(int(v[rng.integers(len(v))]) for v in lists)
            assert (b.sgemm_config_check(b.make_config(*cfg)) == 0) == so.valid(cfg), cfg


def test_tile_edges_with_odd_factors_agree_with_the_oracle():
    """Edges of 3, 5 and 7 times a power of two are tile sizes, other multiples of 8 are not; the
    library and the oracle draw the line at the same place and agree on everything behind it."""
    edges = [40, 48, 56, 72, 80, 88, 96, 104, 112, 120, 144, 160, 176, 192, 208, 224, 240, 320, 448]
    assert [e for e in edges if so.tile_edge_ok(e)] == [40, 48, 56, 80, 96, 112, 160, 192, 224, 320, 448]
    rng = np.random.default_rng(7)
    seen_valid = 0
    for _ in range(3000):
        cfg = (int(rng.choice(edges)), int(rng.choice(edges)), int(rng.choice([32, 64])), int(rng.choice([8, 16, 32])),
               int(rng.choice([8, 16, 32])), 4, 4, 1, 1, int(rng.integers(2)), int(rng.choice([8, 16])),
               int(rng.choice([1, 2])), int(rng.integers(2)), int(rng.choice([1, 2, 4])), 2, int(rng.choice([1, 2, 4])))
        ok = b.sgemm_config_check(b.make_config(*cfg)) == 0
        assert ok == so.valid(cfg), cfg
        seen_valid += ok
    assert seen_valid > 15          # most of the list is not a tile size, or no wave tile fits
    for cfg in [(160, 160, 32, 16, 16, 4, 4, 1, 1, 1, 8, 2, 1, 1, 2, 1), (224, 224, 32, 16, 16, 4, 4, 1, 1, 1, 8, 2, 1, 1, 2, 1)]:
        assert so.valid(cfg) and b.sgemm_config_check(b.make_config(*cfg)) == 0      # the built-in templates


def test_every_emitted_config_meets_the_device_limits():
    for preset in (b.SPACE_FULL, b.SPACE_MFMA, b.SPACE_EXT, b.SPACE_DIRECT, b.SPACE_KSPLIT):
        n = b.sgemm_space_size(preset)
        for i in range(0, n, 11 if n < 50000 else 173):
            c = b.sgemm_space_get(preset, i)
            t = c.as_tuple()
            threads = c.mdimc * c.ndimc * c.ksw
            assert threads % 64 == 0 and threads <= 1024
            assert c.mwg % c.mdimc == 0 and c.nwg % c.ndimc == 0 and c.kwg % (c.kwi * c.ksw) == 0
            assert c.ksw == 1 or c.mfma
            lds = b.sgemm_config_lds_bytes(c)
            assert lds == so.worst_lds_bytes(t) <= 160 * 1024
            if c.sa:
                assert (c.mwg * c.kwg) % (threads * c.vwm) == 0
            if c.sb:
                assert (c.nwg * c.kwg) % (threads * c.vwn) == 0
            if c.mfma:
                tile = 32 if c.mfma == 1 else 16
                assert (8 * c.mwg // c.mdimc) % tile == 0 and (8 * c.nwg // c.ndimc) % tile == 0


def test_paper_style_best_configs_are_not_rejected_by_divisibility():
    """The paper's Table IV winners, mapped onto this parameterisation (tile, workgroup shape,
    vector widths, KWI; both operands staged), satisfy the divisibility constraints; whatever
    is rejected is rejected for a gfx950 reason (workgroup not a multiple of 64 lanes)."""
    table4 = {
        "K40m": (128, 128, 16, 16, 16, 2, 1, 8),
        "GTX480": (64, 64, 32, 8, 16, 2, 2, 8),
        "HD7970": (128, 128, 32, 16, 16, 4, 4, 2),
        "Iris": (64, 64, 16, 8, 8, 4, 4, 8),
    }
    for dev, (mwg, nwg, kwg, mdimc, ndimc, vwm, vwn, kwi) in table4.items():
        cfg = b.make_config(mwg, nwg, kwg, mdimc, ndimc, vwm, vwn, 1, 1, 1, kwi, 0, 0)
        assert b.sgemm_config_check(cfg) == 0, dev
        assert so.valid(cfg.as_tuple()), dev


def test_invalid_examples():
    ok = (64, 64, 16, 8, 8, 4, 4, 1, 1, 1, 8, 1, 0)
    assert b.sgemm_config_check(b.make_config(*ok)) == 0
    for field, value in [("mwg", 80), ("mwg", 48), ("kwg", 12), ("mdimc", 4), ("vwm", 3), ("kwi", 32),
                         ("mfma", 3), ("sa", 3), ("mwg", 1024), ("sk", -1), ("sk", 65), ("ns", 1), ("ns", 5),
                         ("ns", 3),       # three buffers need LDS-direct staging
                         ("ksw", 3), ("ksw", 8), ("ksw", 4)]:      # 16 is not divisible by 8 * 4
        c = b.make_config(*ok)
        setattr(c, field, value)
        assert b.sgemm_config_check(c) == b.E_INVALID, (field, value)
    # LDS capacity: 256 x 256 x 64 tiles double-buffered need 256 KiB
    big = b.make_config(256, 256, 64, 16, 16, 4, 4, 1, 1, 0, 8, 1, 0)
    assert b.sgemm_config_lds_bytes(big) == 2 * 4 * (2 * 256 * 64) > 160 * 1024
    assert b.sgemm_config_check(big) == b.E_INVALID


def test_predicted_lds_size_matches_the_compiled_variants(tmp_path):
    """The LDS model that prunes the space (oracle and library) against what the compiler
    really allocates, for a few variants of every preset, in the layout that needs most."""
    import os
    b.sgemm_kernel_cache_dir(str(tmp_path))
    try:
        for preset in (b.SPACE_FULL, b.SPACE_MFMA, b.SPACE_EXT, b.SPACE_DIRECT, b.SPACE_KSPLIT):
            n = b.sgemm_space_size(preset)
            rng = np.random.default_rng(100 + preset)
            checked = 0
            for i in rng.choice(n, size=40, replace=False):
                c = b.sgemm_space_get(preset, int(i))
                if c.mdimc * c.ndimc * c.ksw > 256 or c.mwg * c.nwg > 128 * 128:
                    continue            # keep to variants that compile in about a second
                t = c.as_tuple()
                layout = max(range(4), key=lambda l: so.lds_bytes(t, l))
                info = b.sgemm_kernel_compile(c, layout, 0)
                assert info.lds_bytes == so.lds_bytes(t, layout) == b.sgemm_config_lds_bytes(c), t
                checked += 1
                if checked == 4:
                    break
            assert checked >= 2
    finally:
        b.sgemm_kernel_cache_dir(os.path.join(os.path.dirname(b.LIB_PATH), "kcache"))


# ---- pins of the device-limit rules that no closed form fixes: the compiler decides ---------
# (paper, "Advanced usage": configurations that exceed a device limit are pruned.  The register
# file and the counter of outstanding loads are such limits; what a variant needs of them is
# known exactly only after compilation, so the oracle's rules are held to the compiler here.)

KERNEL_SOURCE = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))),
                             "paper_1703_06503_amd", "csrc", "sgemm_kernel.hip.inc")
MACRO_NAMES = ("MWG", "NWG", "KWG", "MDIMC", "NDIMC", "VWM", "VWN", "SA", "SB", "PAD", "KWI", "MFMA", "GRP")


def compile_raw(cfg, layout=0, edge=0):
    """Compile the kernel family's source for ANY parameter values, valid or not, through the
    generic tuner (which knows nothing of the GEMM constraints); returns the compiler's report
    or raises SgemmError with the compiler's message."""
    ksw = cfg[15] if len(cfg) > 15 else 1
    text = (f"#define TRA {layout & 1}\n#define TRB {layout >> 1}\n#define EDGE {edge}\n#define NS {cfg[14]}\n"
            f"#define KSW {ksw}\n" + open(KERNEL_SOURCE).read())
    t = b.ktuner_create(text, "sgemm_variant", (64, 1, 1), (64, 1, 1))
    try:
        for name, value in zip(MACRO_NAMES, cfg):
            b.ktuner_add_parameter(t, name, [int(value)])
        assert b.ktuner_space_size(t) == 1
        return b.ktuner_compile(t, 0)
    finally:
        b.ktuner_destroy(t)


def test_register_model_against_the_compiler():
    """A seeded sample of what the oracle admits, compiled for gfx950 (no GPU needed): the
    compiler never exceeds the register budget the oracle derives from the workgroup size, it
    keeps at least the accumulators the oracle counts, and (almost) nothing admitted spills -
    also in the riskiest corner, where the accumulators take half of the budget."""
    rng = np.random.default_rng(77)
    sample = []
    for preset in (so.SPACE_FULL, so.SPACE_MFMA, so.SPACE_EXT, so.SPACE_DIRECT, so.SPACE_KSPLIT):
        space = so.enumerate_space(preset) if preset in (so.SPACE_FULL, so.SPACE_MFMA, so.SPACE_KSPLIT) else None
        if space is None:      # the two large presets: draw from the raw product, keep the valid
            lists = so.VALUES[preset]
            space = []
            while len(space) < 400:
                cfg = tuple(int(v[rng.integers(len(v))]) for v in lists)
                if so.valid(cfg):
                    space.append(cfg)
        picks = [space[int(i)] for i in rng.choice(len(space), size=10, replace=False)]
        corner = [c for c in space if c[11] and 2 * so.register_estimate(c)[0] == so.register_budget(c[3] * c[4] * c[15])]
        picks += [corner[int(i)] for i in rng.choice(len(corner), size=min(4, len(corner)), replace=False)]
        sample += picks
    spilled = []
    for cfg in sample:
        threads = cfg[3] * cfg[4] * cfg[15]
        acc, other = so.register_estimate(cfg)
        info = b.sgemm_kernel_compile(b.make_config(*cfg), 0, 0)
        # registers reported: architected + accumulation together (unified file)
        assert info.vgprs <= so.register_budget(threads), (cfg, info.vgprs)
        assert info.vgprs >= acc, (cfg, info.vgprs, acc)
        if info.scratch_bytes > 0:
            spilled.append(cfg)
    assert len(sample) >= 60
    assert len(spilled) <= 2, spilled           # under 4 % of the sample, corner cases included


def test_what_the_register_model_rejects_does_spill():
    """Three configurations that only the register rules reject (every divisibility and LDS
    rule holds), one per rule: they compile, and the compiler reports spills."""
    cases = [
        # 16x16x4 tiles with all 256 accumulation registers taken by accumulators
        (256, 256, 16, 16, 16, 4, 4, 1, 1, 1, 8, 2, 0, 1, 2, 1),
        # 1024 threads leave 128 registers per lane: 64 accumulators and the rest do not fit
        (256, 256, 16, 32, 32, 4, 4, 1, 1, 1, 8, 1, 0, 1, 2, 1),
        # one wave, 256 accumulators, and 160 staging registers on top
        (64, 256, 32, 8, 8, 4, 4, 1, 1, 1, 8, 1, 0, 1, 2, 1),
    ]
    for cfg in cases:
        assert not so.registers_fit(cfg) and not so.valid(cfg), cfg
        relaxed = so.registers_fit
        so.registers_fit = lambda c: True
        try:
            assert so.valid(cfg), cfg           # nothing but the register rules is in the way
        finally:
            so.registers_fit = relaxed
        assert b.sgemm_config_check(b.make_config(*cfg)) == b.E_INVALID
        info = compile_raw(cfg)
        assert info.scratch_bytes > 0, (cfg, info.vgprs)


def test_builds_that_read_c_ahead_keep_their_registers():
    """Calls with beta != 0 get the build that requests the old C before the main loop where the
    library's rule says a lane can hold it (twice the accumulators plus the estimate within the
    budget and within 256 architected registers).  A seeded sample of matrix-core configurations
    for which the rule says yes compiles without spills in that build; one it refuses (a single
    wave with 128 accumulators: fine against the 512 registers of its budget, not against 256)
    spills when the build is forced."""
    rng = np.random.default_rng(78)
    space = [c for c in so.enumerate_space(so.SPACE_MFMA)] + [c for c in so.enumerate_space(so.SPACE_KSPLIT)]
    chosen, tried = [], 0
    while len(chosen) < 16 and tried < 400:
        cfg = space[int(rng.integers(len(space)))]
        tried += 1
        M, N, K = 4 * cfg[0], 4 * cfg[1], 8 * cfg[2]
        variant, build = b.sgemm_kernel_resolve(b.make_config(*cfg), M, N, K, K, N, N, 0, 1.0)
        if build & b.BUILD_READS_C_AHEAD:
            chosen.append((cfg, variant, build))
    assert len(chosen) == 16
    spilled = [cfg for cfg, variant, build in chosen if b.sgemm_kernel_compile(variant, 0, build).scratch_bytes > 0]
    assert len(spilled) <= 1, spilled
    refused = b.make_config(128, 64, 32, 8, 8, 4, 4, 1, 1, 0, 8, 2, 0, 1, 2, 1)
    assert b.sgemm_config_check(refused) == 0
    assert b.sgemm_kernel_resolve(refused, 512, 256, 256, 256, 256, 256, 0, 1.0)[1] == 0
    assert b.sgemm_kernel_compile(refused, 0, 0).scratch_bytes == 0
    assert b.sgemm_kernel_compile(refused, 0, b.BUILD_READS_C_AHEAD).scratch_bytes > 0


def test_loads_in_flight_rule_is_what_the_kernel_itself_asserts():
    """More than two LDS buffers keep the loads of NS - 2 slabs in flight behind the slab that
    is waited for, and the wait is a 6-bit count: the kernel source refuses to compile beyond
    63.  The oracle's rule draws the same line: 2 x 32 loads is rejected, 1 x 32 is admitted."""
    four = (64, 64, 64, 16, 16, 1, 1, 2, 2, 0, 8, 1, 0, 1, 4, 1)      # 32 loads per slab and thread
    three = four[:14] + (3, 1)
    assert so.valid(three) and not so.valid(four)
    assert b.sgemm_config_check(b.make_config(*three)) == 0
    assert b.sgemm_config_check(b.make_config(*four)) == b.E_INVALID
    assert compile_raw(three).scratch_bytes == 0
    with pytest.raises(b.SgemmError) as e:
        compile_raw(four)
    assert "too many LDS-direct loads in flight" in str(e.value)
