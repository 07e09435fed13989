"""The C-ABI library loads without a GPU and exports every symbol the headers under include/
declare; host-only entry points answer; argument checks reject bad input before any launch."""
import ctypes
import os
import re

import pytest

from paper_1703_06503_amd import binding as b

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    names = set()
    for header in sorted(os.listdir(os.path.join(ROOT, "include"))):
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b([a-z_0-9]+)\s*\(", text))
    return sorted(names - {"defined", "int"})     # "int (*callback_type)(...)" is no function


def test_every_declared_symbol_is_exported_and_bound():
    lib = ctypes.CDLL(b.LIB_PATH) if False else b.lib()
    names = declared_symbols()
    assert "sgemm_tuned" in names and "tune" in names and len(names) >= 25
    for n in names:
        assert hasattr(lib, n), f"{n} declared in the header but not exported"
        assert n in b.EXPORTS, f"{n} has no Python binding"
        assert callable(getattr(b, n)), n
    assert sorted(b.EXPORTS) == names


def test_status_strings():
    assert b.sgemm_status_string(0) == "ok"
    for code in range(-10, 0):
        assert b.sgemm_status_string(code) not in ("ok", "unknown status")
    assert b.sgemm_status_string(-99) == "unknown status"


def test_struct_sizes_match_the_header():
    assert ctypes.sizeof(b.sgemm_config) == 16 * 4
    assert ctypes.sizeof(b.sgemm_kernel_info) == 8 * 4
    assert ctypes.sizeof(b.tune_result) == 16 * 4 + 9 * 4 + 6 * 4
    assert ctypes.sizeof(b.conv2d_config) == 8 * 4
    assert ctypes.sizeof(b.conv2d_tune_result) == 8 * 4 + 10 * 4 + 4 * 4


def test_bad_arguments_are_rejected_without_a_gpu():
    cfg = b.sgemm_config_default(256, 256, 256)
    with pytest.raises(b.SgemmError) as e:
        b.sgemm_run_config(0, cfg, -1, 4, 4, 1.0, 0, 4, 0, 4, 0.0, 0, 4, 0)
    assert e.value.status == b.E_BADARG
    with pytest.raises(b.SgemmError) as e:      # null C for a non-empty problem
        b.sgemm_tuned_on(0, 4, 4, 4, 1.0, 1, 4, 1, 4, 0.0, None, 4, 0)
    assert e.value.status == b.E_BADARG
    with pytest.raises(b.SgemmError) as e:      # unknown layout
        b.sgemm_reference(0, 4, 4, 4, 1.0, 1, 4, 1, 4, 0.0, 1, 4, 4)
    assert e.value.status == b.E_BADARG
    with pytest.raises(b.SgemmError) as e:
        b.tune_ex(0, 4, 4, 0, 1.0, 0.0, b.STRATEGY_FULL, 0)
    assert e.value.status == b.E_BADARG
    with pytest.raises(b.SgemmError) as e:
        b.tune_ex(4, 4, 4, 0, 1.0, 0.0, 17, 0)
    assert e.value.status == b.E_BADARG
    # sizes so close to 2^31 that rounding them up to a tile would leave an int are refused
    huge = 2**31 - 1
    with pytest.raises(b.SgemmError) as e:
        b.sgemm_tuned_on(0, huge, 4, 4, 1.0, 1, 4, 1, 4, 0.0, 1, 4, 0)
    assert e.value.status == b.E_BADARG
    for call in (lambda: b.sgemm_config_default(huge, 4, 4), lambda: b.sgemm_config_select(4, huge, 4, 0),
                 lambda: b.sgemm_config_workspace_bytes(cfg, 4, 4, huge),
                 lambda: b.sgemm_kernel_resolve(cfg, huge, 4, 4, 4, 4, 4, 0, 0.0)):
        with pytest.raises(b.SgemmError) as e:
            call()
        assert e.value.status == b.E_BADARG
    assert b.sgemm_config_check(b.sgemm_config_default(2**31 - 1025, 4, 4)) == 0      # the largest size there is
    # a prepared call (arguments marshalled once) reports what the ordinary call reports
    with pytest.raises(b.SgemmError) as e:
        b.sgemm_tuned_prepare(0, -1, 4, 4, 1.0, 0, 4, 0, 4, 0.0, 0, 4, 0)()
    assert e.value.status == b.E_BADARG
    assert b.sgemm_tuned_prepare(0, 0, 4, 4, 1.0, 0, 4, 0, 4, 0.0, 0, 4, 0)() == 0
    # empty problems are fine and launch nothing
    assert b.sgemm_run_config(0, cfg, 0, 4, 4, 1.0, 0, 4, 0, 4, 0.0, 0, 4, 0) == 0


def test_kernel_generator_compiles_without_a_gpu(tmp_path):
    b.sgemm_kernel_cache_dir(str(tmp_path))
    try:
        cfg = b.make_config(64, 64, 16, 8, 8, 4, 4, 1, 1, 1, 8, 1, 0)
        info = b.sgemm_kernel_compile(cfg, 0, 1)
        assert info.from_cache == 0 and info.code_bytes > 1000 and info.scratch_bytes == 0
        assert info.lds_bytes == 2 * 4 * (64 * 20 + 16 * 68)        # row-major A and B
        assert b.sgemm_config_lds_bytes(cfg) == 2 * 4 * (64 * 20 + 64 * 20)   # worst layout
        assert b.sgemm_kernel_compile(cfg, 2, 0).lds_bytes == 2 * 4 * (64 * 20 + 64 * 20)
        assert info.agprs + info.vgprs >= 64            # 8 x 8 accumulators per lane
        where = b.sgemm_kernel_cache_path(cfg, 0, 1)
        assert where.startswith(str(tmp_path)) and where.endswith(".hsaco") and os.path.exists(where)
        assert b.sgemm_kernel_cache_path(cfg, 0, 0) != where
        assert not os.path.exists(b.sgemm_kernel_cache_path(cfg, 0, 0))
        again = b.sgemm_kernel_compile(cfg, 0, 1)
        assert again.from_cache == 1 and again.code_bytes == info.code_bytes
        macros = b.sgemm_kernel_macros(cfg, 3, 1)
        assert "-DMWG=64" in macros and "-DTRA=1" in macros and "-DTRB=1" in macros and "-DEDGE=1" in macros
        # LDS-direct staging with three buffers: dense (unpadded) tiles, NS of them
        direct = b.make_config(64, 64, 16, 8, 8, 4, 4, 2, 2, 0, 8, 1, 0, 1, 3)
        dinfo = b.sgemm_kernel_compile(direct, 0, 0)
        assert dinfo.lds_bytes == 3 * 4 * (64 * 16 + 16 * 64) and dinfo.scratch_bytes == 0
        assert "-DSA=2" in b.sgemm_kernel_macros(direct, 0, 0)
        assert "-DNS=3" in b.sgemm_kernel_macros(direct, 0, 0)
        assert b.sgemm_kernel_compile(direct, 1, 1).scratch_bytes == 0      # guarded form
        # the split itself is applied at launch: every sk > 1 shares one build, which differs
        # from the unsplit one only by the code that handles the partial planes
        split8 = b.make_config(64, 64, 16, 8, 8, 4, 4, 1, 1, 1, 8, 1, 0, 8)
        split3 = b.make_config(64, 64, 16, 8, 8, 4, 4, 1, 1, 1, 8, 1, 0, 3)
        assert b.sgemm_kernel_macros(split8, 0, 0) == b.sgemm_kernel_macros(split3, 0, 0)
        assert "-DSPLITK=1" in b.sgemm_kernel_macros(split8, 0, 0)
        assert (b.sgemm_kernel_macros(split8, 0, 0).replace("-DSPLITK=1", "-DSPLITK=0")
                == b.sgemm_kernel_macros(cfg, 0, 0))
        assert b.sgemm_kernel_compile(split8, 0, 1).scratch_bytes == 0
        bad = b.make_config(64, 64, 16, 8, 8, 4, 4, 0, 1, 1, 8, 1, 0)   # VWM without staging A
        with pytest.raises(b.SgemmError) as e:
            b.sgemm_kernel_compile(bad, 0, 0)
        assert e.value.status == b.E_INVALID
    finally:
        b.sgemm_kernel_cache_dir(os.path.join(os.path.dirname(b.LIB_PATH), "kcache"))


def test_split_k_plan_and_workspace_size():
    """sk workgroups per tile, limited to the number of K slabs, parts of whole slabs, none
    empty; the workspace holds one M x N plane per part."""
    cfg = b.make_config(64, 64, 32, 16, 16, 4, 4, 1, 1, 1, 8, 1, 0, 4)
    assert b.sgemm_config_workspace_bytes(cfg, 100, 50, 4096) == (4 * 100 * 50 * 4, 4, 1024)
    assert b.sgemm_config_workspace_bytes(cfg, 100, 50, 100) == (4 * 100 * 50 * 4, 4, 32)   # 4 slabs
    assert b.sgemm_config_workspace_bytes(cfg, 100, 50, 33) == (2 * 100 * 50 * 4, 2, 32)    # 2 slabs
    assert b.sgemm_config_workspace_bytes(cfg, 100, 50, 32) == (0, 1, 32)                   # 1 slab
    # 9 slabs over 4 parts: chunks of 3 slabs leave nothing for a fourth part
    assert b.sgemm_config_workspace_bytes(cfg, 8, 8, 9 * 32) == (3 * 8 * 8 * 4, 3, 96)
    # 10 slabs over 4 parts: 3, 3, 3, 1
    assert b.sgemm_config_workspace_bytes(cfg, 8, 8, 10 * 32) == (4 * 8 * 8 * 4, 4, 96)
    for K in range(1, 700, 13):
        for sk in (1, 2, 3, 4, 6, 8, 12, 16):
            c = b.make_config(64, 64, 32, 16, 16, 4, 4, 1, 1, 1, 8, 1, 0, sk)
            nbytes, parts, chunk = b.sgemm_config_workspace_bytes(c, 3, 5, K)
            slabs = -(-K // 32)
            assert 1 <= parts <= min(sk, slabs)
            if parts > 1:
                assert chunk % 32 == 0 and (parts - 1) * chunk < K <= parts * chunk
                assert nbytes == parts * 3 * 5 * 4
            else:
                assert chunk == K and nbytes == 0
    unsplit = b.make_config(64, 64, 32, 16, 16, 4, 4, 1, 1, 1, 8, 1, 0)
    assert b.sgemm_config_workspace_bytes(unsplit, 100, 50, 4096) == (0, 1, 4096)


def test_default_configuration_is_valid_and_sized_to_the_problem():
    """What sgemm_tuned() falls back on when nothing was tuned for a storage layout."""
    sizes = [1, 7, 64, 100, 256, 1000, 1536, 3000, 4096, 20000]
    for M in sizes:
        for N in sizes:
            for K in (1, 33, 2048, 9216):
                c = b.sgemm_config_default(M, N, K)
                assert b.sgemm_config_check(c) == 0, (M, N, K, c)
                assert c.mfma in (1, 2) and c.sa == c.sb == 1
                nbytes, parts, chunk = b.sgemm_config_workspace_bytes(c, M, N, K)
                assert 1 <= parts <= 16
    # degenerate sizes get an answer too (a call with K = 0 or an empty C launches no variant at all)
    for shape in [(0, 0, 0), (5, 7, 0), (0, 9, 100), (1, 1, 1)]:
        c = b.sgemm_config_default(*shape)
        assert b.sgemm_config_check(c) == 0 and b.sgemm_config_select(*shape, 2).as_tuple() == c.as_tuple()
        assert b.sgemm_config_workspace_bytes(c, *shape)[1] == 1
    # whole rounds of 256 workgroups where the size allows it
    assert b.sgemm_config_default(4096, 4096, 4096).mwg == 256
    assert b.sgemm_config_default(3000, 3000, 3000).mwg == 192        # 16 x 16 tiles
    assert b.sgemm_config_default(1536, 1536, 1536).mwg == 96         # 16 x 16 tiles
    # the tile is chosen for how its grid quantises the problem, not for its size: 6144 = 48 x 128
    # gives nine whole rounds of 256 workgroups where the 256-wide tile would run 2.25 (three)
    c = b.sgemm_config_default(6144, 6144, 6144)
    assert (c.mwg, c.nwg) == (128, 128) and (6144 // 128) ** 2 % 256 == 0
    assert b.sgemm_config_default(5120, 5120, 5120).mwg == 160        # 32 x 32 tiles: four whole rounds
    assert b.sgemm_config_default(3584, 3584, 3584).mwg == 224        # 16 x 16 tiles
    assert b.sgemm_config_default(512, 512, 512).mwg == 32            # 256 tiles of 32 x 32
    # few tiles and a long K: split K, into parts that put two workgroups on every CU
    assert b.sgemm_config_default(128, 4096, 4096).sk > 1
    assert b.sgemm_config_default(128, 4096, 64).sk == 1
    c = b.sgemm_config_default(64, 8192, 8192)
    assert (c.mwg, c.nwg, c.sk) == (64, 64, 4)                        # 128 tiles x 4 parts = 2 x 256


def test_per_shape_cache_roundtrip(tmp_path):
    b.sgemm_cache_clear()
    assert b.sgemm_cache_count() == 0 and b.sgemm_config_get(512, 512, 512, 0) is None
    c1 = b.make_config(64, 64, 16, 8, 8, 4, 4, 1, 1, 1, 8, 1, 0)
    c2 = b.make_config(128, 128, 16, 16, 16, 4, 4, 2, 2, 0, 8, 1, 1, 4, 3)   # split K, 3 buffers
    b.sgemm_config_set(512, 512, 512, 0, c1, 0.01)
    b.sgemm_config_set(4096, 4096, 4096, 0, c2, 1.0)
    assert b.sgemm_config_get(512, 512, 512, 0).as_tuple() == c1.as_tuple()
    # a miss takes the nearest tuned shape's configuration where the call has that shape's launch
    # geometry (the same grid of tiles and the same split of K) ...
    assert b.sgemm_config_select(500, 490, 500, 0).as_tuple() == c1.as_tuple()
    assert b.sgemm_config_select(4000, 4090, 4000, 0).as_tuple() == c2.as_tuple()
    # ... and otherwise only if no built-in template quantises the problem better: here one does
    assert b.sgemm_config_select(600, 500, 512, 0).as_tuple() == b.sgemm_config_default(600, 500, 512, 0).as_tuple()
    assert b.sgemm_config_select(3000, 3000, 3000, 0).as_tuple() == b.sgemm_config_default(3000, 3000, 3000, 0).as_tuple()
    assert b.sgemm_config_select(512, 512, 512, 1).as_tuple() == b.sgemm_config_default(512, 512, 512, 1).as_tuple()
    path = str(tmp_path / "cache.txt")
    b.sgemm_cache_save(path)
    b.sgemm_cache_clear()
    assert b.sgemm_cache_count() == 0
    b.sgemm_cache_load(path)
    assert b.sgemm_cache_count() == 2
    assert b.sgemm_config_get(4096, 4096, 4096, 0).as_tuple() == c2.as_tuple()
    # a table written before the SK, NS and KSW columns existed still loads (SK = 1, NS = 2, KSW = 1)
    old = tmp_path / "old.txt"
    old.write_text("# M N K layout ms MWG NWG KWG MDIMC NDIMC VWM VWN SA SB PAD KWI MFMA GRP\n"
                   "1024 1024 1024 0 0.05 128 128 16 16 16 4 4 1 1 1 8 1 1\n")
    b.sgemm_cache_load(str(old))
    got = b.sgemm_config_get(1024, 1024, 1024, 0)
    assert got.as_tuple() == (128, 128, 16, 16, 16, 4, 4, 1, 1, 1, 8, 1, 1, 1, 2, 1)
    c3 = b.make_config(64, 64, 64, 16, 16, 4, 4, 1, 1, 1, 8, 1, 1, 2, 2, 4)      # wave groups share K
    b.sgemm_config_set(800, 800, 800, 0, c3, 0.02)
    b.sgemm_cache_save(path)
    b.sgemm_cache_clear()
    b.sgemm_cache_load(path)
    assert b.sgemm_config_get(800, 800, 800, 0).as_tuple() == c3.as_tuple()
    with pytest.raises(b.SgemmError) as e:
        b.sgemm_cache_load(str(tmp_path / "missing.txt"))
    assert e.value.status == b.E_IO
    bad = b.make_config(100, 64, 16, 8, 8, 1, 1, 1, 1, 0, 2, 0, 0)
    with pytest.raises(b.SgemmError) as e:
        b.sgemm_config_set(1, 1, 1, 0, bad, 0.0)
    assert e.value.status == b.E_INVALID
    b.sgemm_cache_clear()


def test_dispatch_pads_only_large_problems_with_rows_that_break_the_load_vector():
    """Also: a row length that is even but not a multiple of 4 narrows a 4-float load to 2, not 1."""
    cfg = b.make_config(256, 256, 32, 32, 8, 4, 4, 1, 1, 0, 8, 1, 0, 1, 2)
    def pads(M, N, K, beta=0.0):
        return b.sgemm_config_prefers_padding(cfg, M, N, K, K, N, N, 0, beta)
    assert pads(4091, 4091, 4091) == 1 and pads(8191, 8191, 8191) == 1 and pads(6143, 6143, 6143, 1.0) == 1
    assert pads(4093, 4093, 4093, 1.0) == 0       # beta != 0 adds two copies of C: not yet worth it
    assert pads(4090, 4090, 4090) == 0 and pads(8190, 8190, 8190) == 0   # even rows keep 2-float loads
    assert pads(4096, 4096, 4096) == 0            # multiples of the tile: nothing to guard
    assert pads(3000, 3000, 3000) == 0            # rows are multiples of 4: guards cost little
    assert pads(4090, 4096, 4096) == 0            # only M is ragged: no stored row is cut
    assert pads(1021, 1021, 1021) == 0            # too small for the copies to pay
    v, edge = b.sgemm_kernel_resolve(cfg, 4090, 4090, 4090, 4090, 4090, 4090, 0)
    assert (v.vwm, v.vwn, edge) == (2, 2, 1)
    v, edge = b.sgemm_kernel_resolve(cfg, 4091, 4091, 4091, 4091, 4091, 4091, 0)
    assert (v.vwm, v.vwn, edge) == (1, 1, 1)
    scalar = b.make_config(64, 64, 16, 8, 8, 1, 1, 1, 1, 0, 8, 0, 0, 1, 2)
    assert b.sgemm_config_prefers_padding(scalar, 4091, 4091, 4091, 4091, 4091, 4091, 0, 0.0) == 0


def test_calls_that_read_c_get_the_build_that_requests_it_ahead_where_registers_allow():
    """beta != 0 on the matrix-core schedule: the build reads the old C before the main loop
    when a lane can hold it beside its accumulators; never for split-K launches (the reduction
    reads C), never on the vector-ALU schedule, never for beta == 0."""
    def build(cfg, M, N, K, beta):
        return b.sgemm_kernel_resolve(cfg, M, N, K, K, N, N, 0, beta)[1]
    mid = b.make_config(192, 192, 32, 32, 16, 4, 4, 1, 1, 1, 8, 2, 1, 1, 2)      # 72 accumulators of 256 registers
    assert build(mid, 3000, 3000, 3000, 1.0) == b.BUILD_GUARDED | b.BUILD_READS_C_AHEAD
    assert build(mid, 3000, 3000, 3000, 0.0) == b.BUILD_GUARDED
    assert build(mid, 3072, 3072, 3072, 0.5) == b.BUILD_READS_C_AHEAD
    big = b.make_config(256, 256, 32, 32, 8, 4, 4, 1, 1, 0, 8, 1, 0, 1, 2)       # 256 accumulators: no room
    assert build(big, 4096, 4096, 4096, 1.0) == 0
    split = b.make_config(64, 64, 64, 16, 16, 4, 4, 1, 1, 0, 8, 1, 1, 4, 2)
    assert build(split, 128, 4096, 4096, 1.0) == 0
    valu = b.make_config(64, 64, 16, 8, 8, 4, 4, 1, 1, 0, 8, 0, 0, 1, 2)
    assert build(valu, 1024, 1024, 1024, 1.0) == 0
    assert "-DCPF=1" in b.sgemm_kernel_macros(mid, 0, b.BUILD_READS_C_AHEAD)
    assert "-DCPF" not in b.sgemm_kernel_macros(mid, 0, b.BUILD_GUARDED)
    assert "-DCPF" not in b.sgemm_kernel_macros(valu, 0, b.BUILD_READS_C_AHEAD)
    paths = {b.sgemm_kernel_cache_path(mid, 0, f) for f in (0, 1, 2, 3)}
    assert len(paths) == 4                                                      # four builds, four code objects


def test_a_tuned_configuration_is_only_lent_to_shapes_like_its_own():
    """Dispatch on a miss: the nearest tuned shape of the same storage layout serves a call only
    when the shapes are alike; otherwise the built-in rule plans tile and split K for the
    actual sizes.  The A-transposed table holds two skinny split-K shapes only: a cube in
    that layout must not inherit their split K."""
    table = os.path.join(os.path.dirname(b.LIB_PATH), "..", "tuned_configs.txt")
    b.sgemm_cache_clear()
    b.sgemm_cache_load(table)
    try:
        skinny = b.sgemm_config_get(128, 4096, 4096, 1)
        assert skinny is not None and skinny.sk > 1
        cube = b.sgemm_config_select(4096, 4096, 4096, 1)
        assert cube.as_tuple() == b.sgemm_config_default(4096, 4096, 4096, 1).as_tuple()
        assert cube.sk == 1
        assert b.sgemm_config_workspace_bytes(cube, 4096, 4096, 4096)[0] == 0
        # a shape close to the tuned one borrows its configuration: with the same launch geometry
        # always, with another one where the cost model finds no template that fits better
        assert b.sgemm_config_select(100, 4090, 4000, 1).as_tuple() == skinny.as_tuple()
        assert b.sgemm_config_select(128, 4000, 4200, 1).as_tuple() == skinny.as_tuple()
        other = b.sgemm_config_select(160, 3072, 4096, 1)          # three rows of tiles instead of two
        assert other.as_tuple() == b.sgemm_config_default(160, 3072, 4096, 1).as_tuple()
        # and the exact shape gets its own
        assert b.sgemm_config_select(128, 4096, 4096, 1).as_tuple() == skinny.as_tuple()
    finally:
        b.sgemm_cache_clear()
        b.sgemm_cache_load(table)


def test_noalloc_entry_point_checks_its_arguments_like_the_others():
    with pytest.raises(b.SgemmError) as e:
        b.sgemm_tuned_noalloc(0, 4, 4, 4, 1.0, 1, 4, 1, 4, 0.0, None, 4, 0)
    assert e.value.status == b.E_BADARG
    assert b.sgemm_tuned_noalloc(0, 0, 4, 4, 1.0, 0, 4, 0, 4, 0.0, 0, 4, 0) == 0   # empty: no-op
    assert b.sgemm_status_string(b.E_NOTREADY) not in ("ok", "unknown status")
