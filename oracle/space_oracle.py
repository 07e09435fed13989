"""Oracle for the tuner's search space.  TEST INFRASTRUCTURE ONLY; shares no code with the
library.

The paper builds its space as the cartesian product of short per-parameter value lists,
pruned by user constraints and by device limits (sections "Advanced usage" and "Search
strategies and search-space properties").  This file writes out, in plain Python, the value
lists of the library's five presets and every constraint of its GEMM kernel family, and
enumerates the product in lexicographic order (first parameter slowest).

Parameters, in order: MWG NWG KWG MDIMC NDIMC VWM VWN SA SB PAD KWI MFMA GRP SK NS KSW.
(KSW: the K slab of a workgroup is shared out among KSW groups of waves, each group holding a
full set of accumulators for the whole tile; the groups' sums are added at the end.  The
workgroup then has MDIMC * NDIMC * KSW threads.)

parity unpinned: the paper's own count of 241 600 valid GEMM configurations cannot be
reproduced, because its constraint list is not printed; the counts here are pinned only by
the independent re-derivation below and by brute-force checks in the tests.
"""
import itertools

NAMES = ("MWG", "NWG", "KWG", "MDIMC", "NDIMC", "VWM", "VWN", "SA", "SB", "PAD", "KWI", "MFMA",
         "GRP", "SK", "NS", "KSW")

SPACE_FULL, SPACE_SMALL, SPACE_MFMA, SPACE_EXT, SPACE_DIRECT = 0, 1, 2, 3, 4
SPACE_KSPLIT = 6        # (5 is the caller-defined space)

VALUES = {
    SPACE_FULL: ([32, 64, 128, 256], [32, 64, 128, 256], [8, 16, 32], [8, 16], [8, 16], [1, 4],
                 [1, 4], [0, 1], [0, 1], [0, 1], [2, 8], [0, 1], [0, 1], [1], [2], [1]),
    SPACE_SMALL: ([32, 64], [32, 64], [8, 16], [8], [8], [1], [1], [0, 1], [0, 1], [0], [2], [0],
                  [0], [1], [2], [1]),
    SPACE_MFMA: ([64, 128, 256], [64, 128, 256], [8, 16, 32], [8, 16, 32], [8, 16, 32],
                 [1, 2, 4], [1, 2, 4], [1], [1], [0, 1], [2, 8], [1, 2], [0, 1], [1], [2], [1]),
    SPACE_EXT: ([32, 64, 96, 128, 192, 256], [32, 64, 96, 128, 192, 256], [16, 32, 64],
                [8, 16, 32], [8, 16, 32], [1, 2, 4], [1, 2, 4], [1], [1], [0, 1], [2, 8], [1, 2],
                [0, 1], [1, 2, 3, 4, 6, 8, 12, 16], [2], [1]),
    SPACE_DIRECT: ([32, 64, 96, 128, 192, 256], [32, 64, 96, 128, 192, 256], [16, 32, 64],
                   [8, 16, 32], [8, 16, 32], [1, 4], [1, 4], [2], [2], [0], [2, 8], [1, 2],
                   [0, 1], [1, 2, 3, 4, 6, 8, 12, 16], [2, 3, 4], [1]),
    # matrix-core variants whose waves share out the K slab: small tiles, 2 or 4 wave groups
    SPACE_KSPLIT: ([32, 64, 96, 128], [32, 64, 96, 128], [32, 64], [8, 16], [8, 16], [4], [4], [1],
                   [1], [0, 1], [2, 8], [1, 2], [0, 1], [1, 2, 4], [2], [2, 4]),
}

LDS_LIMIT = 160 * 1024          # bytes per workgroup on gfx950
MAX_THREADS = 1024
MAX_SPLIT_K = 64
MAX_LOADS_IN_FLIGHT = 63        # a wave's counter of outstanding vector-memory loads


def _pow2(v):
    return v > 0 and v & (v - 1) == 0


def tile_edge_ok(v):
    """A tile edge is 2^a, 3 * 2^a, 5 * 2^a or 7 * 2^a, between 8 and 512: the odd factors are
    there so that a grid of equal tiles can fill the 256 CUs in whole rounds for sizes that
    powers of two quantise badly (3000 = 15.6 x 192, 2560 = 16 x 160, 3584 = 16 x 224)."""
    return 8 <= v <= 512 and any(v % f == 0 and _pow2(v // f) for f in (1, 3, 5, 7))


def lds_bytes(cfg, layout):
    """NS buffers of each staged tile; a tile keeps the stored orientation of its matrix, and
    PAD adds 4 floats to every row of a register-staged tile (SA/SB = 1; a tile written by
    LDS-direct loads, SA/SB = 2, cannot be padded)."""
    MWG, NWG, KWG, _, _, _, _, SA, SB, PAD = cfg[:10]
    NS = cfg[14] if len(cfg) > 14 else 2
    KSW = cfg[15] if len(cfg) > 15 else 1
    pad_a = 4 if PAD and SA == 1 else 0
    pad_b = 4 if PAD and SB == 1 else 0
    floats = 0
    if SA:
        floats += KWG * (MWG + pad_a) if layout & 1 else MWG * (KWG + pad_a)
    if SB:
        floats += NWG * (KWG + pad_b) if layout & 2 else KWG * (NWG + pad_b)
    floats *= NS
    if KSW > 1:
        # the wave groups hand their sums over through LDS, one tile of C at a time, in the
        # memory of the tile buffers: the allocation is the larger of the two
        floats = max(floats, MWG * NWG)
    return 4 * floats


def worst_lds_bytes(cfg):
    return max(lds_bytes(cfg, layout) for layout in range(4))


# Register file of a gfx950 SIMD: 512 registers per lane (architected VGPRs and accumulation
# VGPRs together), shared by the waves resident on the SIMD; a wave addresses at most 256 of
# each kind.  A workgroup of T threads is T/64 waves on 4 SIMDs, so the compiler may give each
# wave no more than 512 / ceil(T/256) registers (its launch bound).
REGISTERS_PER_LANE = 512
MAX_ACCUMULATION_REGISTERS = 256


def register_budget(threads):
    waves_per_simd = -(-threads // 256)
    return REGISTERS_PER_LANE // waves_per_simd


def register_estimate(cfg):
    """(accumulators, everything else) a lane needs.  Everything else: two blocks of operand
    fragments (the block being multiplied and the one fetched ahead), the registers that stage
    the next slab on its way from global memory to LDS, two address registers per global load
    instruction of a slab, and 24 for loop state, tile origin and the epilogue.  The last two
    terms are fitted to what the compiler reports for sampled variants of every preset, under
    the condition that no configuration close to a measured optimum is rejected."""
    MWG, NWG, KWG, MDIMC, NDIMC, VWM, VWN, SA, SB, _, KWI, MFMA = cfg[:12]
    threads = MDIMC * NDIMC * (cfg[15] if len(cfg) > 15 else 1)
    MWI, NWI = MWG // MDIMC, NWG // NDIMC
    acc = MWI * NWI
    if MFMA:
        tile, depth = (32, 2) if MFMA == 1 else (16, 4)
        fragments = (8 * MWI // tile + 8 * NWI // tile) * (KWI // depth)
    else:
        fragments = MWI + NWI
    staging = loads = 0
    if SA:
        loads += MWG * KWG // (threads * VWM)
        if SA == 1:
            staging += MWG * KWG // threads
    if SB:
        loads += NWG * KWG // (threads * VWN)
        if SB == 1:
            staging += NWG * KWG // threads
    return acc, 2 * fragments + staging + 2 * loads + 24


def registers_fit(cfg):
    MDIMC, NDIMC, MFMA = cfg[3], cfg[4], cfg[11]
    acc, other = register_estimate(cfg)
    budget = register_budget(MDIMC * NDIMC * (cfg[15] if len(cfg) > 15 else 1))
    if not MFMA:
        budget = min(budget, 256)           # no accumulation registers without the matrix cores
    if acc + other > budget:
        return False
    # 16x16x4 tiles whose accumulators would take all 256 accumulation registers: the compiler
    # spills them (64 tiles of 4 registers each; measured on every such variant that was built)
    if MFMA == 2 and acc >= MAX_ACCUMULATION_REGISTERS:
        return False
    return True


def valid(cfg):
    MWG, NWG, KWG, MDIMC, NDIMC, VWM, VWN, SA, SB, PAD, KWI, MFMA, GRP = cfg[:13]
    SK = cfg[13] if len(cfg) > 13 else 1
    NS = cfg[14] if len(cfg) > 14 else 2
    KSW = cfg[15] if len(cfg) > 15 else 1
    if KSW not in (1, 2, 4) or (KSW > 1 and not MFMA):      # only the matrix-core schedule shares K out
        return False
    if not (tile_edge_ok(MWG) and tile_edge_ok(NWG)):
        return False
    if not (_pow2(KWG) and 2 <= KWG <= 128 and _pow2(MDIMC) and _pow2(NDIMC)
            and MDIMC <= 64 and NDIMC <= 64 and _pow2(KWI) and KWI <= 32):
        return False
    if VWM not in (1, 2, 4) or VWN not in (1, 2, 4) or MFMA not in (0, 1, 2):
        return False
    if any(f not in (0, 1) for f in (PAD, GRP)) or not 1 <= SK <= MAX_SPLIT_K:
        return False
    if SA not in (0, 1, 2) or SB not in (0, 1, 2) or NS not in (2, 3, 4):
        return False
    threads = MDIMC * NDIMC * KSW
    if (MDIMC * NDIMC) % 64 or threads > MAX_THREADS:   # whole wavefronts, device limit
        return False
    if MWG % MDIMC or NWG % NDIMC:                      # integer work per thread
        return False
    MWI, NWI = MWG // MDIMC, NWG // NDIMC
    if KWG % (KWI * KSW):                               # whole KWI blocks for every wave group
        return False
    if SA:
        if MWG % VWM or KWG % VWM or (MWG * KWG) % (threads * VWM):
            return False
    elif VWM != 1:                                      # width is meaningless without staging
        return False
    if SB:
        if NWG % VWN or KWG % VWN or (NWG * KWG) % (threads * VWN):
            return False
    if PAD and SA != 1 and SB != 1:                     # only register-staged tiles are padded
        return False
    if (SA == 2 and VWM == 2) or (SB == 2 and VWN == 2):   # LDS-direct loads: 4 or 16 bytes
        return False
    loads = 0                                           # LDS-direct loads per thread and slab
    if SA == 2:
        loads += MWG * KWG // (threads * VWM)
    if SB == 2:
        loads += NWG * KWG // (threads * VWN)
    if loads > MAX_LOADS_IN_FLIGHT:                     # one slab's loads must fit the counter
        return False
    if NS > 2:
        # deeper than double buffering: every staged tile must come by LDS-direct loads, and
        # the loads of the NS - 2 youngest slabs must fit the wave's counter as well
        if SA == 1 or SB == 1 or (SA != 2 and SB != 2):
            return False
        if (NS - 2) * loads > MAX_LOADS_IN_FLIGHT:
            return False
    if MFMA == 0:
        if NWI % VWN or MWI * NWI > 64:
            return False
    else:
        if MDIMC % 8 or NDIMC % 8:
            return False
        if not SB and VWN != 1:
            return False
        tile, depth = (32, 2) if MFMA == 1 else (16, 4)
        if (8 * MWI) % tile or (8 * NWI) % tile or KWI % depth or MWI * NWI > 256:
            return False
    if not registers_fit(cfg):
        return False
    if worst_lds_bytes(cfg) > LDS_LIMIT:
        return False
    return True


def enumerate_space(preset):
    out = []
    for cfg in itertools.product(*VALUES[preset]):
        if not valid(cfg):
            continue
        if preset == SPACE_SMALL and cfg[7] != cfg[8]:  # one LDS switch for both operands
            continue
        out.append(cfg)
    return out


def raw_size(preset):
    n = 1
    for v in VALUES[preset]:
        n *= len(v)
    return n
