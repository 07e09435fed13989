"""Oracle for the tuner's search space.  TEST INFRASTRUCTURE ONLY; shares no code with the
library.

The paper builds its space as the cartesian product of short per-parameter value lists,
pruned by user constraints and by device limits (sections "Advanced usage" and "Search
strategies and search-space properties").  This file writes out, in plain Python, the value
lists of this build's three presets and every constraint of its GEMM kernel family, and
enumerates the product in lexicographic order (first parameter slowest).

Parameters, in order: MWG NWG KWG MDIMC NDIMC VWM VWN SA SB PAD KWI MFMA GRP SK.

parity unpinned: the paper's own count of 241 600 valid GEMM configurations cannot be
reproduced, because its constraint list is not printed; the counts here are pinned only by
the independent re-derivation below and by brute-force checks in the tests.
"""
import itertools

NAMES = ("MWG", "NWG", "KWG", "MDIMC", "NDIMC", "VWM", "VWN", "SA", "SB", "PAD", "KWI", "MFMA",
         "GRP", "SK")

SPACE_FULL, SPACE_SMALL, SPACE_MFMA, SPACE_EXT = 0, 1, 2, 3

VALUES = {
    SPACE_FULL: ([32, 64, 128, 256], [32, 64, 128, 256], [8, 16, 32], [8, 16], [8, 16], [1, 4],
                 [1, 4], [0, 1], [0, 1], [0, 1], [2, 8], [0, 1], [0, 1], [1]),
    SPACE_SMALL: ([32, 64], [32, 64], [8, 16], [8], [8], [1], [1], [0, 1], [0, 1], [0], [2], [0],
                  [0], [1]),
    SPACE_MFMA: ([64, 128, 256], [64, 128, 256], [8, 16, 32], [8, 16, 32], [8, 16, 32],
                 [1, 2, 4], [1, 2, 4], [1], [1], [0, 1], [2, 8], [1, 2], [0, 1], [1]),
    SPACE_EXT: ([32, 64, 96, 128, 192, 256], [32, 64, 96, 128, 192, 256], [16, 32, 64],
                [8, 16, 32], [8, 16, 32], [1, 2, 4], [1, 2, 4], [1], [1], [0, 1], [2, 8], [1, 2],
                [0, 1], [1, 2, 3, 4, 6, 8, 12, 16]),
}

LDS_LIMIT = 160 * 1024          # bytes per workgroup on gfx950
MAX_THREADS = 1024
MAX_SPLIT_K = 64


def _pow2(v):
    return v > 0 and v & (v - 1) == 0


def tile_edge_ok(v):
    """A tile edge is 2^a or 3 * 2^a, between 8 and 512."""
    return 8 <= v <= 512 and (_pow2(v) or (v % 3 == 0 and _pow2(v // 3)))


def lds_bytes(cfg, layout):
    """Two buffers of each staged tile; a tile keeps the stored orientation of its matrix, and
    PAD adds 4 floats to every tile row."""
    MWG, NWG, KWG, _, _, _, _, SA, SB, PAD = cfg[:10]
    pad = 4 if PAD else 0
    floats = 0
    if SA:
        floats += KWG * (MWG + pad) if layout & 1 else MWG * (KWG + pad)
    if SB:
        floats += NWG * (KWG + pad) if layout & 2 else KWG * (NWG + pad)
    return 2 * 4 * floats


def worst_lds_bytes(cfg):
    return max(lds_bytes(cfg, layout) for layout in range(4))


def register_estimate(cfg):
    MWG, NWG, KWG, MDIMC, NDIMC, _, _, SA, SB, _, KWI, MFMA = cfg[:12]
    threads = MDIMC * NDIMC
    MWI, NWI = MWG // MDIMC, NWG // NDIMC
    regs = MWI * NWI + 24                       # accumulators + addressing
    if MFMA:
        tile, depth = (32, 2) if MFMA == 1 else (16, 4)
        regs += (8 * MWI // tile + 8 * NWI // tile) * (KWI // depth)   # one fragment block
    else:
        regs += MWI + NWI
    if SA:
        regs += MWG * KWG // threads            # global -> LDS staging registers
    if SB:
        regs += NWG * KWG // threads
    return regs


def valid(cfg):
    MWG, NWG, KWG, MDIMC, NDIMC, VWM, VWN, SA, SB, PAD, KWI, MFMA, GRP = cfg[:13]
    SK = cfg[13] if len(cfg) > 13 else 1
    if not (tile_edge_ok(MWG) and tile_edge_ok(NWG)):
        return False
    if not (_pow2(KWG) and 2 <= KWG <= 128 and _pow2(MDIMC) and _pow2(NDIMC)
            and MDIMC <= 64 and NDIMC <= 64 and _pow2(KWI) and KWI <= 32):
        return False
    if VWM not in (1, 2, 4) or VWN not in (1, 2, 4) or MFMA not in (0, 1, 2):
        return False
    if any(f not in (0, 1) for f in (SA, SB, PAD, GRP)) or not 1 <= SK <= MAX_SPLIT_K:
        return False
    threads = MDIMC * NDIMC
    if threads % 64 or threads > MAX_THREADS:           # whole wavefronts, device limit
        return False
    if MWG % MDIMC or NWG % NDIMC:                      # integer work per thread
        return False
    MWI, NWI = MWG // MDIMC, NWG // NDIMC
    if KWG % KWI:
        return False
    if SA:
        if MWG % VWM or KWG % VWM or (MWG * KWG) % (threads * VWM):
            return False
    elif VWM != 1:                                      # width is meaningless without staging
        return False
    if SB:
        if NWG % VWN or KWG % VWN or (NWG * KWG) % (threads * VWN):
            return False
    if PAD and not (SA or SB):
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
    if register_estimate(cfg) > (512 if MFMA else 256):
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
