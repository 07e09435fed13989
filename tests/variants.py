"""Which kernel variants the GPU tests launch: the fixed samples of the search spaces, the
shapes they run on and the hand-picked configurations.  The tests take their cases from here and
tests/precompile_test_variants.py compiles exactly these ahead of time, so that a GPU run
compiles nothing.  No arithmetic of the method and nothing of the oracle lives here."""
import numpy as np

from paper_1703_06503_amd import binding as b


def sample_configs(space, count, seed):
    """A fixed pseudo-random sample of configuration indices of a space (sorted)."""
    n = b.sgemm_space_size(space)
    rng = np.random.default_rng(seed)
    return sorted(int(i) for i in rng.choice(n, size=min(count, n), replace=False))


FULL_SAMPLE = dict(space=b.SPACE_FULL, count=160, seed=1234)
MFMA_SAMPLE = dict(space=b.SPACE_MFMA, count=80, seed=4321)
EXT_SAMPLE = dict(space=b.SPACE_EXT, count=80, seed=777)   # tile edges 96/192, split K
DIRECT_SAMPLE = dict(space=b.SPACE_DIRECT, count=80, seed=555)   # LDS-direct staging, 2-4 buffers
KSPLIT_SAMPLE = dict(space=b.SPACE_KSPLIT, count=64, seed=999)   # wave groups share out the K slab
EXACT_EXT = (768, 768, 1024)      # multiples of 96, 192 and 256; 16..64 slabs to split
RAGGED_EXT = (300, 520, 1000)
EXACT_SHAPE = (256, 512, 96)      # multiples of every tile size: unguarded variants
RAGGED_SHAPE = (200, 136, 68)     # guarded variants, several tiles for small configs
NARROW_SHAPE = (202, 138, 66)     # even, not multiples of 4
RAGGED_BIG = (300, 520, 44)       # more than one tile even at 256 x 256
ODD_SHAPE = (203, 137, 67)        # stored rows end inside a 16-byte vector


def all_sweeps():
    """(space, configuration indices, shape, layout) of every sweep of tests/test_gpu_parity.py."""
    full, mfma = sample_configs(**FULL_SAMPLE), sample_configs(**MFMA_SAMPLE)
    ext, direct = sample_configs(**EXT_SAMPLE), sample_configs(**DIRECT_SAMPLE)
    out = [(b.SPACE_SMALL, list(range(16)), (256, 256, 256), 0),
           (b.SPACE_FULL, full, EXACT_SHAPE, 0), (b.SPACE_FULL, full, RAGGED_SHAPE, 0),
           (b.SPACE_MFMA, mfma, EXACT_SHAPE, 0), (b.SPACE_MFMA, mfma, RAGGED_BIG, 0),
           (b.SPACE_EXT, ext, EXACT_EXT, 0), (b.SPACE_EXT, ext, RAGGED_EXT, 0),
           (b.SPACE_DIRECT, direct, EXACT_EXT, 0), (b.SPACE_DIRECT, direct, RAGGED_EXT, 0),
           (b.SPACE_DIRECT, direct[::4], ODD_SHAPE, 0)]
    ksplit = sample_configs(**KSPLIT_SAMPLE)
    out += [(b.SPACE_KSPLIT, ksplit, EXACT_EXT, 0), (b.SPACE_KSPLIT, ksplit, RAGGED_EXT, 0),
            (b.SPACE_KSPLIT, ksplit[::4], ODD_SHAPE, 0)]
    for layout in (1, 2, 3):
        k = sample_configs(b.SPACE_KSPLIT, 16, seed=400 + layout)
        out += [(b.SPACE_KSPLIT, k, EXACT_EXT, layout), (b.SPACE_KSPLIT, k, RAGGED_EXT, layout)]
        d = sample_configs(b.SPACE_DIRECT, 24, seed=300 + layout)
        out += [(b.SPACE_DIRECT, d, EXACT_EXT, layout), (b.SPACE_DIRECT, d, RAGGED_EXT, layout),
                (b.SPACE_EXT, sample_configs(b.SPACE_EXT, 24, seed=200 + layout), RAGGED_EXT, layout)]
        f = sample_configs(b.SPACE_FULL, 40, seed=100 + layout)
        out += [(b.SPACE_FULL, f, EXACT_SHAPE, layout), (b.SPACE_FULL, f, RAGGED_SHAPE, layout)]
    return out


def some_configs():
    """A vector-ALU variant, a 32x32x2 MFMA variant, a 16x16x4 MFMA variant, and three
    split-K variants (vector ALU, MFMA with a 96-wide tile, MFMA split 16 ways), and three
    variants fed by LDS-direct loads (three LDS buffers; four buffers with split K; vector ALU
    with A direct and B through registers), and three whose waves share out the K slab (four
    groups of 32x32 wave tiles; two groups of 16x16x4 tiles with split K on top; four groups fed
    by LDS-direct loads)."""
    return [
        b.make_config(64, 64, 16, 8, 8, 4, 4, 1, 1, 1, 8, 0, 0),
        b.make_config(128, 128, 16, 16, 16, 4, 4, 1, 1, 1, 8, 1, 1),
        b.make_config(64, 64, 16, 16, 16, 2, 2, 1, 1, 0, 8, 2, 1),
        b.make_config(64, 64, 16, 8, 8, 4, 4, 1, 1, 1, 8, 0, 0, 3),
        b.make_config(96, 64, 16, 8, 16, 4, 4, 1, 1, 1, 8, 1, 1, 4),
        b.make_config(32, 32, 8, 8, 8, 1, 1, 1, 1, 0, 2, 1, 0, 16),
        b.make_config(128, 128, 16, 16, 16, 4, 4, 2, 2, 0, 8, 1, 1, 1, 3),
        b.make_config(64, 64, 32, 8, 8, 4, 4, 2, 2, 0, 8, 2, 0, 2, 4),
        b.make_config(64, 64, 16, 8, 8, 4, 4, 2, 1, 1, 8, 0, 0, 1, 2),
        b.make_config(64, 64, 64, 16, 16, 4, 4, 1, 1, 1, 8, 1, 1, 1, 2, 4),
        b.make_config(32, 64, 64, 8, 16, 4, 4, 1, 1, 0, 8, 2, 0, 2, 2, 2),
        b.make_config(64, 32, 32, 8, 8, 4, 4, 2, 2, 0, 2, 1, 1, 1, 2, 4),
    ]


# configurations run at the full benchmark sizes beside the tuned winners
BENCH_CONFIGS = [
    b.make_config(256, 256, 32, 32, 16, 4, 4, 1, 1, 1, 8, 1, 1),
    b.make_config(256, 256, 32, 16, 16, 4, 4, 2, 2, 0, 8, 1, 1, 1, 2),
    b.make_config(128, 128, 16, 16, 16, 4, 4, 1, 1, 1, 8, 1, 1),
    b.make_config(64, 64, 16, 8, 8, 4, 4, 1, 1, 1, 8, 0, 1),
]
SKINNY_CONFIGS = [b.make_config(64, 64, 16, 16, 16, 4, 4, 1, 1, 1, 8, 1, 0),
                  b.make_config(64, 64, 32, 16, 16, 4, 4, 1, 1, 1, 8, 1, 0, 8)]

# tile edges of 5 and 7 times a power of two (the built-in templates for sizes like 2560 and 3584 use
# them): the two templates, a mixed tile with wave groups and split K, and one with unpadded LDS rows
ODD_EDGE_CONFIGS = [b.make_config(160, 160, 32, 16, 16, 4, 4, 1, 1, 1, 8, 2, 1),
                    b.make_config(224, 224, 32, 16, 16, 4, 4, 1, 1, 1, 8, 2, 1),
                    b.make_config(80, 112, 64, 8, 8, 4, 4, 1, 1, 1, 8, 2, 0, 2, 2, 4),
                    b.make_config(112, 80, 64, 8, 8, 4, 4, 1, 1, 0, 8, 2, 1, 1, 2, 2)]
ODD_EDGE_SHAPES = [(1120, 1120, 128), (333, 500, 200)]     # a multiple of every such tile, and a ragged one

# (M, N, K, layout) of calls that go through the dispatch without an exactly tuned shape
DISPATCHED_CALLS = ([(250, 250, 128, 0), (4091, 4091, 4091, 0), (300, 200, 150, 0), (2560, 2560, 1536, 0), (3584, 3584, 1024, 3), (300000, 24, 40, 0)]
                    + [(M, N, K, layout) for layout in (2, 3)
                       for (M, N, K) in [(300, 200, 150), (96, 1000, 4100), (1536, 1536, 64)]])

# tests of the entry point that allocates nothing: (M, N, K, layout, alpha, beta).  The first is
# benchmark configuration 5's first shape (tuned with split K 8: 16 MiB of planes), the second a
# smaller long-K shape that the built-in default splits as well, the third does not split K.
NOALLOC_CALLS = [(128, 4096, 4096, 1, 1.0, 0.0), (96, 1000, 4100, 2, 1.25, 0.5), (300, 200, 150, 0, 1.0, 1.0)]
NOALLOC_TOO_BIG = ((2048, 2048, 4096, 3), b.make_config(128, 128, 32, 16, 16, 4, 4, 1, 1, 1, 8, 1, 1, 4))

# ---- 2D convolution -------------------------------------------------------------------------
CONV_SAMPLES = {(3, 3): (24, 1), (7, 7): (40, 2), (11, 11): (24, 3), (5, 3): (16, 4), (4, 2): (12, 5)}
CONV_CONFIGS = [(32, 8, 1, 8, 0, 1, 0, 1), (32, 16, 2, 4, 2, 2, 1, 1), (32, 8, 2, 4, 1, 2, 0, 1),
                (16, 16, 4, 2, 2, 4, 0, 0), (64, 8, 8, 1, 2, 8, 0, 1), (8, 8, 1, 1, 1, 1, 1, 0),
                (64, 16, 4, 4, 1, 4, 1, 0), (8, 64, 8, 8, 0, 8, 0, 1)]
CONV_DEFAULT_FILTERS = [(3, 3), (5, 5), (7, 7), (11, 11), (1, 1), (2, 5), (9, 9), (11, 3), (13, 13), (31, 5), (17, 17)]


def conv_sample(Xf, Yf):
    count, seed = CONV_SAMPLES[(Xf, Yf)]
    n = b.conv2d_space_size(Xf, Yf)
    rng = np.random.default_rng(seed)
    return sorted(int(i) for i in rng.choice(n, size=count, replace=False))
