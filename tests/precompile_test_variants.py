"""Put every kernel variant that tests/test_gpu_parity.py launches into the on-disk kernel
cache, in parallel and without a GPU, so that the GPU run spends no time compiling:

    python tests/precompile_test_variants.py

(The tests pass without this step; they then compile each variant on first use.)"""
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))

from paper_1703_06503_amd import binding as b            # noqa: E402
from paper_1703_06503_amd.precompile import precompile   # noqa: E402
from tests import gpu_util as gu                         # noqa: E402
from tests import test_gpu_parity as t                   # noqa: E402


def main():
    jobs = min(8, os.cpu_count() or 1)
    precompile(b.SPACE_SMALL, (0,), (0,), jobs)
    full = gu.sample_configs(**t.FULL_SAMPLE)
    precompile(b.SPACE_FULL, (0,), (0, 1), jobs, indices=full)
    mfma = gu.sample_configs(**t.MFMA_SAMPLE)
    precompile(b.SPACE_MFMA, (0,), (0, 1), jobs, indices=mfma)
    precompile(b.SPACE_EXT, (0,), (0, 1), jobs, indices=gu.sample_configs(**t.EXT_SAMPLE))
    precompile(b.SPACE_DIRECT, (0,), (0, 1), jobs, indices=gu.sample_configs(**t.DIRECT_SAMPLE))
    for layout in (1, 2, 3):
        precompile(b.SPACE_FULL, (layout,), (0, 1), jobs,
                   indices=gu.sample_configs(b.SPACE_FULL, 40, seed=100 + layout))
        precompile(b.SPACE_EXT, (layout,), (1,), jobs,
                   indices=gu.sample_configs(b.SPACE_EXT, 24, seed=200 + layout))
        precompile(b.SPACE_DIRECT, (layout,), (0, 1), jobs,
                   indices=gu.sample_configs(b.SPACE_DIRECT, 24, seed=300 + layout))


if __name__ == "__main__":
    main()
