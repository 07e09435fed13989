"""The hit path of sgemm_tuned_on(): what a call costs on the host once its shape has been seen,
measured from C (tests/native/dispatch_overhead.hip) beside a plain HIP launch of an empty kernel."""
import json
import os
import subprocess

import pytest

from tests.native import build as native

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("shape", [(256, 256, 256, 0), (128, 4096, 4096, 1)])
def test_a_dispatch_hit_costs_little_more_than_the_launch_itself(shape):
    """One hash lookup on integers under one lock, then the launch (two launches when K is
    split): within 3 microseconds of HIP's own launch cost per kernel launched."""
    exe = native.DISPATCH_OVERHEAD
    if not os.path.exists(exe):
        native.build()
    out = subprocess.run([exe, *map(str, shape), "4096"], check=True, capture_output=True, text=True, timeout=120)
    r = json.loads(out.stdout.strip().splitlines()[-1])
    print(r)
    launches = 2 if shape[3] == 1 else 1        # the skinny shape is tuned with split K
    assert r["sgemm_tuned_on_us"] <= launches * r["empty_launch_us"] + 3.0, r
