"""The blocked CPU SGEMM that bench.py reports as a baseline is itself held to the oracle."""
import numpy as np
import pytest

from oracle import cpu_blocked
from oracle import sgemm_oracle as orc
from paper_1703_06503_amd import synth


@pytest.mark.parametrize("layout", [0, 1, 2, 3])
def test_blocked_cpu_sgemm_matches_oracle(layout):
    for (M, N, K), (alpha, beta) in [((130, 1100, 300), (1.5, -0.5)), ((65, 70, 513), (1.0, 0.0)),
                                     ((1, 1, 1), (2.0, 1.0))]:
        A, B, C = synth.make_inputs(M, N, K, layout, seed=70 + layout)
        got = cpu_blocked.sgemm(alpha, A, B, beta, C, layout)
        ref = orc.sgemm(alpha, A, B, beta, C, layout)
        tol = orc.tolerance(K, np.abs(A).max(), np.abs(B).max(), ref)
        assert np.all(np.abs(got - ref) <= tol)


def test_blocked_cpu_sgemm_edge_cases():
    A, B, C = synth.make_inputs(40, 50, 60, 0, seed=75, dist="smallint")
    assert np.array_equal(cpu_blocked.sgemm(2.0, A, B, -3.0, C), orc.sgemm(2.0, A, B, -3.0, C))
    Cn = C.copy(); Cn[0, 0] = np.nan
    assert np.all(np.isfinite(cpu_blocked.sgemm(1.0, A, B, 0.0, Cn)))
    assert np.array_equal(cpu_blocked.sgemm(0.0, A, B, 1.0, C), C)
