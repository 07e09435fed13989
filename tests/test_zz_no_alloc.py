"""sgemm_tuned_noalloc(): the entry point for callers that cannot allocate device memory (its
split-K planes lie in the library's static device array).  Its output must equal that of
sgemm_tuned_on() - same variant, same launch plan, so bit for bit - and meet the oracle bound,
on two calls in a row, the second on a smaller problem that reuses the same scratch memory."""
import numpy as np
import pytest

from oracle import sgemm_oracle as orc
from paper_1703_06503_amd import binding as b
from paper_1703_06503_amd import synth
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu

from tests.variants import NOALLOC_CALLS as CALLS, NOALLOC_TOO_BIG  # noqa: E402


def _operands(call, seed):
    import torch
    M, N, K, layout, alpha, beta = call
    A, B, C = synth.make_inputs(M, N, K, layout, seed=seed)
    return (A, B, C), [torch.from_numpy(x).cuda() for x in (A, B, C)]


def test_noalloc_matches_the_allocating_entry_point_and_the_oracle():
    import os
    import torch
    b.sgemm_cache_clear()
    b.sgemm_cache_load(os.path.join(os.path.dirname(b.LIB_PATH), "..", "tuned_configs.txt"))
    host, dev, want = [], [], []
    for n, call in enumerate(CALLS):
        M, N, K, layout, alpha, beta = call
        h, d = _operands(call, seed=400 + n)
        host.append(h)
        dev.append(d)
        lda, ldb = h[0].shape[1], h[1].shape[1]
        cfg = b.sgemm_config_select(M, N, K, layout)
        nbytes, parts, _ = b.sgemm_config_workspace_bytes(cfg, M, N, K)
        assert (parts > 1) == (n < 2) and nbytes <= b.NOALLOC_SCRATCH_BYTES, (call, cfg)
        if n == 0:
            # not prepared yet: an error, nothing launched, C untouched
            dC = d[2].clone()
            with pytest.raises(b.SgemmError) as e:
                b.sgemm_tuned_noalloc(None, M, N, K, alpha, d[0], lda, d[1], ldb, beta, dC, N, layout)
            assert e.value.status == b.E_NOTREADY
            torch.cuda.synchronize()
            assert torch.equal(dC, d[2])
        # the existing entry point: prepares the call and gives the expected output
        dC = d[2].clone()
        b.sgemm_tuned_on(None, M, N, K, alpha, d[0], lda, d[1], ldb, beta, dC, N, layout)
        torch.cuda.synchronize()
        want.append(dC.cpu().numpy())
    # two (three) calls in a row through the entry point that allocates nothing, the later ones
    # on smaller problems; nothing is waited for between them
    got = []
    for call, h, d in zip(CALLS, host, dev):
        M, N, K, layout, alpha, beta = call
        dC = d[2].clone()
        b.sgemm_tuned_noalloc(None, M, N, K, alpha, d[0], h[0].shape[1], d[1], h[1].shape[1], beta, dC, N, layout)
        got.append(dC)
    torch.cuda.synchronize()
    for call, h, g, w in zip(CALLS, host, got, want):
        M, N, K, layout, alpha, beta = call
        g = g.cpu().numpy()
        assert np.array_equal(g, w), call
        r, c = synth.sample_positions(M, N, 7, rows=4, cols=4, scattered=2048, edge=min(64, M, N))
        ref = orc.sgemm_sample(alpha, h[0], h[1], beta, h[2], r, c, layout)
        tol = orc.tolerance(K, np.abs(h[0]).max(), np.abs(h[1]).max(), ref)
        assert np.all(np.abs(g[r, c] - ref) <= tol), call
    # and once more in the other order: the big problem after the small ones
    for call, h, d, w in reversed(list(zip(CALLS, host, dev, want))):
        M, N, K, layout, alpha, beta = call
        dC = d[2].clone()
        b.sgemm_tuned_noalloc(None, M, N, K, alpha, d[0], h[0].shape[1], d[1], h[1].shape[1], beta, dC, N, layout)
        torch.cuda.synchronize()
        assert np.array_equal(dC.cpu().numpy(), w), call


def test_noalloc_rejects_a_call_whose_planes_exceed_the_static_scratch():
    import torch
    (M, N, K, layout), cfg = NOALLOC_TOO_BIG
    nbytes, parts, _ = b.sgemm_config_workspace_bytes(cfg, M, N, K)
    assert parts == 4 and nbytes > b.NOALLOC_SCRATCH_BYTES
    A, B, C = synth.make_inputs(M, N, K, layout, seed=410)
    dA, dB, dC = (torch.from_numpy(x).cuda() for x in (A, B, C))
    b.sgemm_config_set(M, N, K, layout, cfg)
    try:
        b.sgemm_tuned_on(None, M, N, K, 1.0, dA, M, dB, K, 0.0, dC, N, layout)     # prepares it
        torch.cuda.synchronize()
        want = dC.clone()
        dC.fill_(7.0)
        with pytest.raises(b.SgemmError) as e:
            b.sgemm_tuned_noalloc(None, M, N, K, 1.0, dA, M, dB, K, 0.0, dC, N, layout)
        assert e.value.status == b.E_RESOURCE and "scratch" in str(e.value)
        torch.cuda.synchronize()
        assert bool((dC == 7.0).all())
        r, c = synth.sample_positions(M, N, 8, rows=2, cols=2, scattered=512)
        ref = orc.sgemm_sample(1.0, A, B, 0.0, C, r, c, layout)
        tol = orc.tolerance(K, np.abs(A).max(), np.abs(B).max(), ref)
        assert np.all(np.abs(want.cpu().numpy()[r, c] - ref) <= tol)
    finally:
        b.sgemm_cache_clear()
        import os
        b.sgemm_cache_load(os.path.join(os.path.dirname(b.LIB_PATH), "..", "tuned_configs.txt"))
