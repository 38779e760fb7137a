"""GPU: the GEMM entry point that takes no workspace and allocates nothing (for callers that
cannot call hipMalloc: code under graph capture without scratch of its own, tight serving loops)
gives what nestedfp_gemm gives, bit for bit, on consecutive calls that share its fixed scratch."""
import numpy as np
import pytest
import torch

from paper_2506_02024_amd import workloads
from helpers import bits, to_dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def nfp():
    from paper_2506_02024_amd import binding

    return binding


def _both(nfp, M, N, K, seed):
    W = to_dev(workloads.weight_host(N, K, seed=seed))
    X = to_dev(workloads.act_host(M, K, seed=seed + 1))
    up, lo = nfp.decompose(W)
    want = {mode: nfp.gemm(X, up, None if mode == nfp.MODE_FP8 else lo, mode) for mode in (nfp.MODE_FP16, nfp.MODE_FP8)}
    out = {mode: torch.zeros((M, N), dtype=torch.float16, device="cuda:0") for mode in want}
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    for mode in want:
        nfp.gemm_static(X, up, None if mode == nfp.MODE_FP8 else lo, mode, out[mode])
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    for mode in want:
        assert np.array_equal(bits(out[mode]), bits(want[mode])), (M, N, K, mode)


def test_two_calls_in_a_row_share_the_fixed_scratch(nfp):
    # a grid-level K split (arrival counters and partial sums in the scratch) and quantised
    # activations, then a smaller problem that finds the first call's leftovers there, then a
    # prefill-sized one on the tiled kernels, then the first again
    _both(nfp, 16, 4096 + 8, 14336, seed=3)
    _both(nfp, 4, 304, 2048 + 64, seed=5)
    _both(nfp, 300, 520, 1040, seed=7)
    _both(nfp, 16, 4096 + 8, 14336, seed=3)


def test_problems_beyond_the_fixed_scratch_are_refused(nfp):
    M, N, K = 16384, 1024, 4096                        # 64 MiB of quantised activations
    assert nfp.gemm_workspace_size(M, N, K, nfp.MODE_FP8) > nfp.STATIC_SCRATCH_BYTES
    W = to_dev(workloads.weight_host(N, K, seed=1))
    up, lo = nfp.decompose(W)
    X = torch.zeros((M, K), dtype=torch.float16, device="cuda:0")
    out = torch.zeros((M, N), dtype=torch.float16, device="cuda:0")
    with pytest.raises(nfp.NestedFPError) as e:
        nfp.gemm_static(X, up, None, nfp.MODE_FP8, out)
    assert e.value.status == nfp.ERR_WORKSPACE
    assert int(out.count_nonzero()) == 0
