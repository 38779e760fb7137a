"""GPU parity: exception layers (Sec. 4.1 "Handling Exception Layers") keep their FP16 weights
and run the FP16 GEMM in both modes; applicable layers follow the requested mode."""
import numpy as np
import pytest
import torch

import oracle
from paper_2506_02024_amd import workloads
from helpers import assert_gemm_close, bits, to_dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def nfp():
    from paper_2506_02024_amd import binding

    return binding


@pytest.mark.parametrize("packed", [False, True], ids=["rowmajor", "packed"])
@pytest.mark.parametrize("M", [8, 200])
def test_planted_outlier_makes_an_exception_layer(nfp, M, packed):
    N, K = 272, 1040
    W = workloads.weight_host(N, K, seed=5)
    W_bad = W.copy()
    W_bad[137, 555] = np.float16(2.5)                  # one weight past the 1.75 bound
    W_bad[3, 0] = np.float16(-1.8125)
    X = workloads.act_host(M, K, seed=6)
    Xd = to_dev(X)
    good, bad = nfp.Layer(to_dev(W), packed=packed), nfp.Layer(to_dev(W_bad), packed=packed)
    assert not good.is_exception and good.out_of_range == 0
    assert bad.is_exception and bad.out_of_range == 2 and bad.upper is None

    ref_bad = oracle.gemm_fp16(X, W_bad)
    plain = bits(nfp.plain_gemm_fp16(Xd, to_dev(W_bad)))
    for mode in (nfp.MODE_FP16, nfp.MODE_FP8):
        y = nfp.linear(Xd, bad, mode)
        assert_gemm_close(y.cpu().numpy(), ref_bad, "exception layer, mode %d" % mode)
        assert np.array_equal(bits(y), plain)          # the FP16 kernel, whatever the mode

    # the applicable layer follows the mode: identical to nestedfp_gemm on its planes
    for mode in (nfp.MODE_FP16, nfp.MODE_FP8):
        y = nfp.linear(Xd, good, mode)
        z = nfp.gemm(Xd, good.upper, None if mode == nfp.MODE_FP8 else good.lower, mode)
        assert np.array_equal(bits(y), bits(z))
    up, _, _ = oracle.decompose(W)
    Xq, sc = oracle.quantize_act(X)
    assert_gemm_close(nfp.linear(Xd, good, nfp.MODE_FP8).cpu().numpy(), oracle.gemm_fp8(Xq, sc, up), "FP8 mode")


def test_mixed_stack_switches_only_the_applicable_layers(nfp):
    # a small "model": four linears, one of them an exception; per-step mode switching
    K = 512
    Ws = [workloads.weight_host(256, K, seed=20 + i) for i in range(4)]
    Ws[2][10, 10] = np.float16(3.0)
    layers = [nfp.Layer(to_dev(w), packed=(i % 2 == 1)) for i, w in enumerate(Ws)]
    assert [l.is_exception for l in layers] == [False, False, True, False]
    X = workloads.act_host(16, K, seed=9)
    Xd = to_dev(X)
    out16 = [bits(nfp.linear(Xd, l, nfp.MODE_FP16)) for l in layers]
    out8 = [bits(nfp.linear(Xd, l, nfp.MODE_FP8)) for l in layers]
    assert np.array_equal(out16[2], out8[2])           # exception layer: same result in both modes
    for i in (0, 1, 3):
        assert not np.array_equal(out16[i], out8[i])   # the others really change precision
        assert_gemm_close(out16[i].view(np.float16), oracle.gemm_fp16(X, Ws[i]), "layer %d" % i)
