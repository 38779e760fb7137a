"""GPU parity: per-token E4M3 activation quantisation is bit-exact against the oracle."""
import numpy as np
import pytest
import torch

import oracle
from paper_2506_02024_amd import workloads
from helpers import to_dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def nfp():
    from paper_2506_02024_amd import binding

    return binding


@pytest.mark.parametrize("hw", [1, 0])
@pytest.mark.parametrize("M,K", [(16, 1024), (1, 16), (7, 4112), (64, 14336), (3, 20480), (300, 512),
                                 (2, 32768), (2, 32784)])
def test_gaussian_rows(nfp, hw, M, K):
    X = workloads.act_host(M, K, seed=M)
    if M > 2:
        X[1] = 0                                   # all-zero row: scale 1, codes 0
        X[2, 3] = np.float16(65504.0)              # largest finite half as row maximum
    nfp.tune("quant_hw", hw)
    try:
        Xq, s = nfp.quantize_act(to_dev(X))
        Xq, s = Xq.cpu().numpy(), s.cpu().numpy()
    finally:
        nfp.tune("quant_hw", -1)
    Xq_ref, s_ref = oracle.quantize_act(X)
    assert np.array_equal(s, s_ref)
    assert np.array_equal(Xq, Xq_ref)


@pytest.mark.parametrize("M,K", [(300, 8208), (520, 14336), (260, 4096), (3, 32768), (270, 32784)])
def test_single_pass_and_two_pass_kernels_agree_with_the_oracle(nfp, M, K):
    # rows kept in registers between the maximum and the conversion (decode-sized batches and long
    # rows) or read twice (the rest; rows beyond 32768 columns always): forced either way
    X = workloads.act_host(M, K, seed=K)
    X[1] = 0
    X[2, K - 1] = np.float16(-65504.0)
    Xq_ref, s_ref = oracle.quantize_act(X)
    for onepass in (1, 0, -1):
        nfp.tune("quant_onepass", onepass)
        try:
            Xq, s = nfp.quantize_act(to_dev(X))
        finally:
            nfp.tune("quant_onepass", -1)
        assert np.array_equal(s.cpu().numpy(), s_ref), onepass
        assert np.array_equal(Xq.cpu().numpy(), Xq_ref), onepass


@pytest.mark.parametrize("hw", [1, 0])
def test_every_finite_half_under_several_row_scales(nfp, hw):
    # each row holds every finite FP16 word whose magnitude does not exceed the row's maximum;
    # row maxima chosen to hit ties, E4M3 subnormals and saturation at the top
    words = workloads.all_fp16_words()
    vals = words.view(np.float16)
    finite = np.isfinite(vals.astype(np.float32))
    rows = []
    for amax in (65504.0, 448.0, 1.0, 0.3337, 7.0, 2.0 ** -10, 6.1e-5, 240.0):
        a16 = np.float16(amax)
        keep = finite & (np.abs(vals.astype(np.float32)) <= np.float32(a16))
        row = np.full(65536, a16, dtype=np.float16)
        row[: keep.sum()] = vals[keep]
        rows.append(row)
    X = np.stack(rows)
    nfp.tune("quant_hw", hw)
    try:
        Xq, s = nfp.quantize_act(to_dev(X))
        Xq, s = Xq.cpu().numpy(), s.cpu().numpy()
    finally:
        nfp.tune("quant_hw", -1)
    Xq_ref, s_ref = oracle.quantize_act(X)
    assert np.array_equal(s, s_ref)
    mism = np.nonzero(Xq != Xq_ref)
    assert mism[0].size == 0, "first mismatch row %d col %d: x=%r got %#x want %#x" % (
        mism[0][0], mism[1][0], X[mism[0][0], mism[1][0]], Xq[mism[0][0], mism[1][0]],
        Xq_ref[mism[0][0], mism[1][0]])


def test_static_per_tensor_scale(nfp):
    X = workloads.act_host(5, 256, seed=3)
    sc = torch.tensor([0.0625], dtype=torch.float32, device="cuda:0")
    Xq, s = nfp.quantize_act(to_dev(X), static_scale=sc)
    Xq_ref, s_ref = oracle.quantize_act(X, static_scale=0.0625)
    assert np.array_equal(s.cpu().numpy(), s_ref)
    assert np.array_equal(Xq.cpu().numpy(), Xq_ref)


def test_quotient_is_the_correctly_rounded_division_for_every_half_and_many_scales(nfp):
    # The kernels divide by multiplying with the row's reciprocal and one FMA correction.
    # Every finite FP16 word against a few hundred scales (random over the binary32 range the
    # method can produce, all-ones and power-of-two significands, amax/448 of odd maxima):
    # the codes must equal the oracle's, which performs the binary32 division itself.
    words = workloads.all_fp16_words()
    vals = words.view(np.float16)
    finite = vals[np.isfinite(vals.astype(np.float32))]
    X = np.zeros((32, 2048), dtype=np.float16)
    X.reshape(-1)[: finite.size] = finite
    rng = np.random.default_rng(11)
    scales = list(np.exp(rng.uniform(np.log(1e-7), np.log(300.0), 160)).astype(np.float32))
    scales += [np.float32(1.0), np.float32(2.0 ** -20), np.float32(146.2143), np.float32(0.99999994),
               np.float32(1.9999999), np.float32(3.0), np.float32(1.0 / 3.0), np.float32(65504.0 / 448.0)]
    scales += [np.float32(np.float16(a)) / np.float32(448.0) for a in (0.3337, 7.0, 1.0, 33.0, 6.1e-5, 5.96e-8)]
    scales += [np.frombuffer(np.uint32(b).tobytes(), dtype=np.float32)[0]
               for b in (0x3f7fffff, 0x3fffffff, 0x3effffff, 0x40ffffff, 0x3c7fffff, 0x3f800001, 0x3fc00001)]
    Xd = to_dev(X)
    for sc in scales:
        sd = torch.tensor([float(sc)], dtype=torch.float32, device="cuda:0")
        Xq, _ = nfp.quantize_act(Xd, static_scale=sd)
        Xq_ref, _ = oracle.quantize_act(X, static_scale=float(sc))
        got = Xq.cpu().numpy()
        mism = np.nonzero(got != Xq_ref)
        assert mism[0].size == 0, "scale %r: x=%r got %#x want %#x" % (
            sc, X[mism[0][0], mism[1][0]], got[mism[0][0], mism[1][0]], Xq_ref[mism[0][0], mism[1][0]])

