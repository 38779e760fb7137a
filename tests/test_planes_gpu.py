"""GPU parity: range check, decompose and reconstruct are bit-exact against the oracle."""
import numpy as np
import pytest
import torch

import oracle
from paper_2506_02024_amd import workloads
from helpers import assert_plane_equal, bits, to_dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def nfp():
    from paper_2506_02024_amd import binding

    return binding


@pytest.fixture(params=[False, True], ids=["rowmajor", "packed"])
def packed(request):
    return request.param


def test_exhaustive_fp16_words(nfp, packed):
    # all 65,536 FP16 words as a [256,256] "layer": planes, count and round trip
    W = workloads.all_fp16_words().reshape(256, 256)
    up_ref, lo_ref, bad_ref = oracle.decompose(W)
    assert bad_ref == 33278
    Wd = to_dev(W.view(np.float16))
    up, lo, bad = nfp.decompose_count(Wd, packed=packed)
    assert bad == bad_ref
    assert nfp.range_check(Wd) == bad_ref
    assert_plane_equal(up, up_ref)
    assert_plane_equal(lo, lo_ref)
    with pytest.raises(nfp.NestedFPError) as e:
        nfp.decompose(Wd, packed=packed)
    assert e.value.status == nfp.ERR_RANGE
    # lossless on every in-range word (Sec. 4.1)
    ok = np.array([oracle.in_range(int(w)) for w in W.reshape(-1)]).reshape(256, 256)
    back = bits(nfp.reconstruct(up, lo))
    assert np.array_equal(back[ok], W[ok])
    assert np.array_equal(back[ok], oracle.reconstruct(up_ref, lo_ref)[ok])


def test_in_range_words_only_pass_the_check(nfp, packed):
    words = workloads.all_fp16_words()
    ok = np.array([oracle.in_range(int(w)) for w in words])
    good = words[ok]
    good = np.resize(good, (2017 * 16,)).reshape(2017, 16)        # ragged row count, K = 16
    Wd = to_dev(good.view(np.float16))
    assert nfp.range_check(Wd) == 0
    up, lo = nfp.decompose(Wd, packed=packed)
    up_ref, lo_ref, bad = oracle.decompose(good)
    assert bad == 0
    assert_plane_equal(up, up_ref)
    assert_plane_equal(lo, lo_ref)
    assert np.array_equal(bits(nfp.reconstruct(up, lo)), good)


@pytest.mark.parametrize("N,K", [(1024, 1024), (1, 16), (3, 48), (777, 4112), (4096, 4096)])
def test_gaussian_layers(nfp, N, K, packed):
    W = workloads.weight_host(N, K, seed=N + K)
    Wd = to_dev(W)
    up, lo = nfp.decompose(Wd, packed=packed)
    up_ref, lo_ref, bad = oracle.decompose(W)
    assert bad == 0
    assert_plane_equal(up, up_ref)
    assert_plane_equal(lo, lo_ref)
    back = nfp.reconstruct(up, lo)
    assert np.array_equal(bits(back), W.view(np.uint16))


def test_strided_weight_rows(nfp, packed):
    N, K, ld = 65, 160, 200
    big = workloads.weight_host(N, ld, seed=5)
    Wd = to_dev(big)[:, :K]
    assert Wd.stride(0) == ld
    up, lo = nfp.decompose(Wd, packed=packed)
    up_ref, lo_ref, _ = oracle.decompose(big[:, :K])
    assert_plane_equal(up, up_ref)
    assert_plane_equal(lo, lo_ref)
    out = torch.full((N, ld), -1.0, dtype=torch.float16, device="cuda:0")
    nfp.reconstruct(up, lo, out=out[:, :K])
    got = bits(out)
    assert np.array_equal(got[:, :K], big[:, :K].view(np.uint16))
    assert np.all(got[:, K:] == np.float16(-1.0).view(np.uint16))      # padding untouched


def test_planted_outliers_are_counted(nfp, packed):
    W = workloads.weight_host(128, 256, seed=9)
    W[3, 7] = np.float16(1.7509765625)     # first FP16 value above 1.75
    W[100, 255] = np.float16(-2.0)
    W[64, 0] = np.float16(np.inf)
    W[65, 1] = np.float16(np.nan)
    W[5, 5] = np.float16(1.75)             # boundary value is in range
    Wd = to_dev(W)
    assert oracle.count_out_of_range(W) == 4
    assert nfp.range_check(Wd) == 4
    up, lo, bad = nfp.decompose_count(Wd, packed=packed)
    assert bad == 4
    up_ref, lo_ref, _ = oracle.decompose(W)
    assert_plane_equal(up, up_ref)
    assert_plane_equal(lo, lo_ref)


def test_empty_layer(nfp, packed):
    W = torch.empty((0, 64), dtype=torch.float16, device="cuda:0")
    up, lo = nfp.decompose(W, packed=packed)
    assert tuple(up.shape) == (0, 64)
    assert nfp.reconstruct(up, lo).shape == (0, 64)


@pytest.mark.parametrize("N,K", [(16, 64), (33, 80), (300, 1040)])
def test_pack_and_unpack_are_inverse_permutations(nfp, N, K):
    # the optional packed storage holds the same bytes: pack(row-major plane) equals what
    # decompose_packed writes, unpack gives the row-major plane back, and packed FP16 weights
    # follow their own definition (helpers.pack_fp16_ref)
    from helpers import pack_fp16_ref, pack_plane_ref

    W = workloads.weight_host(N, K, seed=N)
    Wd = to_dev(W)
    up, lo = nfp.decompose(Wd)
    up_p, lo_p = nfp.decompose(Wd, packed=True)
    for rm, pk in ((up, up_p), (lo, lo_p)):
        again = nfp.pack_plane(rm)
        n = nfp.plane_bytes(N, K)
        assert torch.equal(again.data[:n], pk.data[:n])
        assert torch.equal(pk.unpack(), rm)
        assert np.array_equal(pk.data[:n].cpu().numpy(), pack_plane_ref(rm.cpu().numpy()))
    Wp = nfp.pack_fp16(Wd)
    want = pack_fp16_ref(W)
    assert np.array_equal(Wp.data[:want.size].cpu().numpy(), want)


def test_four_wide_merge_equals_the_per_element_rule_in_every_byte_lane(nfp, packed):
    # the kernels rebuild four weights per 32-bit word (Sec. 4.2, Alg. 1): no borrow may cross a
    # byte.  Every in-range word in each of the four byte lanes of a word, next to neighbours
    # with extreme bytes (zero, largest magnitude of either sign, minus zero, a carry into the
    # exponent, a subnormal), against the oracle's per-element reconstruction
    words = workloads.all_fp16_words()
    ok = np.array([oracle.in_range(int(w)) for w in words])
    w = words[ok]
    w = np.concatenate([w, w[:(-w.size) % 4]])                      # a multiple of 4 rows
    neighbours = [0x0000, 0x3F00, 0xBF00, 0x8000, 0x3BFF, 0x0041]
    quads = []
    for lane in range(4):
        for nb in neighbours:
            q = np.full((w.size, 4), nb, dtype=np.uint16)
            q[:, lane] = w
            quads.append(q)
    W = np.concatenate(quads).reshape(-1, 16)                        # rows of 16 words = four 32-bit groups
    up_ref, lo_ref, bad = oracle.decompose(W)
    assert bad == 0
    Wd = to_dev(W.view(np.float16))
    up, lo = nfp.decompose(Wd, packed=packed)
    assert_plane_equal(up, up_ref)
    assert_plane_equal(lo, lo_ref)
    back = bits(nfp.reconstruct(up, lo))
    assert np.array_equal(back, oracle.reconstruct(up_ref, lo_ref))
    assert np.array_equal(back, W)
