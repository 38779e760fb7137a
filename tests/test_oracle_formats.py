"""Pins for the oracle's number formats (Sec. 2.1, Eq. 1) against library routines:
numpy's float16 and PyTorch's CPU float8_e4m3fn."""
import numpy as np
import torch

import oracle
from paper_2506_02024_amd import workloads


def test_fp16_value_equals_numpy_float16_on_every_word():
    words = workloads.all_fp16_words()
    ref = words.view(np.float16).astype(np.float64)
    got = np.array([oracle.fp16_value(int(w)) for w in words])
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], ref[~nan])
    # signed zeros keep their sign
    assert np.signbit(oracle.fp16_value(0x8000)) and not np.signbit(oracle.fp16_value(0x0000))


def test_e4m3_value_equals_torch_float8_e4m3fn_on_every_code():
    codes = torch.arange(256, dtype=torch.int32).to(torch.uint8)
    ref = codes.view(torch.float8_e4m3fn).to(torch.float32).numpy().astype(np.float64)
    got = np.array([oracle.e4m3_value(int(c)) for c in range(256)])
    nan = np.isnan(ref)
    assert set(np.nonzero(nan)[0]) == {0x7F, 0xFF}
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], ref[~nan])
    assert oracle.e4m3_value(0x7E) == 448.0            # largest finite
    assert oracle.e4m3_value(0x01) == 2.0 ** -9        # smallest subnormal


def test_e4m3_encode_equals_torch_cast_inside_the_finite_range():
    rng = np.random.default_rng(0)
    vals = [0.0, -0.0, 448.0, -448.0, 2.0 ** -9, 2.0 ** -10, 3 * 2.0 ** -10, 2.0 ** -11]
    # every midpoint between neighbouring codes (ties) and points just off it
    mags = [oracle.e4m3_value(c) for c in range(0x7F)]
    for a, b in zip(mags[:-1], mags[1:]):
        mid = 0.5 * (a + b)
        vals += [mid, -mid, np.nextafter(np.float32(mid), np.float32(0)),
                 np.nextafter(np.float32(mid), np.float32(1e9))]
    vals += list(rng.uniform(-448, 448, 4000))
    vals += list(rng.standard_normal(4000) * 3.0)
    vals += list(rng.standard_normal(2000) * 0.01)
    v32 = np.array(vals, dtype=np.float32)
    ref = torch.from_numpy(v32).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = np.array([oracle.e4m3_encode(float(v)) for v in v32], dtype=np.uint8)
    assert np.array_equal(got, ref)


def test_e4m3_encode_saturates_and_never_emits_nan_code():
    for v in (449.0, 463.9, 464.0, 480.0, 1e4, 65504.0):
        assert oracle.e4m3_encode(v) == 0x7E
        assert oracle.e4m3_encode(-v) == 0xFE


def test_e4m3_encode_is_identity_on_codes():
    for c in range(256):
        if c & 0x7F == 0x7F:
            continue
        assert oracle.e4m3_encode(oracle.e4m3_value(c)) == c
