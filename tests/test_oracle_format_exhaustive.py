"""Pins for the oracle's decompose / reconstruct (Sec. 4.1) over all 65,536 FP16 words."""
import os

import numpy as np
import torch

import oracle
from paper_2506_02024_amd import workloads

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "format_words.txt")


def _tables():
    words = workloads.all_fp16_words()
    ok = np.array([oracle.in_range(int(w)) for w in words])
    up = np.zeros(65536, np.uint8)
    lo = np.zeros(65536, np.uint8)
    for w in words[ok]:
        up[w], lo[w] = oracle.decompose_one(int(w))
    return words, ok, up, lo


WORDS, OK, UP, LO = _tables()


def test_range_is_magnitude_at_most_1p75():
    # Sec. 4.1: |w| <= 1.75; as a bit test the magnitude field is at most 0x3F00
    vals = WORDS.view(np.float16).astype(np.float64)
    with np.errstate(invalid="ignore"):
        expect = np.abs(vals) <= 1.75
    assert np.array_equal(OK, expect)
    assert np.array_equal(OK, (WORDS & 0x7FFF) <= 0x3F00)
    assert int(OK.sum()) == 32258 and int((~OK).sum()) == 33278
    # every in-range word has a zero exponent MSB (the unused bit of Sec. 4.1)
    assert np.all((WORDS[OK] >> 14) & 1 == 0)


def test_round_trip_is_lossless_on_every_in_range_word():
    for w in WORDS[OK]:
        assert oracle.reconstruct_one(int(UP[w]), int(LO[w])) == int(w)


def test_upper_is_e4m3_rne_of_weight_times_256():
    # Sec. 4.1: the format "effectively applies E4M3 quantization with a fixed
    # scaling factor of 2^8"; checked against PyTorch's CPU cast
    w = WORDS[OK]
    scaled = w.view(np.float16).astype(np.float32) * np.float32(256.0)
    ref = torch.from_numpy(scaled).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(UP[w], ref)
    # no in-range word lands on the NaN code
    assert not np.any((UP[w] & 0x7F) == 0x7F)
    # and the value relation itself, through the oracle's own decoders' pins
    dec = np.array([oracle.e4m3_value(int(c)) for c in UP[w]])
    exact = scaled.astype(np.float64)
    spacing = np.maximum(2.0 ** (np.floor(np.log2(np.maximum(np.abs(exact), 2.0 ** -6))) - 3),
                         2.0 ** -9)
    assert np.all(np.abs(dec - exact) <= 0.5 * spacing)


def test_lower_is_low_mantissa_byte():
    w = WORDS[OK]
    assert np.array_equal(LO[w], (w & 0xFF).astype(np.uint8))


def test_checksum_bit_marks_round_up():
    # Sec. 4.1 "FP16 Reconstruction": LSB(upper) != MSB(lower) <=> rounded up
    w = WORDS[OK].astype(np.int64)
    truncated = (w & 0x7FFF) >> 7
    rounded_up = (UP[w].astype(np.int64) & 0x7F) != (truncated & 0x7F)
    checksum = (UP[w] & 1) != (LO[w] >> 7)
    assert np.array_equal(rounded_up, checksum)
    assert rounded_up.any() and (~rounded_up).any()


def test_closed_form_of_upper():
    w = WORDS[OK].astype(np.int64)
    mag = w & 0x7FFF
    closed = ((w >> 15) << 7) | ((mag + 0x3F + ((mag >> 7) & 1)) >> 7)
    assert np.array_equal(UP[WORDS[OK]].astype(np.int64), closed)


def test_golden_words():
    n = 0
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        h, u, l = line.split()[:3]
        bits = int(h, 16)
        assert oracle.in_range(bits)
        assert oracle.decompose_one(bits) == (int(u, 16), int(l, 16)), line
        assert oracle.reconstruct_one(int(u, 16), int(l, 16)) == bits, line
        n += 1
    assert n >= 12


def test_tensor_forms_agree_with_scalar_forms_and_count_rejects():
    W = WORDS.reshape(256, 256)
    up, lo, bad = oracle.decompose(W)
    assert bad == 33278 == oracle.count_out_of_range(W)
    ok = OK.reshape(256, 256)
    assert np.array_equal(up[ok], UP[WORDS[OK]])
    assert np.array_equal(lo[ok], LO[WORDS[OK]])
    back = oracle.reconstruct(up, lo)
    assert np.array_equal(back[ok], W[ok])
