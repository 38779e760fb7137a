"""Pins for the oracle's activation quantisation and both GEMM modes."""
import numpy as np
import torch

import oracle
from paper_2506_02024_amd import workloads


def _f64(a16):
    return np.asarray(a16).view(np.float16).astype(np.float64)


def test_fp16_mode_equals_numpy_float64_matmul():
    W = workloads.weight_host(96, 208, seed=0)
    X = workloads.act_host(7, 208, seed=0)
    Y = oracle.gemm_fp16(X, W)
    ref = X.astype(np.float64) @ W.astype(np.float64).T
    assert Y.shape == (7, 96)
    assert np.allclose(Y, ref, rtol=1e-13, atol=1e-15)
    # a transposed or mis-strided operand would not survive a non-square case
    assert not np.allclose(Y[:, :7], (W[:7].astype(np.float64) @ X.astype(np.float64).T))


def test_fp16_mode_brute_force_tiny():
    W = workloads.weight_host(5, 16, seed=1)
    X = workloads.act_host(3, 16, seed=1)
    Y = oracle.gemm_fp16(X, W)
    for m in range(3):
        for n in range(5):
            acc = 0.0
            for k in range(16):
                acc += float(X[m, k]) * float(W[n, k])
            assert Y[m, n] == acc
            assert oracle.dot_fp16(X[m], W[n]) == acc


def test_fp16_mode_one_hot_rows_return_weight_columns_exactly():
    W = workloads.weight_host(33, 48, seed=2)
    X = np.zeros((48, 48), np.float16)
    X[np.arange(48), np.arange(48)] = 1.0
    Y = oracle.gemm_fp16(X, W)
    assert np.array_equal(Y, W.astype(np.float64).T)


def test_fp16_mode_through_planes_is_the_same_product():
    W = workloads.weight_host(40, 64, seed=3)
    X = workloads.act_host(4, 64, seed=3)
    up, lo, bad = oracle.decompose(W)
    assert bad == 0
    assert np.array_equal(oracle.gemm_fp16_planes(X, up, lo), oracle.gemm_fp16(X, W))


def test_quantize_act_scales_and_codes_match_torch():
    X = workloads.act_host(9, 256, seed=4)
    X[3] = 0                                   # an all-zero row keeps scale 1
    X[5, 7] = np.float16(60000.0)              # a row with a large outlier
    Xq, s = oracle.quantize_act(X)
    xt = torch.from_numpy(X.astype(np.float32))
    amax = xt.abs().amax(dim=1)
    s_ref = torch.where(amax == 0, torch.ones_like(amax), amax / 448.0)
    assert np.array_equal(s, s_ref.numpy())
    q_ref = (xt / s_ref[:, None]).clamp(-448, 448).to(torch.float8_e4m3fn).view(torch.uint8)
    assert np.array_equal(Xq, q_ref.numpy())
    assert not np.any((Xq & 0x7F) == 0x7F)
    # the row maximum always lands on +-448
    rows = [m for m in range(9) if m != 3]
    assert all(0x7E in (Xq[m] & 0x7F) for m in rows)
    assert np.all(Xq[3] == 0)


def test_quantize_act_static_scale():
    X = workloads.act_host(3, 64, seed=5)
    Xq, s = oracle.quantize_act(X, static_scale=0.03125)
    assert np.all(s == np.float32(0.03125))
    xt = torch.from_numpy(X.astype(np.float32)) / 0.03125
    ref = xt.clamp(-448, 448).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(Xq, ref)


def test_fp8_mode_equals_float64_matmul_of_decoded_operands():
    W = workloads.weight_host(72, 160, seed=6)
    X = workloads.act_host(6, 160, seed=6)
    up, lo, _ = oracle.decompose(W)
    Xq, s = oracle.quantize_act(X)
    Y = oracle.gemm_fp8(Xq, s, up)
    dq = torch.from_numpy(Xq).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    dw = torch.from_numpy(up).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    ref = (dq @ dw.T) * s.astype(np.float64)[:, None] * 2.0 ** -8
    assert np.allclose(Y, ref, rtol=1e-13, atol=1e-18)
    assert oracle.dot_fp8(Xq[2], s[2], up[11]) == Y[2, 11]


def test_fp8_mode_one_hot_recovers_upper_plane_values_times_2_pow_minus_8():
    W = workloads.weight_host(20, 32, seed=7)
    up, lo, _ = oracle.decompose(W)
    X = np.zeros((32, 32), np.float16)
    X[np.arange(32), np.arange(32)] = 448.0      # amax = 448 -> scale exactly 1
    Xq, s = oracle.quantize_act(X)
    assert np.all(s == 1.0)
    Y = oracle.gemm_fp8(Xq, s, up)
    dw = torch.from_numpy(up).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    assert np.array_equal(Y, 448.0 * dw.T * 2.0 ** -8)


def test_fp8_mode_with_exact_operands_equals_fp16_mode():
    # weights already representable in E4M3 after the 2^8 shift, activations that
    # quantise exactly (powers of two, row maximum 448 * 2^j): both modes agree
    rng = np.random.default_rng(8)
    wvals = np.array([oracle.e4m3_value(c) for c in range(0x08, 0x7F)]) * 2.0 ** -8
    W = rng.choice(np.concatenate([wvals, -wvals]), size=(24, 64)).astype(np.float16)
    up, lo, bad = oracle.decompose(W)
    assert bad == 0 and np.all(lo & 0x7F == 0)
    X = (2.0 ** rng.integers(-3, 3, size=(5, 64))).astype(np.float16)
    X[:, 0] = np.float16(448.0 / 16)             # row maximum 28 = 448 * 2^-4
    Xq, s = oracle.quantize_act(X)
    assert np.all(s == np.float32(2.0 ** -4))
    assert np.array_equal(oracle.gemm_fp8(Xq, s, up), oracle.gemm_fp16(X, W))


def test_fp8_mode_error_is_the_expected_quantisation_error_only():
    W = workloads.weight_host(256, 1024, seed=9)
    X = workloads.act_host(8, 1024, seed=9)
    up, lo, _ = oracle.decompose(W)
    Xq, s = oracle.quantize_act(X)
    y8 = oracle.gemm_fp8(Xq, s, up)
    y16 = oracle.gemm_fp16(X, W)
    rel = np.linalg.norm(y8 - y16) / np.linalg.norm(y16)
    assert 0.005 < rel < 0.10
