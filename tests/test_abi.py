"""CPU-side checks of the C-ABI library: it loads, exports every declared symbol, and
rejects bad arguments before touching a device (no compute calls here)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "nestedfp.h")


@pytest.fixture(scope="module")
def L():
    from paper_2506_02024_amd import binding, build

    if build.is_stale():
        build.build_library()
    return binding.lib()


def declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(nestedfp_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_three_calls_of_the_method():
    names = declared_symbols()
    for n in ("nestedfp_decompose", "nestedfp_gemm", "nestedfp_reconstruct"):
        assert n in names


def test_library_exports_every_declared_symbol(L):
    for name in declared_symbols():
        assert hasattr(L, name), name
        assert ctypes.cast(getattr(L, name), ctypes.c_void_p).value


def test_status_strings(L):
    seen = set()
    for st in range(6):
        s = L.nestedfp_status_string(st).decode()
        assert s and s not in seen
        seen.add(s)
    assert L.nestedfp_version() >= 100


def test_workspace_query_never_scales_with_weight_count(L):
    ws = L.nestedfp_gemm_workspace_size
    for mode in (0, 1):
        for M in (1, 16, 64, 512, 8192):
            for N, K in ((4096, 4096), (28672, 4096), (4096, 14336), (8192, 28672), (57344, 8192),
                         (1024, 65536 * 2)):
                need = ws(M, N, K, mode)
                # at most 8 split-K partial copies of Y plus the quantised activations and scales
                # plus the arrival counters at the start of every workspace
                assert need <= 8 * M * N * 4 + M * K + 4 * M + 1024 + 16384, (mode, M, N, K, need)
        # the decode-sized scratch is a vanishing fraction of the planes it multiplies
        assert ws(16, 57344, 8192, mode) < 57344 * 8192 // 50
    assert ws(16, 4096, 4100, 0) == 0        # K % 16 != 0
    assert ws(16, 4096, 4096, 7) == 0        # unknown mode
    assert ws(-1, 4096, 4096, 0) == 0


def test_argument_errors_are_reported_before_any_launch(L):
    P = ctypes.c_void_p
    fake = P(0x1000)         # aligned, never dereferenced: every call below fails validation first
    # NULL pointers
    assert L.nestedfp_decompose(P(0), 4, 16, 16, fake, fake, P(0), P(0), P(0)) == 1
    assert L.nestedfp_decompose(fake, 4, 16, 16, P(0), fake, P(0), P(0), P(0)) == 1
    assert L.nestedfp_reconstruct(P(0), fake, 4, 16, fake, 16, P(0)) == 1
    # K not a multiple of 16, leading dimension too small, misaligned pointer
    assert L.nestedfp_decompose(fake, 4, 24, 24, fake, fake, P(0), P(0), P(0)) == 2
    assert L.nestedfp_decompose(fake, 4, 32, 16, fake, fake, P(0), P(0), P(0)) == 2
    assert L.nestedfp_decompose(P(0x1004), 4, 32, 32, fake, fake, P(0), P(0), P(0)) == 2
    # gemm: unknown mode, FP16 mode without the lower plane, K % 16
    args = lambda mode, lower, K: (fake, 4, K, K, fake, lower, 8, mode, P(0), fake, 8, fake, 1 << 20, P(0))
    assert L.nestedfp_gemm(*args(5, fake, 32)) == 1
    assert L.nestedfp_gemm(*args(0, P(0), 32)) == 1
    assert L.nestedfp_gemm(*args(0, fake, 40)) == 2
    # workspace missing / too small for FP8 mode (quantised activations live there)
    assert L.nestedfp_gemm(fake, 4, 32, 32, fake, P(0), 8, 1, P(0), fake, 8, P(0), 0, P(0)) == 4
    assert L.nestedfp_gemm(fake, 4, 32, 32, fake, P(0), 8, 1, P(0), fake, 8, fake, 8, P(0)) == 4
    # empty problems are a no-op
    assert L.nestedfp_gemm(fake, 0, 32, 32, fake, fake, 8, 0, P(0), fake, 8, P(0), 0, P(0)) == 0
    assert L.nestedfp_reconstruct(fake, fake, 0, 32, fake, 32, P(0)) == 0
    # sizes the kernels' 32-bit tile offsets cannot address are refused, not mis-computed
    big = (1 << 21) + 16
    assert L.nestedfp_gemm(fake, 4, big, big, fake, fake, 8, 0, P(0), fake, 8, fake, 1 << 20, P(0)) == 2
    assert L.nestedfp_gemm(fake, 4, 32, big, fake, fake, 8, 0, P(0), fake, 8, fake, 1 << 20, P(0)) == 2
    assert L.nestedfp_gemm_packed(fake, 4, big, big, fake, fake, 8, 0, P(0), fake, 8, fake, 1 << 20, P(0)) == 2
    assert L.nestedfp_plain_gemm_fp16(fake, 4, 32, 32, fake, 8, big, fake, 8, fake, 1 << 20, P(0)) == 2
    assert L.nestedfp_decompose(fake, 4, big, big, fake, fake, P(0), P(0), P(0)) == 2
    assert L.nestedfp_gemm_workspace_size(4, 8, big, 0) == 0
    # packed entry points validate like the row-major ones
    assert L.nestedfp_gemm_packed(*args(5, fake, 32)) == 1
    assert L.nestedfp_gemm_packed(*args(0, P(0), 32)) == 1
    assert L.nestedfp_decompose_packed(fake, 4, 24, 24, fake, fake, P(0), P(0), P(0)) == 2
    assert L.nestedfp_reconstruct_packed(P(0), fake, 4, 16, fake, 16, P(0)) == 1
    # unknown plane layout
    assert L.nestedfp_gemm_fp8_prequantized(fake, fake, 4, 32, fake, 8, 7, ctypes.c_float(1.0), fake, 8, fake, 1 << 20, P(0)) == 1
    # workspace initialisation: nothing to clear is fine, a missing or misaligned buffer is not
    L.nestedfp_workspace_init.argtypes = [P, ctypes.c_size_t, P]
    assert L.nestedfp_workspace_init(P(0), 0, P(0)) == 0
    assert L.nestedfp_workspace_init(P(0), 64, P(0)) == 1
    assert L.nestedfp_workspace_init(P(0x1004), 64, P(0)) == 2
    # the load-aware policy of Sec. 5.4: FP8 mode iff the token count exceeds the threshold
    assert [L.nestedfp_select_mode(t, 1024) for t in (0, 1024, 1025)] == [0, 0, 1]
    # measurement probes reject bad arguments
    assert L.nestedfp_probe_stream_read(P(0), 65536, fake, P(0)) == 1
    assert L.nestedfp_probe_stream_read(fake, 1000, fake, P(0)) == 2
    assert L.nestedfp_probe_stream_read_sparse(P(0), 131072, fake, P(0)) == 1
    assert L.nestedfp_probe_stream_read_sparse(fake, 65536, fake, P(0)) == 2
    assert L.nestedfp_probe_mfma(fake, 0, 0, fake, None, P(0)) == 1
    # tuning hook
    assert L.nestedfp_tune(b"no_such_knob", 1) == 1
    assert L.nestedfp_tune(b"small_split", 2) == 0 and L.nestedfp_tune(b"small_split", -1) == 0
    names = []
    i = 0
    while L.nestedfp_tune_name(i):
        names.append(L.nestedfp_tune_name(i).decode())
        i += 1
    assert "small_split" in names and "large_bm" in names


def test_plane_bytes_is_the_padded_block_count(L):
    L.nestedfp_plane_bytes.restype = ctypes.c_size_t
    L.nestedfp_plane_bytes.argtypes = [ctypes.c_int64, ctypes.c_int64]
    # 1 KB per 16-row x 64-column block, rows rounded up to 16 and columns to 64
    assert L.nestedfp_plane_bytes(16, 64) == 1024
    assert L.nestedfp_plane_bytes(17, 64) == 2048
    assert L.nestedfp_plane_bytes(16, 80) == 2048
    assert L.nestedfp_plane_bytes(4096, 4096) == 4096 * 4096
    assert L.nestedfp_plane_bytes(300, 1040) == 304 * 1088
    assert L.nestedfp_plane_bytes(8, 24) == 0          # K must be a multiple of 16
    assert L.nestedfp_plane_bytes(-1, 64) == 0
    assert L.nestedfp_packed_fp16_bytes(300, 1040) == 2 * 304 * 1088


def test_layer_entry_points_reject_missing_descriptors(L):
    P = ctypes.c_void_p
    fake = P(0x1000)
    L.nestedfp_linear_workspace_size.restype = ctypes.c_size_t
    L.nestedfp_linear_workspace_size.argtypes = [ctypes.c_int64, P, ctypes.c_int]
    assert L.nestedfp_linear_workspace_size(16, P(0), 0) == 0
    L.nestedfp_linear.argtypes = [P, ctypes.c_int64, ctypes.c_int64, P, ctypes.c_int, P, P, ctypes.c_int64, P,
                                  ctypes.c_size_t, P]
    assert L.nestedfp_linear(fake, 4, 32, P(0), 0, P(0), fake, 8, P(0), 0, P(0)) == 1
    L.nestedfp_layer_prepare.argtypes = [P, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int, P, P, P, P, P]
    assert L.nestedfp_layer_prepare(fake, 4, 32, 32, 0, fake, fake, fake, P(0), P(0)) == 1
    assert L.nestedfp_layer_prepare(fake, 4, 32, 32, 1, fake, fake, P(0), fake, P(0)) == 1
    assert L.nestedfp_layer_prepare(fake, 4, 32, 32, 9, fake, fake, fake, fake, P(0)) == 1

