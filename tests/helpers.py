"""Shared helpers for the GPU parity tests (comparison rule and host<->device glue)."""
import numpy as np

REL_TOL = 1e-2   # the build's stated GEMM tolerance: relative, fp16 output, fp32 accumulation


def assert_gemm_close(y_gpu, y_ref, what=""):
    """|y - ref| <= 1e-2 |ref| + 1e-2 rms(ref row), and ||y - ref||_F <= 1e-2 ||ref||_F.

    y_gpu: fp16 array from the HIP path; y_ref: float64 from the oracle."""
    y = np.asarray(y_gpu).astype(np.float64)
    assert y.shape == y_ref.shape, (y.shape, y_ref.shape)
    assert np.all(np.isfinite(y)), what + ": non-finite output"
    rms = np.sqrt(np.mean(y_ref ** 2, axis=1, keepdims=True))
    err = np.abs(y - y_ref)
    bound = REL_TOL * np.abs(y_ref) + REL_TOL * rms
    bad = err > bound
    assert not bad.any(), "%s: %d of %d elements out of tolerance, worst err %g at %s" % (
        what, int(bad.sum()), bad.size, float(err.max()), np.unravel_index(np.argmax(err - bound), err.shape))
    den = np.linalg.norm(y_ref)
    if den > 0:
        rel = np.linalg.norm(y - y_ref) / den
        assert rel <= REL_TOL, "%s: normwise error %g" % (what, rel)
        return rel
    return 0.0


def to_dev(a, device="cuda:0"):
    import torch

    return torch.from_numpy(np.ascontiguousarray(a)).to(device)


def bits(t):
    """uint16 numpy view of an fp16 torch tensor."""
    return t.detach().cpu().contiguous().numpy().view(np.uint16)


def pack_plane_ref(a):
    """Packed plane storage written out from its definition: 1 KB blocks of 16 rows x 64
    columns, block (i, j) at (i * Kp/64 + j) * 1024, 16-byte chunk of row r, column group g
    at chunk index r + 16 g; rows and columns past the matrix are zero."""
    a = np.asarray(a, dtype=np.uint8)
    N, K = a.shape
    Np, Kp = -(-N // 16) * 16, -(-K // 64) * 64
    p = np.zeros((Np, Kp), dtype=np.uint8)
    p[:N, :K] = a
    p = p.reshape(Np // 16, 16, Kp // 64, 4, 16)        # i, r, j, g, byte
    return np.ascontiguousarray(p.transpose(0, 2, 3, 1, 4)).reshape(-1)


def pack_fp16_ref(w):
    """Packed FP16 storage written out from its definition: 2 KB blocks of 16 rows x 64 columns,
    each made of two halves of 1 KB; chunk r + 16 g of half h holds columns 16 g + 8 h .. + 7 of
    row r (8 FP16 words); rows and columns past the matrix are zero."""
    w = np.asarray(w).view(np.uint16)
    N, K = w.shape
    Np, Kp = -(-N // 16) * 16, -(-K // 64) * 64
    p = np.zeros((Np, Kp), dtype=np.uint16)
    p[:N, :K] = w
    p = p.reshape(Np // 16, 16, Kp // 64, 4, 2, 8)      # i, r, j, g, h, word
    return np.ascontiguousarray(p.transpose(0, 2, 4, 3, 1, 5)).reshape(-1).view(np.uint8)


def assert_plane_equal(plane, ref):
    """plane: what the library wrote -- a row-major uint8 [N,K] tensor (compared with the
    oracle's array as it is) or a PackedPlane (raw packed bytes, padding included, against the
    layout's definition, and the library's own unpacking); ref: row-major uint8 [N,K] from the
    oracle."""
    ref = np.asarray(ref, dtype=np.uint8)
    if hasattr(plane, "unpack"):
        want = pack_plane_ref(ref)
        got = plane.data[:want.size].cpu().numpy()
        assert np.array_equal(got, want)
        assert np.array_equal(plane.unpack().cpu().numpy(), ref)
    else:
        assert tuple(plane.shape) == ref.shape
        assert np.array_equal(plane.cpu().numpy(), ref)


def structured_sample(M, N, seed=0, full_rows=4, full_cols=4, band_rows=128, band_cols=256):
    """Which outputs of a full-size [M,N] result are compared with the oracle: a few complete rows
    (all N), a few complete columns (all M), and the first and last row / column of every 64-row
    and 128-column band (the edges of every tile shape the kernels use), thinned to band_rows x
    band_cols by a seeded choice that keeps the first and last band.  Returns three (rows, cols)
    pairs of sorted index arrays."""
    rng = np.random.default_rng(4099 + seed)
    full_rows = max(full_rows, -(-32768 // max(N, 1)))          # at least 2^15 outputs in the complete rows alone

    def pick(n, k, always):
        k = min(k, n)
        rest = np.setdiff1d(np.arange(n), always)
        extra = rng.choice(rest, size=max(0, k - len(always)), replace=False) if len(rest) else []
        return np.unique(np.concatenate([np.asarray(always, dtype=np.int64), np.asarray(extra, dtype=np.int64)]))

    def edges(n, band):
        e = np.unique(np.concatenate([np.arange(0, n, band), np.minimum(np.arange(0, n, band) + band - 1, n - 1)]))
        return e

    rows_full = pick(M, full_rows, [0, M - 1] if M > 1 else [0])
    cols_full = pick(N, full_cols, [0, N - 1] if N > 1 else [0])
    er, ec = edges(M, 64), edges(N, 128)
    keep_r = np.unique(np.concatenate([er[:2], er[-2:]]))
    keep_c = np.unique(np.concatenate([ec[:2], ec[-2:]]))
    rows_band = er if len(er) <= band_rows else np.unique(np.concatenate([keep_r, rng.choice(er, band_rows - len(keep_r), replace=False)]))
    cols_band = ec if len(ec) <= band_cols else np.unique(np.concatenate([keep_c, rng.choice(ec, band_cols - len(keep_c), replace=False)]))
    return [(rows_full, np.arange(N)), (np.arange(M), cols_full), (rows_band, cols_band)]


def decompose_ref(W, workers=16):
    """oracle.decompose over row blocks of W on a few host threads (the oracle is called as it
    stands; ctypes releases the interpreter lock during the call).  Returns (upper, lower, bad)."""
    import os
    from concurrent.futures import ThreadPoolExecutor

    import oracle

    W = np.asarray(W)
    N = W.shape[0]
    workers = max(1, min(workers, os.cpu_count() or 1, (N + 255) // 256))
    if workers == 1:
        return oracle.decompose(W)
    bounds = np.linspace(0, N, workers + 1).astype(np.int64)
    with ThreadPoolExecutor(max_workers=workers) as pool:
        parts = list(pool.map(lambda i: oracle.decompose(W[bounds[i]:bounds[i + 1]]), range(workers)))
    return (np.concatenate([p[0] for p in parts]), np.concatenate([p[1] for p in parts]), sum(p[2] for p in parts))
