"""Shared helpers for the GPU parity tests (comparison rule and host<->device glue)."""
import numpy as np

REL_TOL = 1e-2   # the benchmark spec: relative tolerance, fp16 output, fp32 accumulation


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


def assert_plane_equal(plane, ref):
    """plane: PackedPlane from the library; ref: row-major uint8 [N,K] from the oracle.
    Checks the raw packed bytes (padding included) and the library's own unpacking."""
    want = pack_plane_ref(ref)
    got = plane.data[:want.size].cpu().numpy()
    assert np.array_equal(got, want)
    assert np.array_equal(plane.unpack().cpu().numpy(), np.asarray(ref, dtype=np.uint8))
