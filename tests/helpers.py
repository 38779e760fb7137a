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
