"""Python binding of the NestedFP C ABI (include/nestedfp.h): argument marshalling only.

Tensors are torch CUDA tensors (device memory and the current stream come from
PyTorch); every computation runs in the HIP library.  The library is loaded on first
use and a missing build is an error -- there is no fallback path.
"""
import ctypes
import os

import torch

from . import build as _build

MODE_FP16 = 0
MODE_FP8 = 1
LAYOUT_ROWMAJOR = 0
LAYOUT_PACKED = 1
WORKSPACE_COUNTER_BYTES = 16384

OK, ERR_ARG, ERR_SHAPE, ERR_RANGE, ERR_WORKSPACE, ERR_HIP = range(6)

_lib = None


class NestedFPError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__("%s: %s (status %d)" % (where, status_string(status), status))


def lib():
    """The loaded libnestedfp.so (ctypes.CDLL)."""
    global _lib
    if _lib is not None:
        return _lib
    path = os.environ.get("NESTEDFP_LIB") or _build.lib_path()
    if not os.path.exists(path):
        raise RuntimeError(
            "NestedFP HIP library not built: %s is missing; run "
            "`python -c 'import __graft_entry__ as g; g.build()'` first" % path)
    L = ctypes.CDLL(path)
    c = ctypes
    vp, i64, sz, ci, f32 = c.c_void_p, c.c_int64, c.c_size_t, c.c_int, c.c_float
    L.nestedfp_version.restype = ci
    L.nestedfp_version.argtypes = []
    L.nestedfp_status_string.restype = c.c_char_p
    L.nestedfp_status_string.argtypes = [ci]
    L.nestedfp_range_check.restype = ci
    L.nestedfp_range_check.argtypes = [vp, i64, i64, i64, vp, vp, vp]
    for name in ("nestedfp_decompose", "nestedfp_decompose_packed"):
        getattr(L, name).restype = ci
        getattr(L, name).argtypes = [vp, i64, i64, i64, vp, vp, vp, vp, vp]
    for name in ("nestedfp_reconstruct", "nestedfp_reconstruct_packed"):
        getattr(L, name).restype = ci
        getattr(L, name).argtypes = [vp, vp, i64, i64, vp, i64, vp]
    L.nestedfp_packed_fp16_bytes.restype = sz
    L.nestedfp_packed_fp16_bytes.argtypes = [i64, i64]
    L.nestedfp_pack_fp16.restype = ci
    L.nestedfp_pack_fp16.argtypes = [vp, i64, i64, i64, vp, vp]
    L.nestedfp_workspace_init.restype = ci
    L.nestedfp_workspace_init.argtypes = [vp, sz, vp]
    L.nestedfp_plane_bytes.restype = sz
    L.nestedfp_plane_bytes.argtypes = [i64, i64]
    L.nestedfp_pack_plane.restype = ci
    L.nestedfp_pack_plane.argtypes = [vp, i64, i64, i64, vp, vp]
    L.nestedfp_unpack_plane.restype = ci
    L.nestedfp_unpack_plane.argtypes = [vp, i64, i64, vp, i64, vp]
    L.nestedfp_quantize_act.restype = ci
    L.nestedfp_quantize_act.argtypes = [vp, i64, i64, i64, vp, vp, vp, vp]
    L.nestedfp_gemm_workspace_size.restype = sz
    L.nestedfp_gemm_workspace_size.argtypes = [i64, i64, i64, ci]
    for name in ("nestedfp_gemm", "nestedfp_gemm_packed"):
        getattr(L, name).restype = ci
        getattr(L, name).argtypes = [vp, i64, i64, i64, vp, vp, i64, ci, vp, vp, i64, vp, sz, vp]
    L.nestedfp_gemm_static.restype = ci
    L.nestedfp_gemm_static.argtypes = [vp, i64, i64, i64, vp, vp, i64, ci, vp, vp, i64, vp]
    L.nestedfp_plain_gemm_fp16.restype = ci
    L.nestedfp_plain_gemm_fp16.argtypes = [vp, i64, i64, i64, vp, i64, i64, vp, i64, vp, sz, vp]
    L.nestedfp_plain_gemm_fp16_packed.restype = ci
    L.nestedfp_plain_gemm_fp16_packed.argtypes = [vp, i64, i64, i64, vp, i64, vp, i64, vp, sz, vp]
    for name in ("nestedfp_plain_gemm_fp8", "nestedfp_plain_gemm_fp8_packed"):
        getattr(L, name).restype = ci
        getattr(L, name).argtypes = [vp, i64, i64, i64, vp, i64, f32, vp, vp, i64, vp, sz, vp]
    L.nestedfp_gemm_fp8_prequantized.restype = ci
    L.nestedfp_gemm_fp8_prequantized.argtypes = [vp, vp, i64, i64, vp, i64, ci, f32, vp, i64, vp, sz, vp]
    L.nestedfp_layer_prepare.restype = ci
    L.nestedfp_layer_prepare.argtypes = [vp, i64, i64, i64, ci, vp, vp, vp, vp, vp]
    L.nestedfp_select_mode.restype = ci
    L.nestedfp_select_mode.argtypes = [i64, i64]
    L.nestedfp_probe_stream_read.restype = ci
    L.nestedfp_probe_stream_read.argtypes = [vp, sz, vp, vp]
    L.nestedfp_probe_stream_read_sparse.restype = ci
    L.nestedfp_probe_stream_read_sparse.argtypes = [vp, sz, vp, vp]
    L.nestedfp_probe_mfma.restype = ci
    L.nestedfp_probe_mfma.argtypes = [vp, ci, ci, vp, c.POINTER(c.c_double), vp]
    L.nestedfp_linear_workspace_size.restype = sz
    L.nestedfp_linear_workspace_size.argtypes = [i64, vp, ci]
    L.nestedfp_linear.restype = ci
    L.nestedfp_linear.argtypes = [vp, i64, i64, vp, ci, vp, vp, i64, vp, sz, vp]
    L.nestedfp_tune.restype = ci
    L.nestedfp_tune.argtypes = [c.c_char_p, i64]
    L.nestedfp_tune_name.restype = c.c_char_p
    L.nestedfp_tune_name.argtypes = [ci]
    _lib = L
    return L


def status_string(status):
    return lib().nestedfp_status_string(int(status)).decode()


def version():
    return lib().nestedfp_version()


def tune(knob, value):
    st = lib().nestedfp_tune(knob.encode(), int(value))
    if st != OK:
        raise NestedFPError(st, "nestedfp_tune(%s)" % knob)


def _check(st, where):
    if st != OK:
        raise NestedFPError(st, where)


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else ctypes.c_void_p(0)


def _rowmajor(t, name):
    if t.dim() != 2 or t.stride(1) != 1:
        raise ValueError("%s must be 2-D with unit inner stride" % name)
    return t.shape[0], t.shape[1], t.stride(0) if t.shape[0] > 1 else max(t.stride(0), t.shape[1])


def new_workspace(nbytes, device):
    """A workspace of at least nbytes for the GEMM calls, its arrival counters cleared
    (nestedfp_workspace_init).  Calls that may overlap in time need workspaces of their own."""
    ws = torch.empty(max(int(nbytes), 16), dtype=torch.uint8, device=device)
    st = lib().nestedfp_workspace_init(_ptr(ws), ws.numel(), _stream())
    _check(st, "nestedfp_workspace_init")
    return ws


_workspace = new_workspace


def range_check(W):
    """Number of weights of W (fp16 [N,K]) outside the format's range (synchronises)."""
    N, K, ldw = _rowmajor(W, "W")
    cnt = torch.empty(1, dtype=torch.int64, device=W.device)
    host = ctypes.c_uint64(0)
    st = lib().nestedfp_range_check(_ptr(W), N, K, ldw, _ptr(cnt), ctypes.byref(host), _stream())
    if st not in (OK, ERR_RANGE):
        raise NestedFPError(st, "nestedfp_range_check")
    return int(host.value)


class PackedPlane:
    """One byte plane of an [N,K] layer in the library's optional packed storage (1 KB blocks of
    16 rows x 64 columns, see include/nestedfp.h).  `data` is the flat uint8 device tensor."""

    def __init__(self, N, K, device=None, data=None):
        self.N, self.K = int(N), int(K)
        nbytes = plane_bytes(self.N, self.K)
        if data is None:
            data = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=device)
        elif data.numel() < nbytes or data.dtype != torch.uint8:
            raise ValueError("plane buffer too small or not uint8")
        self.data = data

    shape = property(lambda self: (self.N, self.K))
    device = property(lambda self: self.data.device)

    def data_ptr(self):
        return self.data.data_ptr()

    def unpack(self):
        """Row-major [N,K] uint8 copy of the plane."""
        out = torch.empty((self.N, self.K), dtype=torch.uint8, device=self.data.device)
        if self.N > 0:
            st = lib().nestedfp_unpack_plane(_ptr(self.data), self.N, self.K, _ptr(out), self.K, _stream())
            _check(st, "nestedfp_unpack_plane")
        return out


class PackedFP16:
    """FP16 weights of an [N,K] layer in packed storage (2 KB blocks), the operand of
    plain_gemm_fp16 on packed weights."""

    def __init__(self, N, K, data):
        self.N, self.K, self.data = int(N), int(K), data

    shape = property(lambda self: (self.N, self.K))

    def data_ptr(self):
        return self.data.data_ptr()


def plane_bytes(N, K):
    return int(lib().nestedfp_plane_bytes(int(N), int(K)))


def pack_plane(B):
    """Row-major uint8 [N,K] (a byte plane, E4M3 codes) -> PackedPlane."""
    N, K, ld = _rowmajor(B, "B")
    P = PackedPlane(N, K, B.device)
    if N > 0:
        st = lib().nestedfp_pack_plane(_ptr(B), N, K, ld, _ptr(P.data), _stream())
        _check(st, "nestedfp_pack_plane")
    return P


def pack_fp16(W):
    """Row-major fp16 [N,K] -> PackedFP16."""
    N, K, ldw = _rowmajor(W, "W")
    nbytes = int(lib().nestedfp_packed_fp16_bytes(N, K))
    data = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=W.device)
    if N > 0:
        st = lib().nestedfp_pack_fp16(_ptr(W), N, K, ldw, _ptr(data), _stream())
        _check(st, "nestedfp_pack_fp16")
    return PackedFP16(N, K, data)


def _is_packed(plane):
    return isinstance(plane, PackedPlane)


def _new_planes(N, K, device, packed):
    if packed:
        return PackedPlane(N, K, device), PackedPlane(N, K, device)
    return (torch.empty((N, K), dtype=torch.uint8, device=device),
            torch.empty((N, K), dtype=torch.uint8, device=device))


def _check_plane(plane, N, K, name):
    if _is_packed(plane):
        if plane.shape != (N, K):
            raise ValueError("%s plane has the wrong shape" % name)
    elif (plane.dtype != torch.uint8 or tuple(plane.shape) != (N, K) or not plane.is_contiguous()):
        raise ValueError("%s must be a contiguous uint8 [N,K] tensor or a PackedPlane" % name)


def decompose(W, upper=None, lower=None, check=True, packed=False):
    """fp16 W [N,K] -> (upper, lower): row-major uint8 [N,K] tensors, or PackedPlanes with
    packed=True (or when PackedPlanes are passed in).  With check=True (default) waits for the
    result and raises NestedFPError(ERR_RANGE) if the layer is not applicable."""
    N, K, ldw = _rowmajor(W, "W")
    if upper is not None:
        packed = _is_packed(upper)
    if upper is None or lower is None:
        u2, l2 = _new_planes(N, K, W.device, packed)
        upper = u2 if upper is None else upper
        lower = l2 if lower is None else lower
    _check_plane(upper, N, K, "upper")
    _check_plane(lower, N, K, "lower")
    cnt = torch.empty(1, dtype=torch.int64, device=W.device)
    host = ctypes.c_uint64(0)
    fn = lib().nestedfp_decompose_packed if packed else lib().nestedfp_decompose
    st = fn(_ptr(W), N, K, ldw, _ptr(upper), _ptr(lower), _ptr(cnt), ctypes.byref(host) if check else None, _stream())
    _check(st, "nestedfp_decompose")
    return upper, lower


def decompose_count(W, packed=False):
    """Like decompose(check=False) but also returns the out-of-range count (synchronises)."""
    N, K, ldw = _rowmajor(W, "W")
    upper, lower = _new_planes(N, K, W.device, packed)
    cnt = torch.empty(1, dtype=torch.int64, device=W.device)
    host = ctypes.c_uint64(0)
    fn = lib().nestedfp_decompose_packed if packed else lib().nestedfp_decompose
    st = fn(_ptr(W), N, K, ldw, _ptr(upper), _ptr(lower), _ptr(cnt), ctypes.byref(host), _stream())
    if st not in (OK, ERR_RANGE):
        raise NestedFPError(st, "nestedfp_decompose")
    return upper, lower, int(host.value)


def reconstruct(upper, lower, out=None):
    N, K = upper.shape
    if out is None:
        out = torch.empty((N, K), dtype=torch.float16, device=upper.device)
    _, _, ldw = _rowmajor(out, "out")
    fn = lib().nestedfp_reconstruct_packed if _is_packed(upper) else lib().nestedfp_reconstruct
    st = fn(_ptr(upper), _ptr(lower), N, K, _ptr(out), ldw, _stream())
    _check(st, "nestedfp_reconstruct")
    return out


def quantize_act(X, static_scale=None):
    """fp16 X [M,K] -> (Xq uint8 [M,K] E4M3 codes, scales float32 [M])."""
    M, K, ldx = _rowmajor(X, "X")
    Xq = torch.empty((M, K), dtype=torch.uint8, device=X.device)
    scales = torch.empty((M,), dtype=torch.float32, device=X.device)
    st = lib().nestedfp_quantize_act(_ptr(X), M, K, ldx, _ptr(static_scale), _ptr(Xq), _ptr(scales),
                                     _stream())
    _check(st, "nestedfp_quantize_act")
    return Xq, scales


def gemm_workspace_size(M, N, K, mode):
    return int(lib().nestedfp_gemm_workspace_size(M, N, K, mode))


def gemm(X, upper, lower, mode, act_scale=None, out=None, workspace=None):
    """Y = X @ W^T over the planes (row-major uint8 tensors or PackedPlanes), in MODE_FP16 or
    MODE_FP8 (lower may be None in FP8)."""
    M, K, ldx = _rowmajor(X, "X")
    N = upper.shape[0]
    if upper.shape[1] != K:
        raise ValueError("K of X and of the planes differ")
    _check_plane(upper, N, K, "upper")
    if lower is not None:
        _check_plane(lower, N, K, "lower")
        if _is_packed(lower) != _is_packed(upper):
            raise ValueError("upper and lower must use the same storage")
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=X.device)
    _, _, ldy = _rowmajor(out, "out")
    if workspace is None:
        workspace = _workspace(gemm_workspace_size(M, N, K, mode), X.device)
    fn = lib().nestedfp_gemm_packed if _is_packed(upper) else lib().nestedfp_gemm
    st = fn(_ptr(X), M, K, ldx, _ptr(upper), _ptr(lower), N, int(mode), _ptr(act_scale), _ptr(out), ldy,
            _ptr(workspace), workspace.numel(), _stream())
    _check(st, "nestedfp_gemm")
    return out


STATIC_SCRATCH_BYTES = 32 << 20


def gemm_static(X, upper, lower, mode, out, act_scale=None):
    """nestedfp_gemm_static: row-major planes, no workspace argument, nothing allocated -- the
    output tensor is the caller's, the scratch is a fixed array inside the library."""
    M, K, ldx = _rowmajor(X, "X")
    N = upper.shape[0]
    _check_plane(upper, N, K, "upper")
    if _is_packed(upper):
        raise ValueError("gemm_static takes row-major planes")
    _, _, ldy = _rowmajor(out, "out")
    st = lib().nestedfp_gemm_static(_ptr(X), M, K, ldx, _ptr(upper), _ptr(lower), N, int(mode), _ptr(act_scale),
                                    _ptr(out), ldy, _stream())
    _check(st, "nestedfp_gemm_static")
    return out


def plain_gemm_fp16(X, W, out=None, workspace=None):
    """W: row-major fp16 [N,K] tensor, or PackedFP16."""
    M, K, ldx = _rowmajor(X, "X")
    packed = isinstance(W, PackedFP16)
    if packed:
        N, ldw = W.shape[0], K
        if W.shape[1] != K:
            raise ValueError("K of X and of W differ")
    else:
        N, _, ldw = _rowmajor(W, "W")
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=X.device)
    _, _, ldy = _rowmajor(out, "out")
    if workspace is None:
        workspace = _workspace(gemm_workspace_size(M, N, K, MODE_FP16), X.device)
    if packed:
        st = lib().nestedfp_plain_gemm_fp16_packed(_ptr(X), M, K, ldx, _ptr(W), N, _ptr(out), ldy,
                                                   _ptr(workspace), workspace.numel(), _stream())
    else:
        st = lib().nestedfp_plain_gemm_fp16(_ptr(X), M, K, ldx, _ptr(W), N, ldw, _ptr(out), ldy,
                                            _ptr(workspace), workspace.numel(), _stream())
    _check(st, "nestedfp_plain_gemm_fp16")
    return out


def plain_gemm_fp8(X, Wq, w_scale, act_scale=None, out=None, workspace=None):
    """Wq: E4M3 codes as a row-major uint8 [N,K] tensor or a PackedPlane."""
    M, K, ldx = _rowmajor(X, "X")
    N = Wq.shape[0]
    _check_plane(Wq, N, K, "Wq")
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=X.device)
    _, _, ldy = _rowmajor(out, "out")
    if workspace is None:
        workspace = _workspace(gemm_workspace_size(M, N, K, MODE_FP8), X.device)
    fn = lib().nestedfp_plain_gemm_fp8_packed if _is_packed(Wq) else lib().nestedfp_plain_gemm_fp8
    st = fn(_ptr(X), M, K, ldx, _ptr(Wq), N, float(w_scale), _ptr(act_scale), _ptr(out), ldy, _ptr(workspace),
            workspace.numel(), _stream())
    _check(st, "nestedfp_plain_gemm_fp8")
    return out


def gemm_fp8_prequantized(Xq, scales, upper, w_scale=2.0 ** -8, out=None, workspace=None):
    M, K = Xq.shape
    N = upper.shape[0]
    _check_plane(upper, N, K, "upper")
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=Xq.device)
    _, _, ldy = _rowmajor(out, "out")
    if workspace is None:
        workspace = _workspace(gemm_workspace_size(M, N, K, MODE_FP8), Xq.device)
    layout = LAYOUT_PACKED if _is_packed(upper) else LAYOUT_ROWMAJOR
    st = lib().nestedfp_gemm_fp8_prequantized(_ptr(Xq), _ptr(scales), M, K, _ptr(upper), N, layout,
                                              float(w_scale), _ptr(out), ldy, _ptr(workspace),
                                              workspace.numel(), _stream())
    _check(st, "nestedfp_gemm_fp8_prequantized")
    return out


class _LayerStruct(ctypes.Structure):
    _fields_ = [("N", ctypes.c_int64), ("K", ctypes.c_int64), ("is_exception", ctypes.c_int32),
                ("layout", ctypes.c_int32), ("upper", ctypes.c_void_p), ("lower", ctypes.c_void_p),
                ("W", ctypes.c_void_p), ("ldw", ctypes.c_int64), ("out_of_range", ctypes.c_uint64)]


class Layer:
    """One linear as the library describes it: NestedFP planes (row-major, or packed with
    packed=True), or the FP16 weights themselves if the layer is an exception (some |w| > 1.75).
    Keeps the device buffers alive."""

    def __init__(self, W, packed=False):
        N, K, ldw = _rowmajor(W, "W")
        self.c = _LayerStruct()
        upper, lower = _new_planes(N, K, W.device, packed)
        cnt = torch.empty(1, dtype=torch.int64, device=W.device)
        st = lib().nestedfp_layer_prepare(_ptr(W), N, K, ldw, LAYOUT_PACKED if packed else LAYOUT_ROWMAJOR,
                                          _ptr(upper), _ptr(lower), _ptr(cnt), ctypes.byref(self.c), _stream())
        _check(st, "nestedfp_layer_prepare")
        if self.c.is_exception:
            self.W, self.upper, self.lower = W, None, None     # planes released
        else:
            self.W, self.upper, self.lower = None, upper, lower

    is_exception = property(lambda self: bool(self.c.is_exception))
    out_of_range = property(lambda self: int(self.c.out_of_range))
    shape = property(lambda self: (int(self.c.N), int(self.c.K)))


def linear(X, layer, mode, act_scale=None, out=None, workspace=None):
    """Y = X @ W^T for a Layer in the given mode (exception layers always run in FP16)."""
    M, K, ldx = _rowmajor(X, "X")
    N = layer.shape[0]
    if layer.shape[1] != K:
        raise ValueError("K of X and of the layer differ")
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=X.device)
    _, _, ldy = _rowmajor(out, "out")
    if workspace is None:
        workspace = _workspace(lib().nestedfp_linear_workspace_size(M, ctypes.byref(layer.c), int(mode)), X.device)
    st = lib().nestedfp_linear(_ptr(X), M, ldx, ctypes.byref(layer.c), int(mode), _ptr(act_scale),
                               _ptr(out), ldy, _ptr(workspace), workspace.numel(), _stream())
    _check(st, "nestedfp_linear")
    return out


def select_mode(tokens, threshold=1024):
    """The load-aware policy of Sec. 5.4: MODE_FP8 if tokens > threshold else MODE_FP16."""
    return int(lib().nestedfp_select_mode(int(tokens), int(threshold)))


def probe_stream_read(buf, sink=None, sparse=False):
    """Launches the read-only streaming probe over `buf` (device tensor of a multiple of 64 KiB; 128 KiB
    for the variant with few waves per CU, `sparse`); `sink`: an int32 device tensor to reuse (e.g.
    under graph capture), else one is made."""
    if sink is None:
        sink = torch.zeros(1, dtype=torch.int32, device=buf.device)
    fn = lib().nestedfp_probe_stream_read_sparse if sparse else lib().nestedfp_probe_stream_read
    st = fn(_ptr(buf), buf.numel() * buf.element_size(), _ptr(sink), _stream())
    _check(st, "nestedfp_probe_stream_read")


def probe_mfma(operands, fp8, iters):
    """Launches the MFMA-only probe; returns the flops of the launch."""
    sink = torch.zeros(1, dtype=torch.int32, device=operands.device)
    flops = ctypes.c_double(0.0)
    st = lib().nestedfp_probe_mfma(_ptr(operands), int(bool(fp8)), int(iters), _ptr(sink), ctypes.byref(flops),
                                   _stream())
    _check(st, "nestedfp_probe_mfma")
    return flops.value
