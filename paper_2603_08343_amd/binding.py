"""ctypes binding of libwht_affine.so -- same names as the C ABI (include/wht_affine.h).

Argument marshalling only: torch supplies device memory and the stream, every step of the layer
runs in the HIP kernels.  The `*_raw` calls take integer device addresses and return the status
code; the tensor calls check shapes/dtypes, allocate outputs and the backward workspace with torch,
and raise WhtAffineError on a non-zero status.
"""
import ctypes
import os

DTYPE_F32 = 0
DTYPE_BF16 = 1

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libwht_affine.so")
_lib = None

EXPORTS = (
    "wht_affine_forward",
    "wht_affine_forward_residual",
    "wht_affine_forward_residual_stats",
    "wht_affine_backward_workspace_bytes",
    "wht_affine_backward",
    "wht_affine_backward_static",
    "wht_affine_status_string",
    "wht_affine_version",
)


class WhtAffineError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: status {status} ({wht_affine_status_string(status)})")


def library_path() -> str:
    return _LIB_PATH


def library():
    """The loaded shared library.  Raises if it has not been built: there is no fallback path."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError(
                f"{_LIB_PATH} is missing: build it with `python -m paper_2603_08343_amd.build` "
                "(hipcc, gfx950). The layer has no CPU or eager fallback.")
        lib = ctypes.CDLL(_LIB_PATH)
        vp, i64, i32, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_size_t
        lib.wht_affine_forward.argtypes = [vp, vp, vp, vp, i64, i32, i32, vp]
        lib.wht_affine_forward.restype = ctypes.c_int
        lib.wht_affine_forward_residual.argtypes = [vp, vp, vp, vp, vp, i64, i32, i32, vp]
        lib.wht_affine_forward_residual.restype = ctypes.c_int
        lib.wht_affine_forward_residual_stats.argtypes = [vp, vp, vp, vp, vp, vp, i64, i32, i32, vp]
        lib.wht_affine_forward_residual_stats.restype = ctypes.c_int
        lib.wht_affine_backward_workspace_bytes.argtypes = [i64, i32, i32]
        lib.wht_affine_backward_workspace_bytes.restype = sz
        lib.wht_affine_backward.argtypes = [vp, vp, vp, vp, vp, vp, i64, i32, i32, vp, sz, vp]
        lib.wht_affine_backward.restype = ctypes.c_int
        lib.wht_affine_backward_static.argtypes = [vp, vp, vp, vp, vp, vp, i64, i32, i32, vp]
        lib.wht_affine_backward_static.restype = ctypes.c_int
        lib.wht_affine_status_string.argtypes = [ctypes.c_int]
        lib.wht_affine_status_string.restype = ctypes.c_char_p
        lib.wht_affine_version.argtypes = []
        lib.wht_affine_version.restype = ctypes.c_int
        _lib = lib
    return _lib


# ------------------------------------------------------------------ raw calls (addresses, status)

def wht_affine_forward_raw(x, alpha, beta, y, N, d, dtype, stream=0) -> int:
    return library().wht_affine_forward(x, alpha, beta, y, N, d, dtype, stream)


def wht_affine_forward_residual_raw(x, alpha, beta, resid, y, N, d, dtype, stream=0) -> int:
    return library().wht_affine_forward_residual(x, alpha, beta, resid, y, N, d, dtype, stream)


def wht_affine_forward_residual_stats_raw(x, alpha, beta, resid, y, sumsq, N, d, dtype, stream=0) -> int:
    return library().wht_affine_forward_residual_stats(x, alpha, beta, resid, y, sumsq, N, d, dtype, stream)


def wht_affine_backward_raw(dy, x, alpha, dx, dalpha, dbeta, N, d, dtype, workspace, workspace_bytes,
                            stream=0) -> int:
    return library().wht_affine_backward(dy, x, alpha, dx, dalpha, dbeta, N, d, dtype, workspace,
                                         workspace_bytes, stream)


def wht_affine_backward_static_raw(dy, x, alpha, dx, dalpha, dbeta, N, d, dtype, stream=0) -> int:
    return library().wht_affine_backward_static(dy, x, alpha, dx, dalpha, dbeta, N, d, dtype, stream)


STATIC_WORKSPACE_BYTES = 16 << 20       # WHT_STATIC_WORKSPACE_BYTES


def wht_affine_backward_workspace_bytes(N, d, dtype) -> int:
    return int(library().wht_affine_backward_workspace_bytes(N, d, dtype))


def wht_affine_status_string(status: int) -> str:
    return library().wht_affine_status_string(int(status)).decode()


def wht_affine_version() -> int:
    return int(library().wht_affine_version())


# ------------------------------------------------------------------ tensor calls

_torch_module = None


def _torch():
    """torch, once a GPU has been seen (checked on the first call only: a decoding loop calls this
    binding every few microseconds)."""
    global _torch_module
    if _torch_module is None:
        import torch
        if not torch.cuda.is_available():
            raise RuntimeError("wht_affine needs an AMD GPU (gfx950); there is no CPU fallback")
        _torch_module = torch
    return _torch_module


def _dtype_code(t, torch):
    if t.dtype == torch.float32:
        return DTYPE_F32
    if t.dtype == torch.bfloat16:
        return DTYPE_BF16
    raise TypeError(f"x must be float32 or bfloat16, got {t.dtype}")


def _check_io(t, name, torch, like=None):
    if not t.is_cuda or not t.is_contiguous() or t.dim() != 2:
        raise ValueError(f"{name} must be a contiguous [N,d] GPU tensor")
    if like is not None and (t.shape != like.shape or t.dtype != like.dtype or t.device != like.device):
        raise ValueError(f"{name} must match x in shape, dtype and device")


def _check_param(p, name, d, x, torch):
    if not p.is_cuda or p.dtype != torch.float32 or p.shape != (d,) or not p.is_contiguous() \
            or p.device != x.device:
        raise ValueError(f"{name} must be a contiguous float32 [d] tensor on x's device")


def _stream_handle(stream, torch, device):
    if stream is not None:
        return stream.cuda_stream
    raw = getattr(torch._C, "_cuda_getCurrentRawStream", None)     # the handle without a Stream object
    if raw is not None and device.index is not None:
        return raw(device.index)
    return torch.cuda.current_stream(device).cuda_stream


class _DeviceGuard:
    """`with torch.cuda.device(dev)` only when dev is not the current device already."""

    def __init__(self, torch, device):
        self._ctx = None
        if device.index is not None and device.index != torch.cuda.current_device():
            self._ctx = torch.cuda.device(device)

    def __enter__(self):
        if self._ctx is not None:
            self._ctx.__enter__()

    def __exit__(self, *exc):
        if self._ctx is not None:
            return self._ctx.__exit__(*exc)
        return False


def wht_affine_forward(x, alpha, beta, y=None, stream=None):
    """y = alpha (.) (H x) + beta  (Eq. 1).  x: [N,d] float32|bfloat16 on the GPU; alpha, beta: [d] float32."""
    torch = _torch()
    _check_io(x, "x", torch)
    N, d = x.shape
    _check_param(alpha, "alpha", d, x, torch)
    _check_param(beta, "beta", d, x, torch)
    if y is None:
        y = torch.empty_like(x)
    else:
        _check_io(y, "y", torch, like=x)
    # torch gives an empty tensor a NULL address; the library never touches x, y when N = 0
    xp, yp = (x.data_ptr(), y.data_ptr()) if N > 0 else (alpha.data_ptr(), alpha.data_ptr())
    with _DeviceGuard(torch, x.device):
        rc = wht_affine_forward_raw(xp, alpha.data_ptr(), beta.data_ptr(), yp, N, d,
                                    _dtype_code(x, torch), _stream_handle(stream, torch, x.device))
    if rc != 0:
        raise WhtAffineError(rc, "wht_affine_forward")
    return y


def wht_affine_forward_residual(x, alpha, beta, resid, y=None, stream=None):
    """y = resid + alpha (.) (H x) + beta: the layer with the block's residual add fused in."""
    torch = _torch()
    _check_io(x, "x", torch)
    _check_io(resid, "resid", torch, like=x)
    N, d = x.shape
    _check_param(alpha, "alpha", d, x, torch)
    _check_param(beta, "beta", d, x, torch)
    if y is None:
        y = torch.empty_like(x)
    else:
        _check_io(y, "y", torch, like=x)
    ptrs = (x.data_ptr(), resid.data_ptr(), y.data_ptr()) if N > 0 else (alpha.data_ptr(),) * 3
    with _DeviceGuard(torch, x.device):
        rc = wht_affine_forward_residual_raw(ptrs[0], alpha.data_ptr(), beta.data_ptr(), ptrs[1], ptrs[2], N, d,
                                             _dtype_code(x, torch), _stream_handle(stream, torch, x.device))
    if rc != 0:
        raise WhtAffineError(rc, "wht_affine_forward_residual")
    return y


def wht_affine_forward_residual_stats(x, alpha, beta, resid, y=None, sumsq=None, stream=None):
    """(y, sumsq): y = resid + alpha (.) (H x) + beta and sumsq[n] = sum_j y[n,j]^2 (float32 [N]), the
    statistic of an RMS normalisation that follows the residual stream."""
    torch = _torch()
    _check_io(x, "x", torch)
    _check_io(resid, "resid", torch, like=x)
    N, d = x.shape
    _check_param(alpha, "alpha", d, x, torch)
    _check_param(beta, "beta", d, x, torch)
    if y is None:
        y = torch.empty_like(x)
    else:
        _check_io(y, "y", torch, like=x)
    if sumsq is None:
        sumsq = torch.empty(N, dtype=torch.float32, device=x.device)
    elif not sumsq.is_cuda or sumsq.dtype != torch.float32 or sumsq.shape != (N,) or not sumsq.is_contiguous() \
            or sumsq.device != x.device:
        raise ValueError("sumsq must be a contiguous float32 [N] tensor on x's device")
    ptrs = (x.data_ptr(), resid.data_ptr(), y.data_ptr(), sumsq.data_ptr()) if N > 0 else (alpha.data_ptr(),) * 4
    with _DeviceGuard(torch, x.device):
        rc = wht_affine_forward_residual_stats_raw(ptrs[0], alpha.data_ptr(), beta.data_ptr(), ptrs[1], ptrs[2],
                                                   ptrs[3], N, d, _dtype_code(x, torch),
                                                   _stream_handle(stream, torch, x.device))
    if rc != 0:
        raise WhtAffineError(rc, "wht_affine_forward_residual_stats")
    return y, sumsq


def wht_affine_backward(dy, x, alpha, dx=None, dalpha=None, dbeta=None, workspace=None, stream=None,
                        want_dx=True, want_param_grads=True):
    """Returns (dx, dalpha, dbeta) with dx = H(alpha (.) dy), dalpha = sum_n dy (.) Hx, dbeta = sum_n dy.
    want_dx=False or want_param_grads=False leaves those outputs out (None in the result); without
    the parameter gradients x is not needed and may be None."""
    torch = _torch()
    if not want_dx and not want_param_grads:
        raise ValueError("nothing to compute: want_dx and want_param_grads are both False")
    _check_io(dy, "dy", torch)
    if want_param_grads and x is None:
        raise ValueError("x is needed for the parameter gradients (want_param_grads=True)")
    if x is not None:
        _check_io(x, "x", torch, like=dy)
    N, d = dy.shape
    _check_param(alpha, "alpha", d, dy, torch)
    code = _dtype_code(dy, torch)
    if not want_dx:
        dx = None
    elif dx is None:
        dx = torch.empty_like(dy)
    else:
        _check_io(dx, "dx", torch, like=dy)
    if not want_param_grads:
        dalpha = dbeta = None
    else:
        if dalpha is None:
            dalpha = torch.empty(d, dtype=torch.float32, device=dy.device)
        else:
            _check_param(dalpha, "dalpha", d, dy, torch)
        if dbeta is None:
            dbeta = torch.empty(d, dtype=torch.float32, device=dy.device)
        else:
            _check_param(dbeta, "dbeta", d, dy, torch)
    ws_ptr, ws_bytes = 0, 0
    if want_param_grads:
        need = wht_affine_backward_workspace_bytes(N, d, code)
        if workspace is None:
            workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=dy.device)
        elif not workspace.is_cuda or not workspace.is_contiguous() or workspace.device != dy.device:
            raise ValueError("workspace must be a contiguous GPU tensor on dy's device")
        ws_ptr, ws_bytes = workspace.data_ptr(), workspace.numel() * workspace.element_size()
    # torch gives an empty tensor a NULL address; the library never touches dy, x, dx when N = 0
    dummy = alpha.data_ptr()
    dy_p = dy.data_ptr() if N > 0 else dummy
    x_p = 0 if not want_param_grads else (x.data_ptr() if N > 0 else dummy)
    dx_p = 0 if dx is None else (dx.data_ptr() if N > 0 else dummy)
    with _DeviceGuard(torch, dy.device):
        rc = wht_affine_backward_raw(dy_p, x_p, alpha.data_ptr(), dx_p,
                                     dalpha.data_ptr() if dalpha is not None else 0,
                                     dbeta.data_ptr() if dbeta is not None else 0, N, d, code,
                                     ws_ptr, ws_bytes, _stream_handle(stream, torch, dy.device))
    if rc != 0:
        raise WhtAffineError(rc, "wht_affine_backward")
    return dx, dalpha, dbeta

def wht_affine_backward_static(dy, x, alpha, dx=None, dalpha=None, dbeta=None, stream=None):
    """wht_affine_backward without a workspace: the library's own static scratch holds the partial
    sums (for callers that must not allocate; pass dx, dalpha and dbeta in and nothing is
    allocated here either).  Returns (dx, dalpha, dbeta)."""
    torch = _torch()
    _check_io(dy, "dy", torch)
    if x is None:
        raise ValueError("x is needed for the parameter gradients")
    _check_io(x, "x", torch, like=dy)
    N, d = dy.shape
    _check_param(alpha, "alpha", d, dy, torch)
    if dx is None:
        dx = torch.empty_like(dy)
    else:
        _check_io(dx, "dx", torch, like=dy)
    if dalpha is None:
        dalpha = torch.empty(d, dtype=torch.float32, device=dy.device)
    else:
        _check_param(dalpha, "dalpha", d, dy, torch)
    if dbeta is None:
        dbeta = torch.empty(d, dtype=torch.float32, device=dy.device)
    else:
        _check_param(dbeta, "dbeta", d, dy, torch)
    dummy = alpha.data_ptr()
    ptrs = (dy.data_ptr(), x.data_ptr(), dx.data_ptr()) if N > 0 else (dummy,) * 3
    with _DeviceGuard(torch, dy.device):
        rc = wht_affine_backward_static_raw(ptrs[0], ptrs[1], alpha.data_ptr(), ptrs[2], dalpha.data_ptr(),
                                            dbeta.data_ptr(), N, d, _dtype_code(dy, torch),
                                            _stream_handle(stream, torch, dy.device))
    if rc != 0:
        raise WhtAffineError(rc, "wht_affine_backward_static")
    return dx, dalpha, dbeta
