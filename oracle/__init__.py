"""fp64 CPU oracle for the Walsh-Hadamard output layer (paper Sec. 4.1, Eq. 1; Fig. 1; Fig. 2).

TEST INFRASTRUCTURE ONLY.  Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may
import this package; the product path (paper_2603_08343_amd) never does and shares no code with it.

The arithmetic lives in wht_oracle.c (plain C, IEEE double).  This module only marshals numpy
arrays into it:

    transform(x, method)                      -> z  = H x                        [N,d] float64
    forward(x, alpha, beta, method)           -> y  = alpha*z + beta             [N,d] float64
    forward_residual(x, alpha, beta, resid)   -> y  = resid + alpha*z + beta     [N,d] float64
    forward_residual_stats(x, alpha, beta, resid) -> (y, sumsq), sumsq[n] = sum_j y[n,j]^2
    backward(dy, x, alpha, method, ...)       -> dx, dalpha, dbeta               float64
    hadamard_matrix(d)                        -> H_raw (+-1 integers), entry by entry from the
                                                 oracle's sign rule
    h12()                                     -> the order-12 factor used for d = 12 * 2^m
    butterfly_stage(a, stride)                -> one stage of the Fig. 2 network

`x`/`dy` may be float64, float32, or uint16 arrays holding bfloat16 bit patterns (widened exactly).
method: "matrix" = the O(d^2) definition, "fast" = the butterfly network.  d is 2^n, or 12 * 2^m (this library's reading of the widths
768 and 1536 of Table 2: H = P12 (x) Sylvester, see wht_oracle.c).  Every public function
here is pinned by tests/test_oracle_pins.py (no function is "parity unpinned").
"""
import ctypes
import numpy as np

from .build import ensure_built

_METHODS = {"matrix": 0, "fast": 1}
_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(ensure_built())
        i64, i32, vp = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p
        lib.wht_oracle_transform.argtypes = [vp, vp, i64, i64, i32, i32]
        lib.wht_oracle_forward.argtypes = [vp, vp, vp, vp, i64, i64, i32, i32]
        lib.wht_oracle_forward_residual.argtypes = [vp, vp, vp, vp, vp, i64, i64, i32, i32]
        lib.wht_oracle_backward.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, i32, i32]
        lib.wht_oracle_row_sumsq.argtypes = [vp, vp, i64, i64]
        lib.wht_oracle_butterfly_stage.argtypes = [vp, i64, i64]
        lib.wht_oracle_butterfly_stage.restype = None
        lib.wht_oracle_sign.argtypes = [ctypes.c_uint32, ctypes.c_uint32]
        lib.wht_oracle_sign_d.argtypes = [i64, ctypes.c_uint32, ctypes.c_uint32]
        lib.wht_oracle_h12.argtypes = [i32, i32]
        lib.wht_oracle_bf16_bits_to_double.argtypes = [ctypes.c_uint16]
        lib.wht_oracle_bf16_bits_to_double.restype = ctypes.c_double
        lib.wht_oracle_set_num_threads.argtypes = [i32]
        lib.wht_oracle_set_num_threads.restype = None
        _lib = lib
    return _lib


def _stored(a):
    """(contiguous array, dtype code) for an input tensor; no value is changed."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.float64:
        return a, 0
    if a.dtype == np.float32:
        return a, 1
    if a.dtype == np.uint16:          # bfloat16 bit patterns
        return a, 2
    raise TypeError(f"oracle input must be float64, float32 or uint16(bf16 bits), got {a.dtype}")


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)   # float32 -> float64 is exact


def _ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p) if a is not None else None


def _shape2(a):
    if a.ndim == 1:
        return 1, a.shape[0]
    if a.ndim != 2:
        raise ValueError("expected [N,d] or [d]")
    return a.shape


def _check(rc):
    if rc != 0:
        raise ValueError(f"oracle rejected its arguments (rc={rc}): d must be 2^n or 12 * 2^m")


def num_threads() -> int:
    return int(_load().wht_oracle_num_threads())


def set_num_threads(n: int) -> None:
    _load().wht_oracle_set_num_threads(int(n))


def sign(j: int, k: int) -> int:
    return int(_load().wht_oracle_sign(j, k))


def hadamard_matrix(d: int) -> np.ndarray:
    """Unnormalised d x d sign matrix, built entry by entry from the oracle's sign rule."""
    lib = _load()
    H = np.empty((d, d), dtype=np.int64)
    for j in range(d):
        for k in range(d):
            H[j, k] = lib.wht_oracle_sign_d(d, j, k)
    if (H == 0).any():
        raise ValueError("d must be 2^n or 12 * 2^m")
    return H


def h12() -> np.ndarray:
    """The symmetric, normalised order-12 Hadamard matrix used for d = 12 * 2^m."""
    lib = _load()
    return np.array([[lib.wht_oracle_h12(a, b) for b in range(12)] for a in range(12)], dtype=np.int64)


def bf16_bits_to_float64(bits) -> np.ndarray:
    lib = _load()
    bits = np.asarray(bits, dtype=np.uint16)
    out = np.empty(bits.shape, dtype=np.float64)
    flat_in, flat_out = bits.reshape(-1), out.reshape(-1)
    for i in range(flat_in.size):
        flat_out[i] = lib.wht_oracle_bf16_bits_to_double(int(flat_in[i]))
    return out


def butterfly_stage(a, stride: int) -> np.ndarray:
    a = np.array(a, dtype=np.float64, copy=True)
    d = a.shape[-1]
    if a.ndim != 1 or stride < 1 or d % (2 * stride) != 0:
        raise ValueError("butterfly_stage: 1-D input whose length is a multiple of 2*stride")
    _load().wht_oracle_butterfly_stage(_ptr(a), d, stride)
    return a


def transform(x, method: str = "fast") -> np.ndarray:
    x, code = _stored(x)
    N, d = _shape2(x)
    z = np.empty((N, d), dtype=np.float64)
    _check(_load().wht_oracle_transform(_ptr(x), _ptr(z), N, d, code, _METHODS[method]))
    return z.reshape(x.shape)


def forward(x, alpha, beta, method: str = "fast") -> np.ndarray:
    x, code = _stored(x)
    N, d = _shape2(x)
    alpha, beta = _f64(alpha), _f64(beta)
    if alpha.shape != (d,) or beta.shape != (d,):
        raise ValueError("alpha and beta must have shape [d]")
    y = np.empty((N, d), dtype=np.float64)
    _check(_load().wht_oracle_forward(_ptr(x), _ptr(alpha), _ptr(beta), _ptr(y), N, d, code,
                                      _METHODS[method]))
    return y.reshape(x.shape)


def forward_residual(x, alpha, beta, resid, method: str = "fast") -> np.ndarray:
    """y = resid + alpha*(H x) + beta (Eq. 1 followed by the block's residual connection)."""
    x, code = _stored(x)
    resid, code_r = _stored(resid)
    if code != code_r or x.shape != resid.shape:
        raise ValueError("x and resid must have the same dtype and shape")
    N, d = _shape2(x)
    alpha, beta = _f64(alpha), _f64(beta)
    if alpha.shape != (d,) or beta.shape != (d,):
        raise ValueError("alpha and beta must have shape [d]")
    y = np.empty((N, d), dtype=np.float64)
    _check(_load().wht_oracle_forward_residual(_ptr(x), _ptr(alpha), _ptr(beta), _ptr(resid), _ptr(y),
                                               N, d, code, _METHODS[method]))
    return y.reshape(x.shape)


def forward_residual_stats(x, alpha, beta, resid, method: str = "fast"):
    """(y, sumsq): y = resid + alpha*(H x) + beta and sumsq[n] = sum_j y[n,j]^2, the statistic of a
    following RMS normalisation."""
    y = forward_residual(x, alpha, beta, resid, method)
    y2 = np.ascontiguousarray(y.reshape(-1, y.shape[-1]))
    sumsq = np.empty(y2.shape[0], dtype=np.float64)
    _check(_load().wht_oracle_row_sumsq(_ptr(y2), _ptr(sumsq), y2.shape[0], y2.shape[1]))
    return y, sumsq


def backward(dy, x, alpha, method: str = "fast", want_dx: bool = True, want_param_grads: bool = True):
    """Returns (dx or None, dalpha or None, dbeta or None), all float64."""
    x, code = _stored(x)
    dy, code_dy = _stored(dy)
    if code != code_dy or x.shape != dy.shape:
        raise ValueError("x and dy must have the same dtype and shape")
    N, d = _shape2(x)
    alpha = _f64(alpha)
    if alpha.shape != (d,):
        raise ValueError("alpha must have shape [d]")
    dx = np.empty((N, d), dtype=np.float64) if want_dx else None
    dalpha = np.empty(d, dtype=np.float64) if want_param_grads else None
    dbeta = np.empty(d, dtype=np.float64) if want_param_grads else None
    _check(_load().wht_oracle_backward(_ptr(dy), _ptr(x), _ptr(alpha), _ptr(dx), _ptr(dalpha),
                                       _ptr(dbeta), N, d, code, _METHODS[method]))
    if dx is not None:
        dx = dx.reshape(x.shape)
    return dx, dalpha, dbeta
