"""Shared helpers of the GPU parity tests: tensor plumbing and the error metrics.

Tolerances (stated where they are used as well):
  float32 tensors ........ max_j |got - ref| / max(|ref_j|, rms(ref))  <= 1e-5
  bfloat16 tensors ....... |got - ref| <= ulp_bf16(ref) + 1e-3 per element, ref the unrounded fp64
                           value, ulp_bf16(v) = 2^(floor(log2 |v|) - 7)
  dalpha, dbeta .......... max_j |got - ref| / max(|ref_j|, rms(ref))  <= 1e-4
A purely elementwise relative error is undefined where the reference is 0, hence the rms floor.
"""
import numpy as np
import torch

F32_TOL = 1e-5
GRAD_TOL = 1e-4
BF16_ABS = 1e-3


def to_gpu(a: np.ndarray, dtype: str) -> torch.Tensor:
    if dtype == "bf16":
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(a).cuda()


def to_f64(t: torch.Tensor) -> np.ndarray:
    """GPU result -> float64 numpy, exactly (torch's own widening: nothing of the product package
    takes part in decoding what the kernels wrote)."""
    return t.detach().cpu().to(torch.float64).numpy()


def nan_filled(N: int, d: int, dtype: str) -> torch.Tensor:
    """Output buffer pre-filled with NaN, so that a row the kernel never wrote fails the comparison."""
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    return torch.full((N, d), float("nan"), dtype=tdt, device="cuda")


def rel_err_rms_floor(got: np.ndarray, ref: np.ndarray) -> float:
    ref = np.asarray(ref, dtype=np.float64)
    rms = float(np.sqrt(np.mean(ref ** 2))) if ref.size else 0.0
    den = np.maximum(np.abs(ref), max(rms, 1e-300))
    return float(np.max(np.abs(got - ref) / den)) if ref.size else 0.0


def ulp_bf16(ref: np.ndarray) -> np.ndarray:
    mag = np.maximum(np.abs(ref), 2.0 ** -126)
    return np.exp2(np.floor(np.log2(mag)) - 7.0)


def assert_io_close(got_t: torch.Tensor, ref: np.ndarray, dtype: str, what: str):
    got = to_f64(got_t)
    assert got.shape == ref.shape, what
    assert np.all(np.isfinite(got)), f"{what}: non-finite output"
    if dtype == "f32":
        err = rel_err_rms_floor(got, ref)
        assert err <= F32_TOL, f"{what}: fp32 relative error {err:.3e} > {F32_TOL}"
    else:
        excess = np.abs(got - ref) - (ulp_bf16(ref) + BF16_ABS)
        worst = float(np.max(excess)) if excess.size else -1.0
        assert worst <= 0.0, f"{what}: bf16 error exceeds 1 ulp + 1e-3 by {worst:.3e}"


def assert_grad_close(got_t: torch.Tensor, ref: np.ndarray, what: str):
    got = to_f64(got_t)
    assert np.all(np.isfinite(got)), f"{what}: non-finite output"
    err = rel_err_rms_floor(got, ref)
    assert err <= GRAD_TOL, f"{what}: relative error {err:.3e} > {GRAD_TOL}"
