"""The layer's kernels in the debug build that poisons LDS (libwht_affine_poison.so: after every read
of an exchange region or of a wave's own stage slot the thread overwrites what it read with NaN).  A
read that comes before the data it is meant to see -- a missing barrier between a put and a get, a
missing wait on a prefetch -- returns NaN there instead of the previous token group's plausible
values, so the ordinary comparison against the oracle turns a synchronisation mistake into a hard
failure.  Widths in this build: 512 (butterfly schedule, LDS re-deals), 4096 and 8192 (matrix-core
schedule, one exchange; the three-team backward), 16384 (two exchanges in the backward), 6144
(12 * 2^m rows), bf16 and, up to 8192, float32."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
import paper_2603_08343_amd as wht
from paper_2603_08343_amd import synth
from paper_2603_08343_amd.build import POISON_LIB
from parity import assert_grad_close, assert_io_close, nan_filled, to_gpu

pytestmark = pytest.mark.gpu

_lib = None


def poison_lib():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(POISON_LIB)
        vp, i64, i32, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_size_t
        lib.wht_affine_forward.argtypes = [vp, vp, vp, vp, i64, i32, i32, vp]
        lib.wht_affine_forward_residual_stats.argtypes = [vp, vp, vp, vp, vp, vp, i64, i32, i32, vp]
        lib.wht_affine_backward_workspace_bytes.argtypes = [i64, i32, i32]
        lib.wht_affine_backward_workspace_bytes.restype = sz
        lib.wht_affine_backward.argtypes = [vp, vp, vp, vp, vp, vp, i64, i32, i32, vp, sz, vp]
        _lib = lib
    return _lib


@pytest.mark.parametrize("d,dtype,N", [(512, "bf16", 300), (512, "f32", 300), (4096, "bf16", 1031), (4096, "f32", 70),
                                       (8192, "bf16", 700), (8192, "f32", 300), (16384, "bf16", 300), (6144, "bf16", 600)])
def test_poisoned_lds_build_matches_the_oracle(d, dtype, N):
    print(f"[poison] d={d} {dtype} N={N}", flush=True)
    lib = poison_lib()
    inp = synth.make_inputs(N, d, dtype, seed=d + N)
    code = wht.DTYPE_BF16 if dtype == "bf16" else wht.DTYPE_F32
    x, dy = to_gpu(inp.x, dtype), to_gpu(inp.dy, dtype)
    a, b = torch.from_numpy(inp.alpha).cuda(), torch.from_numpy(inp.beta).cuda()
    stream = torch.cuda.current_stream().cuda_stream
    y = nan_filled(N, d, dtype)
    assert lib.wht_affine_forward(x.data_ptr(), a.data_ptr(), b.data_ptr(), y.data_ptr(), N, d, code, stream) == 0
    yr, ss = nan_filled(N, d, dtype), torch.full((N,), float("nan"), device="cuda")
    assert lib.wht_affine_forward_residual_stats(x.data_ptr(), a.data_ptr(), b.data_ptr(), dy.data_ptr(), yr.data_ptr(),
                                                 ss.data_ptr(), N, d, code, stream) == 0
    need = lib.wht_affine_backward_workspace_bytes(N, d, code)
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    dx = nan_filled(N, d, dtype)
    da, db = torch.full((d,), float("nan"), device="cuda"), torch.full((d,), float("nan"), device="cuda")
    assert lib.wht_affine_backward(dy.data_ptr(), x.data_ptr(), a.data_ptr(), dx.data_ptr(), da.data_ptr(), db.data_ptr(),
                                   N, d, code, ws.data_ptr(), need, stream) == 0
    dx_only = nan_filled(N, d, dtype)
    assert lib.wht_affine_backward(dy.data_ptr(), 0, a.data_ptr(), dx_only.data_ptr(), 0, 0, N, d, code, 0, 0, stream) == 0
    torch.cuda.synchronize()
    method = "matrix" if d <= 512 else "fast"
    assert_io_close(y, oracle.forward(inp.x, inp.alpha, inp.beta, method), dtype, f"poison fwd d={d}")
    ref_yr, ref_ss = oracle.forward_residual_stats(inp.x, inp.alpha, inp.beta, inp.dy, method)
    assert_io_close(yr, ref_yr, dtype, f"poison fwd+resid d={d}")
    assert np.max(np.abs(ss.cpu().numpy().astype(np.float64) - ref_ss) / ref_ss) <= 1e-5
    rdx, rda, rdb = oracle.backward(inp.dy, inp.x, inp.alpha, method)
    assert_io_close(dx, rdx, dtype, f"poison bwd dx d={d}")
    assert_io_close(dx_only, rdx, dtype, f"poison bwd dx-only d={d}")
    assert_grad_close(da, rda, f"poison dalpha d={d}")
    assert_grad_close(db, rdb, f"poison dbeta d={d}")
