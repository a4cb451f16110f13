"""MI355X-native Walsh-Hadamard output layer: y = alpha (.) (H x) + beta (paper Sec. 4.1, Eq. 1).

All arithmetic runs in the HIP kernels of libwht_affine.so (C ABI in include/wht_affine.h); this
package only marshals arguments.  There is no CPU fallback: without the built library, or without a
GPU, the calls raise.  `autograd` (imported on demand: it needs torch) wraps the entry points in a
torch.autograd.Function and a Module.
"""
from .binding import (  # noqa: F401
    DTYPE_BF16,
    DTYPE_F32,
    WhtAffineError,
    library,
    library_path,
    wht_affine_backward,
    wht_affine_backward_static,
    wht_affine_backward_workspace_bytes,
    wht_affine_forward,
    wht_affine_forward_residual,
    wht_affine_forward_residual_stats,
    wht_affine_status_string,
    wht_affine_version,
)
