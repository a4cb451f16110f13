"""torch.autograd plumbing over the C-ABI entry points: a Function and a Module for the
Walsh-Hadamard output layer (paper Sec. 4.1, Eq. 1), so that it drops into a PyTorch attention block
where the dense output projection W_O used to be.  Nothing is computed here: forward calls
wht_affine_forward (or wht_affine_forward_residual), backward calls wht_affine_backward, which
recomputes H x from the saved input instead of storing it.

The paper does not say how alpha and beta start; this module starts them at 1 and 0, which makes
the layer the orthogonal transform itself at initialisation.
"""
import torch

from . import binding


class WhtAffineFunction(torch.autograd.Function):
    """y = [resid +] alpha (.) (H x) + beta over the last dimension of x."""

    @staticmethod
    def forward(ctx, x, alpha, beta, resid=None):
        d = x.shape[-1]
        x2 = x.reshape(-1, d)
        if not x2.is_contiguous():
            x2 = x2.contiguous()
        if resid is None:
            y = binding.wht_affine_forward(x2, alpha, beta)
        else:
            r2 = resid.reshape(-1, d)
            y = binding.wht_affine_forward_residual(x2, alpha, beta, r2 if r2.is_contiguous() else r2.contiguous())
        ctx.save_for_backward(x2, alpha)
        ctx.has_resid = resid is not None
        return y.view(x.shape)

    @staticmethod
    def backward(ctx, dy):
        x2, alpha = ctx.saved_tensors
        d = x2.shape[-1]
        dy2 = dy.reshape(-1, d)
        if not dy2.is_contiguous():
            dy2 = dy2.contiguous()
        want_dx = ctx.needs_input_grad[0]
        want_pg = ctx.needs_input_grad[1] or ctx.needs_input_grad[2]
        dx = dalpha = dbeta = None
        if want_dx or want_pg:
            dx, dalpha, dbeta = binding.wht_affine_backward(dy2, x2, alpha, want_dx=want_dx,
                                                            want_param_grads=want_pg)
        # the residual stream's gradient is dy itself
        return (dx.view(dy.shape) if dx is not None else None, dalpha, dbeta,
                dy if ctx.has_resid and ctx.needs_input_grad[3] else None)


def wht_affine(x, alpha, beta, resid=None):
    """Differentiable y = [resid +] alpha (.) (H x) + beta; x: [..., d] bfloat16|float32 on the GPU."""
    return WhtAffineFunction.apply(x, alpha, beta, resid)


class WhtAffine(torch.nn.Module):
    """The parameter-free transform plus its 2d learnable parameters (Eq. 1; Table 1 counts 2d).
    alpha and beta are float32 whatever the activations' dtype is."""

    def __init__(self, d: int, device=None):
        super().__init__()
        self.d = d
        self.alpha = torch.nn.Parameter(torch.ones(d, dtype=torch.float32, device=device))
        self.beta = torch.nn.Parameter(torch.zeros(d, dtype=torch.float32, device=device))

    def forward(self, x, resid=None):
        return wht_affine(x, self.alpha, self.beta, resid)

    def extra_repr(self):
        return f"d={self.d}"
