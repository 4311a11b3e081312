"""`signature` as a differentiable PyTorch operation (paper section 5.3): the forward pass is
`sig_signature`, the backward pass `sig_backward`; both run in the HIP library.  Glue only."""
from __future__ import annotations

import torch

from . import binding


class _Signature(torch.autograd.Function):
    @staticmethod
    def forward(ctx, path, basepoint_value, depth, stream, basepoint, inverse):
        path = path.contiguous()
        bp = basepoint_value.contiguous() if basepoint_value is not None else bool(basepoint)
        plain = binding.sig_signature(path, depth, stream=stream, basepoint=bp)
        d = path.shape[2]
        out = binding.sig_invert(plain, d, depth) if inverse else plain
        ctx.save_for_backward(path, plain, basepoint_value)
        ctx.args = (depth, stream, basepoint, inverse, d)
        return out

    @staticmethod
    def backward(ctx, grad_out):
        path, plain, basepoint_value = ctx.saved_tensors
        depth, stream, basepoint, inverse, d = ctx.args
        grad_out = grad_out.contiguous()
        if inverse:
            # the inverse is a signed permutation that is its own transpose
            grad_out = binding.sig_invert(grad_out, d, depth)
        bp = basepoint_value.contiguous() if basepoint_value is not None else bool(basepoint)
        grad_bp = torch.empty_like(basepoint_value) if basepoint_value is not None else None
        grad_path = binding.sig_backward(path, plain, grad_out, depth, stream=stream, basepoint=bp,
                                         grad_basepoint=grad_bp)
        return grad_path, grad_bp, None, None, None, None


def signature(path, depth: int, stream: bool = False, basepoint=False, inverse: bool = False):
    """Depth-`depth` signature of a batch of paths `[B, L, d]` on the GPU, differentiable in `path`
    and in `basepoint` when that is a `[B, d]` tensor (argument names as in section 5.5)."""
    value = basepoint if isinstance(basepoint, torch.Tensor) else None
    return _Signature.apply(path, value, int(depth), bool(stream), value is not None or bool(basepoint), bool(inverse))
