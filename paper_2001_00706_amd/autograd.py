"""`signature` as a differentiable PyTorch operation (paper section 5.3): the forward pass is
`sig_forward`, the backward pass `sig_backward`; both run in the HIP library.  Glue only."""
from __future__ import annotations

import torch

from . import binding


class _Signature(torch.autograd.Function):
    @staticmethod
    def forward(ctx, path, depth, stream, basepoint):
        path = path.contiguous()
        out = binding.sig_forward(path, depth, stream=stream, basepoint=basepoint)
        ctx.save_for_backward(path, out)
        ctx.args = (depth, stream, basepoint)
        return out

    @staticmethod
    def backward(ctx, grad_out):
        path, out = ctx.saved_tensors
        depth, stream, basepoint = ctx.args
        grad_path = binding.sig_backward(path, out, grad_out.contiguous(), depth, stream=stream, basepoint=basepoint)
        return grad_path, None, None, None


def signature(path, depth: int, stream: bool = False, basepoint: bool = False):
    """Depth-`depth` signature of a batch of paths `[B, L, d]` on the GPU, differentiable in `path`
    (the argument names are those of section 5.5)."""
    return _Signature.apply(path, int(depth), bool(stream), bool(basepoint))
