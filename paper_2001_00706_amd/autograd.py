"""`signature` and `logsignature` as differentiable PyTorch operations (paper section 5.3): the forward passes
are `sig_signature`, `sig_log` and `sig_lyndon_gather`, the backward passes `sig_lyndon_scatter`,
`sig_log_backward` and `sig_backward`; all run in the HIP library.  Glue only."""
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


class _SignatureToLogsignature(torch.autograd.Function):
    @staticmethod
    def forward(ctx, sig, channels, depth, mode):
        sig = sig.contiguous()
        full = binding.sig_log(sig, channels, depth)
        ctx.save_for_backward(sig)
        ctx.args = (channels, depth, mode)
        return full if mode == "expand" else binding.sig_lyndon_gather(full, channels, depth)

    @staticmethod
    def backward(ctx, grad_out):
        (sig,) = ctx.saved_tensors
        channels, depth, mode = ctx.args
        grad_out = grad_out.contiguous()
        grad_log = grad_out if mode == "expand" else binding.sig_lyndon_scatter(grad_out, channels, depth)
        return binding.sig_log_backward(sig, grad_log, channels, depth), None, None, None


def signature_to_logsignature(sig, channels: int, depth: int, mode: str = "words"):
    """Logsignature from signatures `[..., S]` (sections 2.3, 4.3), differentiable in `sig`: the logarithm, then for
    mode "words" the coefficients of the Lyndon words (appendix A.2.4); mode "expand" keeps every word."""
    if mode not in ("words", "expand"):
        raise ValueError('mode must be "words" or "expand"')
    return _SignatureToLogsignature.apply(sig, int(channels), int(depth), mode)


def logsignature(path, depth: int, stream: bool = False, basepoint=False, inverse: bool = False, mode: str = "words"):
    """Depth-`depth` logsignature of a batch of paths `[B, L, d]` on the GPU, differentiable in `path` (and in a
    tensor `basepoint`)."""
    return signature_to_logsignature(signature(path, depth, stream, basepoint, inverse), path.shape[2], depth, mode)
