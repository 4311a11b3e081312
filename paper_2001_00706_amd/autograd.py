"""`signature` and `logsignature` as differentiable PyTorch operations (paper section 5.3): the forward passes
are `sig_signature`, `sig_log` and `sig_lyndon_gather`, the backward passes `sig_lyndon_scatter`,
`sig_log_backward` and `sig_backward` (`sig_backward_chunked` for few long paths); all run in the HIP library.  Glue only."""
from __future__ import annotations

import torch

from . import binding


class _Signature(torch.autograd.Function):
    @staticmethod
    def forward(ctx, path, basepoint_value, depth, stream, basepoint, inverse):
        path = path.contiguous()
        bp = basepoint_value.contiguous() if basepoint_value is not None else bool(basepoint)
        B, L, d = path.shape
        chunks = 1 if stream else binding.sig_forward_chunks_hint(B, L, d, depth, bool(basepoint), binding._dtype_of(path))
        if chunks > 1:   # few long paths: the scan as a reduction over the length (section 5.1)
            plain = binding.sig_forward_chunked(path, depth, chunks, basepoint=bp)
        else:
            plain = binding.sig_signature(path, depth, stream=stream, basepoint=bp)
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
        B, L, _ = path.shape
        chunks = 1 if stream else binding.sig_backward_chunks_hint(B, L, d, depth, bool(basepoint), binding._dtype_of(path))
        if chunks > 1:   # few long paths: the walk back along the path cut into stretches
            grad_path = binding.sig_backward_chunked(path, grad_out, depth, chunks, basepoint=bp, grad_basepoint=grad_bp)
        else:
            grad_path = binding.sig_backward(path, plain, grad_out, depth, stream=stream, basepoint=bp,
                                             grad_basepoint=grad_bp)
        return grad_path, grad_bp, None, None, None, None


class _Combine(torch.autograd.Function):
    @staticmethod
    def forward(ctx, a, b, channels, depth):
        a, b = a.contiguous(), b.contiguous()
        ctx.save_for_backward(a, b)
        ctx.args = (channels, depth)
        return binding.sig_combine(a, b, channels, depth)

    @staticmethod
    def backward(ctx, grad_out):
        a, b = ctx.saved_tensors
        channels, depth = ctx.args
        grad_a, grad_b = binding.sig_combine_backward(a, b, grad_out.contiguous(), channels, depth)
        return grad_a, grad_b, None, None


class _CombineGrouped(torch.autograd.Function):
    @staticmethod
    def forward(ctx, a, sigs, channels, depth):
        a, sigs = a.contiguous(), sigs.contiguous()
        ctx.save_for_backward(a, sigs)
        ctx.args = (channels, depth)
        return binding.sig_combine_grouped(a, sigs, channels, depth)

    @staticmethod
    def backward(ctx, grad_out):
        a, sigs = ctx.saved_tensors
        channels, depth = ctx.args
        grad_a, grad_sigs = binding.sig_combine_grouped_backward(a, sigs, grad_out.contiguous(), channels, depth)
        return grad_a, grad_sigs, None, None


def signature_combine(sig1, sig2, channels: int, depth: int):
    """Group product `sig1 [x] sig2` of two batches of signatures `[B, S]` (section 5.5, "combining adjacent
    intervals"), differentiable in both."""
    return _Combine.apply(sig1, sig2, int(channels), int(depth))


def multi_signature_combine(sigs, channels: int, depth: int):
    """Ordered product of a list of batches of signatures `[B, S]`, differentiable in each: neighbours are joined
    pairwise, in ceil(log2 n) rounds of products (the product is associative)."""
    sigs = list(sigs)
    if not sigs:
        raise ValueError("at least one signature is needed")
    while len(sigs) > 1:
        joined = [signature_combine(sigs[i], sigs[i + 1], channels, depth) for i in range(0, len(sigs) - 1, 2)]
        if len(sigs) % 2:
            joined.append(sigs[-1])
        sigs = joined
    return sigs[0]


def signature(path, depth: int, stream: bool = False, basepoint=False, inverse: bool = False, initial=None):
    """Depth-`depth` signature of a batch of paths `[B, L, d]` on the GPU, differentiable in `path`,
    in `basepoint` when that is a `[B, d]` tensor, and in `initial` (argument names as in section 5.5).

    `initial` `[B, S]` is the signature of the data that came before; the result is `initial [x] Sig(path)`, in
    stream mode for every prefix (inverted as a whole if `inverse`)."""
    value = basepoint if isinstance(basepoint, torch.Tensor) else None
    flag = value is not None or bool(basepoint)
    if initial is None:
        return _Signature.apply(path, value, int(depth), bool(stream), flag, bool(inverse))
    d = path.shape[2]
    needs_grad = torch.is_grad_enabled() and any(t is not None and t.requires_grad for t in (path, value, initial))
    if not needs_grad:   # one call, `initial` applied in place behind the scan
        bp = value.contiguous() if value is not None else flag
        return binding.sig_signature(path.contiguous(), int(depth), stream=bool(stream), basepoint=bp, inverse=bool(inverse),
                                     initial=initial.contiguous())
    plain = _Signature.apply(path, value, int(depth), bool(stream), flag, False)
    if stream:
        joined = _CombineGrouped.apply(initial, plain, d, int(depth))
    else:
        joined = signature_combine(initial, plain, d, depth)
    return _Invert.apply(joined, d, int(depth)) if inverse else joined


class _Invert(torch.autograd.Function):
    @staticmethod
    def forward(ctx, sig, channels, depth):
        ctx.args = (channels, depth)
        return binding.sig_invert(sig.contiguous(), channels, depth)

    @staticmethod
    def backward(ctx, grad_out):
        # only used on signatures (group-like elements), where the inverse is a signed permutation of the scalars
        # (section 5.4) and therefore its own transpose
        channels, depth = ctx.args
        return binding.sig_invert(grad_out.contiguous(), channels, depth), None, None


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
