"""Truncated signature transform of batched piecewise-linear paths on AMD MI355X.

`sig_forward` and the size helpers below are thin bindings of the C ABI in
`include/sig.h`; the shared library is loaded on first use.
"""
from .binding import (  # noqa: F401
    SIG_F32,
    SIG_F64,
    SIG_MAX_DEPTH,
    SIG_OK,
    SIG_ERR_HIP,
    SIG_ERR_INVALID_ARG,
    SIG_ERR_OVERFLOW,
    SIG_ERR_TOO_LARGE,
    SIG_ERR_UNSUPPORTED,
    SIG_VARIANT_AUTO,
    SIG_VARIANT_GENERIC,
    SIG_VARIANT_MFMA,
    SIG_VARIANT_MFMA_SHARD,
    SIG_VARIANT_MFMA_STREAM,
    SIG_VARIANT_ROW_STREAM,
    SIG_VARIANT_WIDE,
    SIG_VARIANT_DEPTH2,
    SIG_VARIANT_SMALL,
    SIG_VARIANT_TREE,
    SigError,
    load_library,
    sig_backward,
    sig_backward_chunked,
    sig_backward_chunked_workspace_bytes,
    sig_backward_chunks_hint,
    sig_backward_workspace_bytes,
    sig_combine,
    sig_combine_backward,
    sig_combine_backward_workspace_bytes,
    sig_combine_grouped,
    sig_combine_grouped_backward,
    sig_combine_grouped_backward_workspace_bytes,
    sig_combine_many,
    sig_combine_strided,
    sig_invert,
    sig_log,
    sig_log_backward,
    sig_log_backward_workspace_bytes,
    sig_logsignature,
    sig_logsignature_channels,
    sig_lyndon_gather,
    sig_lyndon_scatter,
    sig_lyndon_indices,
    sig_signature,
    sig_forward,
    sig_forward_chunked,
    sig_forward_chunked_workspace_bytes,
    sig_forward_chunks_hint,
    sig_forward_chunked_static,
    sig_forward_chunked_static_max_bytes,
    sig_forward_raw,
    current_stream_handle,
    sig_fused_fmas,
    sig_output_elems,
    sig_signature_channels,
    sig_status_string,
    sig_variant_name,
)


def signature(path, depth, stream=False, basepoint=False, inverse=False, initial=None):
    """Differentiable signature (torch.autograd); see `autograd.signature`."""
    from .autograd import signature as _signature
    return _signature(path, depth, stream, basepoint, inverse, initial)


def signature_combine(sig1, sig2, channels, depth):
    """Differentiable group product of two batches of signatures; see `autograd.signature_combine`."""
    from .autograd import signature_combine as _combine
    return _combine(sig1, sig2, channels, depth)


def multi_signature_combine(sigs, channels, depth):
    """Differentiable ordered product of a list of batches of signatures; see `autograd.multi_signature_combine`."""
    from .autograd import multi_signature_combine as _combine
    return _combine(sigs, channels, depth)


def logsignature(path, depth, stream=False, basepoint=False, inverse=False, mode="words"):
    """Differentiable logsignature (torch.autograd); see `autograd.logsignature`."""
    from .autograd import logsignature as _logsignature
    return _logsignature(path, depth, stream, basepoint, inverse, mode)


def signature_to_logsignature(sig, channels, depth, mode="words"):
    """Differentiable logsignature of given signatures; see `autograd.signature_to_logsignature`."""
    from .autograd import signature_to_logsignature as _s2l
    return _s2l(sig, channels, depth, mode)


def __getattr__(name):
    if name == "Path":   # needs torch, so it is imported on first use
        from .path import Path
        return Path
    raise AttributeError(name)
