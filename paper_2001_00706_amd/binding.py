"""Thin ctypes binding of `libsig.so` (the C ABI declared in `include/sig.h`).

Argument marshalling only: every step of the signature computation runs in the HIP
kernels.  PyTorch is used for device memory and for the current HIP stream, nothing else.
There is no CPU fallback: if the library is missing or the tensor is not on a GPU the
call raises.
"""
from __future__ import annotations

import ctypes
import os
import threading

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(PKG_DIR, "libsig.so")

SIG_OK, SIG_ERR_INVALID_ARG, SIG_ERR_UNSUPPORTED, SIG_ERR_OVERFLOW, SIG_ERR_HIP, SIG_ERR_TOO_LARGE = range(6)
SIG_F32, SIG_F64 = 0, 1
SIG_VARIANT_AUTO, SIG_VARIANT_GENERIC, SIG_VARIANT_MFMA, SIG_VARIANT_MFMA_SHARD, SIG_VARIANT_SMALL = 0, 1, 2, 3, 4
SIG_VARIANT_TREE = 5
SIG_VARIANT_MFMA_STREAM = 6
SIG_VARIANT_ROW_STREAM = 7
SIG_VARIANT_WIDE = 8
SIG_VARIANT_DEPTH2 = 9
SIG_MAX_DEPTH = 32

# every symbol include/sig.h declares
EXPORTED_SYMBOLS = (
    "sig_signature_channels",
    "sig_output_elems",
    "sig_fused_fmas",
    "sig_forward",
    "sig_forward_variant",
    "sig_forward_chunked",
    "sig_forward_chunked_workspace_bytes",
    "sig_forward_chunks_hint",
    "sig_forward_chunked_static",
    "sig_forward_chunked_static_max_bytes",
    "sig_combine",
    "sig_backward",
    "sig_backward_chunked",
    "sig_backward_chunked_workspace_bytes",
    "sig_backward_chunks_hint",
    "sig_combine_strided",
    "sig_combine_backward",
    "sig_combine_backward_workspace_bytes",
    "sig_combine_grouped",
    "sig_combine_grouped_backward",
    "sig_combine_grouped_backward_workspace_bytes",
    "sig_combine_many",
    "sig_combine_many_workspace_bytes",
    "sig_invert",
    "sig_log",
    "sig_logsignature_channels",
    "sig_lyndon_indices",
    "sig_lyndon_gather",
    "sig_lyndon_scatter",
    "sig_log_backward",
    "sig_log_backward_workspace_bytes",
    "sig_signature",
    "sig_backward_workspace_bytes",
    "sig_variant_name",
    "sig_status_string",
)

_lock = threading.Lock()
_lib = None


class SigError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"libsig: {text} (status {status})")
        self.status = status


class _NoGuard:
    """Stands in for `torch.cuda.device(...)` when the tensor's device is the current one already."""

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        return False


_NO_GUARD = _NoGuard()


def _on_device(device):
    """A context in which `device` is the current HIP device (the library launches on the current device): a guard only
    when it is not already; entering `torch.cuda.device` costs about 2 us per call."""
    import torch

    index = device.index
    if index is None or index == torch.cuda.current_device():
        return _NO_GUARD
    return torch.cuda.device(device)


def current_stream_handle() -> int:
    """The raw handle of torch's current stream on the current device, for callers of the `*_raw` functions."""
    return _current_stream()


def _current_stream() -> int:
    """The raw handle of torch's current stream on the current device (`torch.cuda.current_stream().cuda_stream` builds a
    Stream object on every call: 2.7 us against 0.1)."""
    import torch

    try:
        return torch._C._cuda_getCurrentRawStream(torch.cuda.current_device())
    except AttributeError:   # a torch without the raw accessor
        return torch.cuda.current_stream().cuda_stream



def load_library() -> ctypes.CDLL:
    """Loads `libsig.so`; raises if it has not been built (`__graft_entry__.build()`)."""
    global _lib
    if _lib is not None:
        return _lib
    with _lock:
        if _lib is not None:
            return _lib
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -c 'import __graft_entry__ as g; g.build()'`")
        # torch ships its own HIP runtime: it has to be in the process before libsig.so is, so that the library's
        # calls and the streams and buffers torch hands over belong to one and the same runtime
        import torch  # noqa: F401
        lib = ctypes.CDLL(LIB_PATH)
        i64, i32, vp = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p
        lib.sig_signature_channels.restype = i64
        lib.sig_signature_channels.argtypes = [i32, i32]
        lib.sig_output_elems.restype = i64
        lib.sig_output_elems.argtypes = [i64, i64, i32, i32, i32, i32]
        lib.sig_fused_fmas.restype = i64
        lib.sig_fused_fmas.argtypes = [i32, i32]
        lib.sig_forward.restype = i32
        lib.sig_forward.argtypes = [vp, i64, i64, i32, i32, i32, i32, i32, vp, vp]
        lib.sig_forward_variant.restype = i32
        lib.sig_forward_variant.argtypes = [vp, i64, i64, i32, i32, i32, i32, i32, vp, vp, i32]
        lib.sig_forward_chunked.restype = i32
        lib.sig_forward_chunked.argtypes = [vp, i64, i64, i32, i32, i32, vp, i32, i32, vp, vp, i64, vp]
        lib.sig_forward_chunked_workspace_bytes.restype = i64
        lib.sig_forward_chunked_workspace_bytes.argtypes = [i64, i64, i32, i32, i32, i32, i32]
        lib.sig_forward_chunks_hint.restype = i32
        lib.sig_forward_chunks_hint.argtypes = [i64, i64, i32, i32, i32, i32]
        lib.sig_forward_chunked_static.restype = i32
        lib.sig_forward_chunked_static.argtypes = [vp, i64, i64, i32, i32, i32, vp, i32, i32, vp, vp]
        lib.sig_forward_chunked_static_max_bytes.restype = i64
        lib.sig_forward_chunked_static_max_bytes.argtypes = []
        lib.sig_combine.restype = i32
        lib.sig_combine.argtypes = [vp, vp, i64, i32, i32, i32, vp, vp]
        lib.sig_backward.restype = i32
        lib.sig_backward.argtypes = [vp, vp, vp, i64, i64, i32, i32, i32, i32, vp, i32, vp, vp, vp, i64, vp]
        lib.sig_backward_chunked.restype = i32
        lib.sig_backward_chunked.argtypes = [vp, vp, i64, i64, i32, i32, i32, vp, i32, i32, vp, vp, vp, i64, vp]
        lib.sig_backward_chunked_workspace_bytes.restype = i64
        lib.sig_backward_chunked_workspace_bytes.argtypes = [i64, i64, i32, i32, i32, i32, i32]
        lib.sig_backward_chunks_hint.restype = i32
        lib.sig_backward_chunks_hint.argtypes = [i64, i64, i32, i32, i32, i32]
        lib.sig_combine_backward.restype = i32
        lib.sig_combine_backward.argtypes = [vp, vp, vp, i64, i32, i32, i32, vp, vp, vp, i64, vp]
        lib.sig_combine_backward_workspace_bytes.restype = i64
        lib.sig_combine_backward_workspace_bytes.argtypes = [i64, i32, i32, i32]
        lib.sig_combine_grouped.restype = i32
        lib.sig_combine_grouped.argtypes = [vp, vp, i64, i64, i32, i32, i32, vp, vp]
        lib.sig_combine_grouped_backward.restype = i32
        lib.sig_combine_grouped_backward.argtypes = [vp, vp, vp, i64, i64, i32, i32, i32, vp, vp, vp, i64, vp]
        lib.sig_combine_grouped_backward_workspace_bytes.restype = i64
        lib.sig_combine_grouped_backward_workspace_bytes.argtypes = [i64, i64, i32, i32, i32]
        lib.sig_combine_many.restype = i32
        lib.sig_combine_many.argtypes = [vp, i64, i64, i32, i32, i32, vp, vp, i64, vp]
        lib.sig_combine_many_workspace_bytes.restype = i64
        lib.sig_combine_many_workspace_bytes.argtypes = [i64, i64, i32, i32, i32]
        lib.sig_combine_strided.restype = i32
        lib.sig_combine_strided.argtypes = [vp, i64, vp, i64, i64, i32, i32, i32, vp, i64, vp]
        lib.sig_log.restype = i32
        lib.sig_log.argtypes = [vp, i64, i32, i32, i32, vp, vp]
        lib.sig_logsignature_channels.restype = i64
        lib.sig_logsignature_channels.argtypes = [i32, i32]
        lib.sig_lyndon_indices.restype = i32
        lib.sig_lyndon_indices.argtypes = [i32, i32, ctypes.POINTER(i64), i64]
        lib.sig_lyndon_scatter.restype = i32
        lib.sig_lyndon_scatter.argtypes = [vp, i64, i32, i32, vp, i64, i32, vp, vp]
        lib.sig_log_backward.restype = i32
        lib.sig_log_backward.argtypes = [vp, vp, i64, i32, i32, i32, vp, vp, i64, vp]
        lib.sig_log_backward_workspace_bytes.restype = i64
        lib.sig_log_backward_workspace_bytes.argtypes = [i64, i32, i32, i32]
        lib.sig_lyndon_gather.restype = i32
        lib.sig_lyndon_gather.argtypes = [vp, i64, i32, i32, vp, i64, i32, vp, vp]
        lib.sig_invert.restype = i32
        lib.sig_invert.argtypes = [vp, i64, i32, i32, i32, vp, vp]
        lib.sig_signature.restype = i32
        lib.sig_signature.argtypes = [vp, i64, i64, i32, i32, i32, i32, vp, vp, i32, i32, vp, vp]
        lib.sig_backward_workspace_bytes.restype = i64
        lib.sig_backward_workspace_bytes.argtypes = [i64, i64, i32, i32, i32, i32, i32]
        lib.sig_variant_name.restype = ctypes.c_char_p
        lib.sig_variant_name.argtypes = [i64, i64, i32, i32, i32, i32, i32, i32]
        lib.sig_status_string.restype = ctypes.c_char_p
        lib.sig_status_string.argtypes = [i32]
        _lib = lib
        return lib


def sig_status_string(status: int) -> str:
    return load_library().sig_status_string(int(status)).decode()


def sig_signature_channels(d: int, N: int) -> int:
    return int(load_library().sig_signature_channels(d, N))


def sig_output_elems(B: int, L: int, d: int, N: int, stream: bool, basepoint: bool) -> int:
    return int(load_library().sig_output_elems(B, L, d, N, int(stream), int(basepoint)))


def sig_fused_fmas(d: int, N: int) -> int:
    return int(load_library().sig_fused_fmas(d, N))


def sig_variant_name(B: int, L: int, d: int, N: int, stream: bool, basepoint: bool,
                     dtype: int = SIG_F32, variant: int = SIG_VARIANT_AUTO) -> str:
    return load_library().sig_variant_name(B, L, d, N, int(stream), int(basepoint), dtype, variant).decode()


def sig_forward_raw(path_ptr: int, B: int, L: int, d: int, N: int, stream: int, basepoint: int,
                    dtype: int, out_ptr: int, hip_stream: int, variant: int = SIG_VARIANT_AUTO) -> int:
    """The C call itself, on raw device addresses; returns the status code."""
    lib = load_library()
    if variant == SIG_VARIANT_AUTO:
        return int(lib.sig_forward(path_ptr, B, L, d, N, stream, basepoint, dtype, out_ptr, hip_stream))
    return int(lib.sig_forward_variant(path_ptr, B, L, d, N, stream, basepoint, dtype, out_ptr,
                                       hip_stream, variant))


def sig_forward(path, N: int, stream: bool = False, basepoint: bool = False, out=None,
                variant: int = SIG_VARIANT_AUTO):
    """Signatures of a batch of paths held in a CUDA/HIP torch tensor.

    path: `[B, L, d]` contiguous float32 or float64 tensor on the GPU.
    Returns (and, if `out` is given, fills) a tensor `[B, S]`, or `[B, n_inc, S]` in stream
    mode.  The work is enqueued on torch's current stream and not waited for.
    """
    import torch

    if not isinstance(path, torch.Tensor) or not path.is_cuda:
        raise TypeError("sig_forward needs a torch tensor on the GPU (there is no CPU path)")
    if path.dim() != 3:
        raise ValueError("path must have shape [B, L, d]")
    if path.dtype == torch.float32:
        dtype = SIG_F32
    elif path.dtype == torch.float64:
        dtype = SIG_F64
    else:
        raise TypeError("path must be float32 or float64")
    if not path.is_contiguous():
        raise ValueError("path must be contiguous")
    B, L, d = path.shape
    n_elems = sig_output_elems(B, L, d, N, stream, basepoint)
    if n_elems < 0:
        # let the library name the reason
        status = sig_forward_raw(path.data_ptr(), B, L, d, N, int(stream), int(basepoint), dtype, 0, 0, variant)
        raise SigError(status, sig_status_string(status))
    S = sig_signature_channels(d, N)
    n_inc = L if basepoint else L - 1
    shape = (B, n_inc, S) if stream else (B, S)
    if out is None:
        out = torch.empty(shape, dtype=path.dtype, device=path.device)
    else:
        if out.dtype != path.dtype or out.device != path.device or tuple(out.shape) != shape \
                or not out.is_contiguous():
            raise ValueError(f"out must be a contiguous {path.dtype} tensor of shape {shape} on {path.device}")
    with _on_device(path.device):
        hip_stream = _current_stream()
        status = sig_forward_raw(path.data_ptr(), B, L, d, N, int(stream), int(basepoint), dtype,
                                 out.data_ptr(), hip_stream, variant)
    if status != SIG_OK:
        raise SigError(status, sig_status_string(status))
    return out


def sig_combine(a, b, d: int, N: int, out=None):
    """Group product a [x] b of two batches of signatures `[B, S]` held in GPU torch tensors
    (the signature of two adjacent intervals joined, by Chen's identity)."""
    import torch

    for t in (a, b):
        if not isinstance(t, torch.Tensor) or not t.is_cuda:
            raise TypeError("sig_combine needs torch tensors on the GPU (there is no CPU path)")
    if a.dtype != b.dtype or a.device != b.device or a.shape != b.shape or a.dim() != 2:
        raise ValueError("a and b must be [B, S] tensors of the same dtype, shape and device")
    if a.dtype == torch.float32:
        dtype = SIG_F32
    elif a.dtype == torch.float64:
        dtype = SIG_F64
    else:
        raise TypeError("signatures must be float32 or float64")
    S = sig_signature_channels(d, N)
    if S < 0 or a.shape[1] != S:
        raise ValueError(f"signatures of d={d}, N={N} have {S} channels, got {a.shape[1]}")
    if not (a.is_contiguous() and b.is_contiguous()):
        raise ValueError("a and b must be contiguous")
    if out is None:
        out = torch.empty_like(a)
    elif out.dtype != a.dtype or out.device != a.device or out.shape != a.shape or not out.is_contiguous():
        raise ValueError("out must match a")
    with _on_device(a.device):
        status = int(load_library().sig_combine(a.data_ptr(), b.data_ptr(), a.shape[0], d, N, dtype,
                                                out.data_ptr(), _current_stream()))
    if status != SIG_OK:
        raise SigError(status, sig_status_string(status))
    return out


def sig_backward_workspace_bytes(B: int, L: int, d: int, N: int, stream: bool, basepoint: bool,
                                 dtype: int = SIG_F32) -> int:
    return int(load_library().sig_backward_workspace_bytes(B, L, d, N, int(stream), int(basepoint), dtype))


def _dtype_of(t):
    import torch
    if t.dtype == torch.float32:
        return SIG_F32
    if t.dtype == torch.float64:
        return SIG_F64
    raise TypeError("tensors must be float32 or float64")


def _check_gpu(name, *tensors):
    import torch
    for t in tensors:
        if not isinstance(t, torch.Tensor) or not t.is_cuda:
            raise TypeError(f"{name} needs torch tensors on the GPU (there is no CPU path)")


def _basepoint_args(path, basepoint):
    """(flag, tensor or None) from False / True / a `[B, d]` tensor."""
    import torch
    if isinstance(basepoint, torch.Tensor):
        B, _, d = path.shape
        if basepoint.dtype != path.dtype or basepoint.device != path.device or tuple(basepoint.shape) != (B, d) \
                or not basepoint.is_contiguous():
            raise ValueError(f"basepoint must be a contiguous {path.dtype} tensor of shape {(B, d)} on {path.device}")
        return 1, basepoint
    return int(bool(basepoint)), None


def sig_backward(path, sig, grad_out, N: int, stream: bool = False, basepoint=False,
                 grad_path=None, workspace=None, grad_basepoint=None):
    """Gradient with respect to `path` of a loss whose gradient with respect to
    `sig = sig_forward(path, N, stream, basepoint)` is `grad_out`; all GPU torch tensors.

    Returns (and, if given, fills) `grad_path`, shaped like `path`.  `basepoint` may be a `[B, d]` tensor
    (then `sig` comes from `sig_signature`); `grad_basepoint`, if given, receives its gradient.
    `workspace` is a uint8 GPU tensor of at least `sig_backward_workspace_bytes(...)` bytes; one is
    allocated through torch when the call needs it and none is given.
    """
    import torch

    _check_gpu("sig_backward", path, sig, grad_out)
    if path.dim() != 3:
        raise ValueError("path must have shape [B, L, d]")
    dtype = _dtype_of(path)
    B, L, d = path.shape
    bp_flag, bp_value = _basepoint_args(path, basepoint)
    S = sig_signature_channels(d, N)
    n_inc = L if bp_flag else L - 1
    shape = (B, n_inc, S) if stream else (B, S)
    for name, t in (("sig", sig), ("grad_out", grad_out)):
        if t.dtype != path.dtype or t.device != path.device or tuple(t.shape) != shape or not t.is_contiguous():
            raise ValueError(f"{name} must be a contiguous {path.dtype} tensor of shape {shape} on {path.device}")
    if not path.is_contiguous():
        raise ValueError("path must be contiguous")
    if grad_path is None:
        grad_path = torch.empty_like(path)
    elif grad_path.dtype != path.dtype or grad_path.device != path.device or grad_path.shape != path.shape \
            or not grad_path.is_contiguous():
        raise ValueError("grad_path must match path")
    if grad_basepoint is not None and (grad_basepoint.dtype != path.dtype or grad_basepoint.device != path.device
                                       or tuple(grad_basepoint.shape) != (B, d) or not grad_basepoint.is_contiguous()):
        raise ValueError("grad_basepoint must be a contiguous [B, d] tensor like path")
    with _on_device(path.device):
        need = sig_backward_workspace_bytes(B, L, d, N, stream, bool(bp_flag), dtype)
        if need > 0 and workspace is None:
            workspace = torch.empty(need, dtype=torch.uint8, device=path.device)
        ws_ptr, ws_bytes = (workspace.data_ptr(), workspace.numel() * workspace.element_size()) \
            if workspace is not None else (0, 0)
        status = int(load_library().sig_backward(
            path.data_ptr(), sig.data_ptr(), grad_out.data_ptr(), B, L, d, N, int(stream), bp_flag,
            bp_value.data_ptr() if bp_value is not None else 0, dtype, grad_path.data_ptr(),
            grad_basepoint.data_ptr() if grad_basepoint is not None else 0,
            ws_ptr, ws_bytes, _current_stream()))
    if status != SIG_OK:
        raise SigError(status, sig_status_string(status))
    return grad_path


def sig_backward_chunked_workspace_bytes(B: int, L: int, d: int, N: int, basepoint: bool, chunks: int,
                                         dtype: int = SIG_F32) -> int:
    return int(load_library().sig_backward_chunked_workspace_bytes(B, L, d, N, int(bool(basepoint)), chunks, dtype))


def sig_backward_chunks_hint(B: int, L: int, d: int, N: int, basepoint: bool = False, dtype: int = SIG_F32) -> int:
    """The number of stretches `sig_backward_chunked` should be given for this shape; 1 where `sig_backward` is faster."""
    return int(load_library().sig_backward_chunks_hint(B, L, d, N, int(bool(basepoint)), dtype))


def sig_backward_chunked(path, grad_out, N: int, chunks: int, basepoint=False, grad_path=None, workspace=None,
                         grad_basepoint=None):
    """`sig_backward` in final mode with every path cut into at most `chunks` stretches that are walked back at the same
    time; the forward output is not needed.  `workspace` (uint8, GPU) is allocated through torch if not given."""
    import torch

    _check_gpu("sig_backward_chunked", path, grad_out)
    if path.dim() != 3 or not path.is_contiguous():
        raise ValueError("path must be a contiguous tensor of shape [B, L, d]")
    dtype = _dtype_of(path)
    B, L, d = path.shape
    bp_flag, bp_value = _basepoint_args(path, basepoint)
    S = sig_signature_channels(d, N)
    if grad_out.dtype != path.dtype or grad_out.device != path.device or tuple(grad_out.shape) != (B, S) \
            or not grad_out.is_contiguous():
        raise ValueError(f"grad_out must be a contiguous {path.dtype} tensor of shape {(B, S)} on {path.device}")
    if grad_path is None:
        grad_path = torch.empty_like(path)
    elif grad_path.dtype != path.dtype or grad_path.device != path.device or grad_path.shape != path.shape \
            or not grad_path.is_contiguous():
        raise ValueError("grad_path must match path")
    if grad_basepoint is not None and (grad_basepoint.dtype != path.dtype or grad_basepoint.device != path.device
                                       or tuple(grad_basepoint.shape) != (B, d) or not grad_basepoint.is_contiguous()):
        raise ValueError("grad_basepoint must be a contiguous [B, d] tensor like path")
    with _on_device(path.device):
        need = sig_backward_chunked_workspace_bytes(B, L, d, N, bool(bp_flag), chunks, dtype)
        if need > 0 and workspace is None:
            workspace = torch.empty(need, dtype=torch.uint8, device=path.device)
        ws_ptr, ws_bytes = (workspace.data_ptr(), workspace.numel() * workspace.element_size()) \
            if workspace is not None else (0, 0)
        status = int(load_library().sig_backward_chunked(
            path.data_ptr(), grad_out.data_ptr(), B, L, d, N, bp_flag,
            bp_value.data_ptr() if bp_value is not None else 0, chunks, dtype, grad_path.data_ptr(),
            grad_basepoint.data_ptr() if grad_basepoint is not None else 0, ws_ptr, ws_bytes, _current_stream()))
    if status != SIG_OK:
        raise SigError(status, sig_status_string(status))
    return grad_path


def sig_signature(path, N: int, stream: bool = False, basepoint=False, inverse: bool = False, initial=None, out=None):
    """`sig_forward` with every option of section 5.5: `basepoint` False / True / a `[B, d]` tensor,
    `initial` a `[B, S]` signature of the data that came before, `inverse` for the inverted signature."""
    import torch

    _check_gpu("sig_signature", path)
    if path.dim() != 3 or not path.is_contiguous():
        raise ValueError("path must be a contiguous tensor of shape [B, L, d]")
    dtype = _dtype_of(path)
    B, L, d = path.shape
    bp_flag, bp_value = _basepoint_args(path, basepoint)
    S = sig_signature_channels(d, N)
    n_inc = L if bp_flag else L - 1
    if sig_output_elems(B, L, d, N, stream, bool(bp_flag)) < 0:
        status = int(load_library().sig_signature(path.data_ptr(), B, L, d, N, int(stream), bp_flag, 0, 0, 0, dtype, 0, 0))
        raise SigError(status, sig_status_string(status))
    shape = (B, n_inc, S) if stream else (B, S)
    if initial is not None:
        _check_gpu("sig_signature", initial)
        if initial.dtype != path.dtype or initial.device != path.device or tuple(initial.shape) != (B, S) \
                or not initial.is_contiguous():
            raise ValueError(f"initial must be a contiguous {path.dtype} tensor of shape {(B, S)} on {path.device}")
    if out is None:
        out = torch.empty(shape, dtype=path.dtype, device=path.device)
    elif out.dtype != path.dtype or out.device != path.device or tuple(out.shape) != shape or not out.is_contiguous():
        raise ValueError(f"out must be a contiguous {path.dtype} tensor of shape {shape} on {path.device}")
    with _on_device(path.device):
        status = int(load_library().sig_signature(
            path.data_ptr(), B, L, d, N, int(stream), bp_flag, bp_value.data_ptr() if bp_value is not None else 0,
            initial.data_ptr() if initial is not None else 0, int(bool(inverse)), dtype, out.data_ptr(),
            _current_stream()))
    if status != SIG_OK:
        raise SigError(status, sig_status_string(status))
    return out


def sig_invert(sig, d: int, N: int, out=None):
    """Group inverses of signatures `[..., S]` (the signatures of the reversed paths); `out` may be `sig`."""
    import torch

    _check_gpu("sig_invert", sig)
    dtype = _dtype_of(sig)
    S = sig_signature_channels(d, N)
    if S < 0 or sig.shape[-1] != S or not sig.is_contiguous():
        raise ValueError(f"sig must be contiguous with {S} channels last")
    if out is None:
        out = torch.empty_like(sig)
    elif out.dtype != sig.dtype or out.device != sig.device or out.shape != sig.shape or not out.is_contiguous():
        raise ValueError("out must match sig")
    rows = sig.numel() // S if S > 0 else 0
    with _on_device(sig.device):
        status = int(load_library().sig_invert(sig.data_ptr(), rows, d, N, dtype, out.data_ptr(),
                                               _current_stream()))
    if status != SIG_OK:
        raise SigError(status, sig_status_string(status))
    return out


def sig_combine_strided(a, a_stride: int, b, b_stride: int, B: int, d: int, N: int, out, out_stride: int):
    """`out[p] = a[p] [x] b[p]` for p < B where signature p of each operand starts `p * stride` scalars
    after the tensor's first element (the tensors must be large enough for that; not checked beyond size)."""
    import torch

    _check_gpu("sig_combine_strided", a, b, out)
    dtype = _dtype_of(a)
    S = sig_signature_channels(d, N)
    for t, stride in ((a, a_stride), (b, b_stride), (out, out_stride)):
        if t.dtype != a.dtype or t.device != a.device or not t.is_contiguous():
            raise ValueError("a, b and out must be contiguous tensors of one dtype on one device")
        if B > 0 and (B - 1) * stride + S > t.numel():
            raise ValueError("an operand is too small for B signatures at this stride")
    with _on_device(a.device):
        status = int(load_library().sig_combine_strided(a.data_ptr(), a_stride, b.data_ptr(), b_stride, B, d, N, dtype,
                                                        out.data_ptr(), out_stride,
                                                        _current_stream()))
    if status != SIG_OK:
        raise SigError(status, sig_status_string(status))
    return out


def sig_logsignature_channels(d: int, N: int) -> int:
    return int(load_library().sig_logsignature_channels(d, N))


def sig_lyndon_indices(d: int, N: int):
    """Offsets of the Lyndon-word coefficients inside a flat depth-N element, as a Python list (host side)."""
    n = sig_logsignature_channels(d, N)
    if n < 0:
        raise SigError(SIG_ERR_INVALID_ARG, "bad d or N")
    buf = (ctypes.c_int64 * max(n, 1))()
    status = int(load_library().sig_lyndon_indices(d, N, buf, n))
    if status != SIG_OK:
        raise SigError(status, sig_status_string(status))
    return list(buf[:n])


def sig_log(sig, d: int, N: int, out=None):
    """Logarithm in the tensor algebra of signatures `[..., S]`; same shape, every word kept."""
    import torch

    _check_gpu("sig_log", sig)
    dtype = _dtype_of(sig)
    S = sig_signature_channels(d, N)
    if S < 0 or sig.shape[-1] != S or not sig.is_contiguous():
        raise ValueError(f"sig must be contiguous with {S} channels last")
    if out is None:
        out = torch.empty_like(sig)
    elif out.dtype != sig.dtype or out.device != sig.device or out.shape != sig.shape or not out.is_contiguous() \
            or out.data_ptr() == sig.data_ptr():
        raise ValueError("out must match sig and be a different tensor")
    rows = sig.numel() // S
    with _on_device(sig.device):
        status = int(load_library().sig_log(sig.data_ptr(), rows, d, N, dtype, out.data_ptr(),
                                            _current_stream()))
    if status != SIG_OK:
        raise SigError(status, sig_status_string(status))
    return out


_lyndon_tables = {}


def _lyndon_table(d: int, N: int, device):
    """The Lyndon index table on `device`, built once per (d, N, device)."""
    import torch
    key = (d, N, str(device))
    with _lock:
        t = _lyndon_tables.get(key)
    if t is None:
        t = torch.tensor(sig_lyndon_indices(d, N), dtype=torch.int64, device=device)
        with _lock:
            _lyndon_tables[key] = t
    return t


def sig_lyndon_gather(log_sig, d: int, N: int, out=None):
    """Coefficients of the Lyndon words of logarithms `[..., S]` -> `[..., w(d, N)]`."""
    import torch

    _check_gpu("sig_lyndon_gather", log_sig)
    dtype = _dtype_of(log_sig)
    S = sig_signature_channels(d, N)
    if S < 0 or log_sig.shape[-1] != S or not log_sig.is_contiguous():
        raise ValueError(f"log_sig must be contiguous with {S} channels last")
    table = _lyndon_table(d, N, log_sig.device)
    n = table.numel()
    shape = tuple(log_sig.shape[:-1]) + (n,)
    if out is None:
        out = torch.empty(shape, dtype=log_sig.dtype, device=log_sig.device)
    elif out.dtype != log_sig.dtype or out.device != log_sig.device or tuple(out.shape) != shape or not out.is_contiguous():
        raise ValueError(f"out must be a contiguous tensor of shape {shape}")
    rows = log_sig.numel() // S
    with _on_device(log_sig.device):
        status = int(load_library().sig_lyndon_gather(log_sig.data_ptr(), rows, d, N, table.data_ptr(), n, dtype,
                                                      out.data_ptr(), _current_stream()))
    if status != SIG_OK:
        raise SigError(status, sig_status_string(status))
    return out


def sig_lyndon_scatter(grad_logsig, d: int, N: int, out=None):
    """Transpose of `sig_lyndon_gather`: `[..., w(d, N)]` -> `[..., S]`, zero at every word that is not a Lyndon word."""
    import torch

    _check_gpu("sig_lyndon_scatter", grad_logsig)
    dtype = _dtype_of(grad_logsig)
    S = sig_signature_channels(d, N)
    table = _lyndon_table(d, N, grad_logsig.device)
    n = table.numel()
    if S < 0 or grad_logsig.shape[-1] != n or not grad_logsig.is_contiguous():
        raise ValueError(f"grad_logsig must be contiguous with {n} channels last")
    shape = tuple(grad_logsig.shape[:-1]) + (S,)
    if out is None:
        out = torch.empty(shape, dtype=grad_logsig.dtype, device=grad_logsig.device)
    elif out.dtype != grad_logsig.dtype or out.device != grad_logsig.device or tuple(out.shape) != shape \
            or not out.is_contiguous():
        raise ValueError(f"out must be a contiguous tensor of shape {shape}")
    rows = out.numel() // S
    with _on_device(out.device):
        status = int(load_library().sig_lyndon_scatter(grad_logsig.data_ptr(), rows, d, N, table.data_ptr(), n, dtype,
                                                       out.data_ptr(), _current_stream()))
    if status != SIG_OK:
        raise SigError(status, sig_status_string(status))
    return out


def sig_log_backward_workspace_bytes(rows: int, d: int, N: int, dtype: int = SIG_F32) -> int:
    return int(load_library().sig_log_backward_workspace_bytes(rows, d, N, dtype))


def sig_log_backward(sig, grad_log, d: int, N: int, out=None, workspace=None):
    """Gradient with respect to signatures `sig` `[..., S]` of a loss whose gradient with respect to
    `sig_log(sig, d, N)` is `grad_log`; `workspace` (uint8, GPU) is allocated through torch if not given."""
    import torch

    _check_gpu("sig_log_backward", sig)
    dtype = _dtype_of(sig)
    S = sig_signature_channels(d, N)
    if S < 0 or sig.shape[-1] != S or not sig.is_contiguous():
        raise ValueError(f"sig must be contiguous with {S} channels last")
    if grad_log.dtype != sig.dtype or grad_log.device != sig.device or grad_log.shape != sig.shape \
            or not grad_log.is_contiguous():
        raise ValueError("grad_log must match sig")
    if out is None:
        out = torch.empty_like(sig)
    elif out.dtype != sig.dtype or out.device != sig.device or out.shape != sig.shape or not out.is_contiguous() \
            or out.data_ptr() in (sig.data_ptr(), grad_log.data_ptr()):
        raise ValueError("out must match sig and be a different tensor")
    rows = sig.numel() // S
    lib = load_library()
    with _on_device(sig.device):
        need = int(lib.sig_log_backward_workspace_bytes(rows, d, N, dtype))
        if need < 0:
            raise SigError(SIG_ERR_UNSUPPORTED, "no workspace size for this shape")
        if workspace is None and need > 0:
            workspace = torch.empty(need, dtype=torch.uint8, device=sig.device)
        ws_ptr, ws_bytes = (workspace.data_ptr(), workspace.numel() * workspace.element_size()) \
            if workspace is not None else (0, 0)
        status = int(lib.sig_log_backward(sig.data_ptr(), grad_log.data_ptr(), rows, d, N, dtype, out.data_ptr(), ws_ptr,
                                          ws_bytes, _current_stream()))
    if status != SIG_OK:
        raise SigError(status, sig_status_string(status))
    return out


def sig_logsignature(path, N: int, stream: bool = False, basepoint=False, inverse: bool = False, mode: str = "words"):
    """Logsignature of a batch of paths (sections 2.3, 4.3): `sig_signature`, then `sig_log`, then, for
    mode "words", the coefficients of the Lyndon words (mode "expand" keeps every word)."""
    if mode not in ("words", "expand"):
        raise ValueError('mode must be "words" or "expand"')
    d = path.shape[2]
    full = sig_log(sig_signature(path, N, stream=stream, basepoint=basepoint, inverse=inverse), d, N)
    return full if mode == "expand" else sig_lyndon_gather(full, d, N)


def sig_forward_chunked_workspace_bytes(B: int, L: int, d: int, N: int, basepoint: bool, chunks: int,
                                        dtype: int = SIG_F32) -> int:
    return int(load_library().sig_forward_chunked_workspace_bytes(B, L, d, N, int(bool(basepoint)), chunks, dtype))


def sig_forward_chunks_hint(B: int, L: int, d: int, N: int, basepoint: bool = False, dtype: int = SIG_F32) -> int:
    """The number of chunks `sig_forward_chunked` should be given for this shape; 1 where `sig_forward` is faster."""
    return int(load_library().sig_forward_chunks_hint(B, L, d, N, int(bool(basepoint)), dtype))


def sig_forward_chunked(path, N: int, chunks: int, basepoint=False, out=None, workspace=None):
    """`sig_forward` (final mode) with every path cut into `chunks` stretches (a power of two) that are scanned
    in parallel and joined by group products; `workspace` (uint8, GPU) is allocated through torch if not given."""
    import torch

    _check_gpu("sig_forward_chunked", path)
    if path.dim() != 3 or not path.is_contiguous():
        raise ValueError("path must be a contiguous tensor of shape [B, L, d]")
    dtype = _dtype_of(path)
    B, L, d = path.shape
    bp_flag, bp_value = _basepoint_args(path, basepoint)
    S = sig_signature_channels(d, N)
    need = sig_forward_chunked_workspace_bytes(B, L, d, N, bool(bp_flag), chunks, dtype)
    if need < 0:
        status = int(load_library().sig_forward_chunked(path.data_ptr(), B, L, d, N, bp_flag, 0, chunks, dtype, 0, 0, 0, 0))
        raise SigError(status, sig_status_string(status))
    if out is None:
        out = torch.empty((B, S), dtype=path.dtype, device=path.device)
    elif out.dtype != path.dtype or out.device != path.device or tuple(out.shape) != (B, S) or not out.is_contiguous():
        raise ValueError(f"out must be a contiguous {path.dtype} tensor of shape {(B, S)} on {path.device}")
    with _on_device(path.device):
        if workspace is None:
            workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=path.device)
        status = int(load_library().sig_forward_chunked(
            path.data_ptr(), B, L, d, N, bp_flag, bp_value.data_ptr() if bp_value is not None else 0, chunks, dtype,
            out.data_ptr(), workspace.data_ptr(), workspace.numel() * workspace.element_size(),
            _current_stream()))
    if status != SIG_OK:
        raise SigError(status, sig_status_string(status))
    return out


def sig_forward_chunked_static_max_bytes() -> int:
    return int(load_library().sig_forward_chunked_static_max_bytes())


def sig_forward_chunked_static(path, N: int, chunks: int, basepoint=False, out=None):
    """`sig_forward_chunked` on the library's own fixed scratch array: nothing is allocated by the call itself when
    `out` is given (without it the result tensor comes from torch).  Raises `SigError` with `SIG_ERR_TOO_LARGE` when
    the request needs more than `sig_forward_chunked_static_max_bytes()`."""
    import torch

    _check_gpu("sig_forward_chunked_static", path)
    if path.dim() != 3 or not path.is_contiguous():
        raise ValueError("path must be a contiguous tensor of shape [B, L, d]")
    dtype = _dtype_of(path)
    B, L, d = path.shape
    bp_flag, bp_value = _basepoint_args(path, basepoint)
    S = sig_signature_channels(d, N)
    if S < 0:
        raise SigError(SIG_ERR_INVALID_ARG, "bad d or N")
    if out is None:
        out = torch.empty((B, S), dtype=path.dtype, device=path.device)
    elif out.dtype != path.dtype or out.device != path.device or tuple(out.shape) != (B, S) or not out.is_contiguous():
        raise ValueError(f"out must be a contiguous {path.dtype} tensor of shape {(B, S)} on {path.device}")
    with _on_device(path.device):
        status = int(load_library().sig_forward_chunked_static(
            path.data_ptr(), B, L, d, N, bp_flag, bp_value.data_ptr() if bp_value is not None else 0, chunks, dtype,
            out.data_ptr(), _current_stream()))
    if status != SIG_OK:
        raise SigError(status, sig_status_string(status))
    return out


def sig_combine_many(sigs, d: int, N: int, out=None, workspace=None):
    """Ordered group product of the `n` signatures of every batch row of `sigs` `[B, n, S]` -> `[B, S]`."""
    import torch

    _check_gpu("sig_combine_many", sigs)
    dtype = _dtype_of(sigs)
    S = sig_signature_channels(d, N)
    if sigs.dim() != 3 or sigs.shape[2] != S or sigs.shape[1] < 1 or not sigs.is_contiguous():
        raise ValueError(f"sigs must be a contiguous [B, n, {S}] tensor with n >= 1")
    B, n, _ = sigs.shape
    if out is None:
        out = torch.empty((B, S), dtype=sigs.dtype, device=sigs.device)
    elif out.dtype != sigs.dtype or out.device != sigs.device or tuple(out.shape) != (B, S) or not out.is_contiguous():
        raise ValueError(f"out must be a contiguous tensor of shape {(B, S)} like sigs")
    lib = load_library()
    with _on_device(sigs.device):
        need = int(lib.sig_combine_many_workspace_bytes(B, n, d, N, dtype))
        if need > 0 and workspace is None:
            workspace = torch.empty(need, dtype=torch.uint8, device=sigs.device)
        ws_ptr, ws_bytes = (workspace.data_ptr(), workspace.numel() * workspace.element_size()) \
            if workspace is not None else (0, 0)
        status = int(lib.sig_combine_many(sigs.data_ptr(), B, n, d, N, dtype, out.data_ptr(), ws_ptr, ws_bytes,
                                          _current_stream()))
    if status != SIG_OK:
        raise SigError(status, sig_status_string(status))
    return out


def sig_combine_backward_workspace_bytes(B: int, d: int, N: int, dtype: int = SIG_F32) -> int:
    return int(load_library().sig_combine_backward_workspace_bytes(B, d, N, dtype))


def sig_combine_backward(a, b, grad_out, d: int, N: int, grad_a=None, grad_b=None, workspace=None):
    """Gradients `(grad_a, grad_b)` of a loss with respect to the factors of `sig_combine(a, b, d, N)`, given its
    gradient `grad_out` with respect to the product; all `[B, S]`.  `workspace` (uint8, GPU) is allocated through
    torch if not given."""
    import torch

    _check_gpu("sig_combine_backward", a)
    dtype = _dtype_of(a)
    S = sig_signature_channels(d, N)
    if S < 0 or a.dim() != 2 or a.shape[1] != S:
        raise ValueError(f"signatures of d={d}, N={N} are [B, {S}] tensors")
    for t in (b, grad_out):
        if not isinstance(t, torch.Tensor) or t.dtype != a.dtype or t.device != a.device or t.shape != a.shape:
            raise ValueError("a, b and grad_out must agree in dtype, shape and device")
    if not (a.is_contiguous() and b.is_contiguous() and grad_out.is_contiguous()):
        raise ValueError("a, b and grad_out must be contiguous")
    outs = []
    for t in (grad_a, grad_b):
        if t is None:
            t = torch.empty_like(a)
        elif t.dtype != a.dtype or t.device != a.device or t.shape != a.shape or not t.is_contiguous():
            raise ValueError("grad_a and grad_b must match a")
        outs.append(t)
    lib = load_library()
    with _on_device(a.device):
        need = int(lib.sig_combine_backward_workspace_bytes(a.shape[0], d, N, dtype))
        if need < 0:
            raise SigError(SIG_ERR_UNSUPPORTED, "no workspace size for this shape")
        if workspace is None and need > 0:
            workspace = torch.empty(need, dtype=torch.uint8, device=a.device)
        ws_ptr, ws_bytes = (workspace.data_ptr(), workspace.numel() * workspace.element_size()) \
            if workspace is not None else (0, 0)
        status = int(lib.sig_combine_backward(a.data_ptr(), b.data_ptr(), grad_out.data_ptr(), a.shape[0], d, N, dtype,
                                              outs[0].data_ptr(), outs[1].data_ptr(), ws_ptr, ws_bytes,
                                              _current_stream()))
    if status != SIG_OK:
        raise SigError(status, sig_status_string(status))
    return outs[0], outs[1]


def _check_grouped(name, a, sigs, d, N):
    import torch

    _check_gpu(name, a)
    S = sig_signature_channels(d, N)
    if S < 0 or a.dim() != 2 or a.shape[1] != S:
        raise ValueError(f"signatures of d={d}, N={N} are [B, {S}] tensors")
    if not isinstance(sigs, torch.Tensor) or sigs.dtype != a.dtype or sigs.device != a.device or sigs.dim() != 3 or \
            sigs.shape[0] != a.shape[0] or sigs.shape[2] != S or sigs.shape[1] < 1:
        raise ValueError(f"sigs must be a [B, group, {S}] tensor of a's dtype on a's device")
    if not (a.is_contiguous() and sigs.is_contiguous()):
        raise ValueError("a and sigs must be contiguous")
    return S


def sig_combine_grouped(a, sigs, d: int, N: int, out=None):
    """`out[b, s] = a[b] [x] sigs[b, s]`: one left factor `[B, S]` for a group of right factors `[B, group, S]`."""
    import torch

    _check_grouped("sig_combine_grouped", a, sigs, d, N)
    if out is None:
        out = torch.empty_like(sigs)
    elif out.dtype != sigs.dtype or out.device != sigs.device or out.shape != sigs.shape or not out.is_contiguous():
        raise ValueError("out must match sigs")
    with _on_device(a.device):
        status = int(load_library().sig_combine_grouped(a.data_ptr(), sigs.data_ptr(), sigs.shape[0], sigs.shape[1], d, N,
                                                        _dtype_of(a), out.data_ptr(), _current_stream()))
    if status != SIG_OK:
        raise SigError(status, sig_status_string(status))
    return out


def sig_combine_grouped_backward_workspace_bytes(B: int, group: int, d: int, N: int, dtype: int = SIG_F32) -> int:
    return int(load_library().sig_combine_grouped_backward_workspace_bytes(B, group, d, N, dtype))


def sig_combine_grouped_backward(a, sigs, grad_out, d: int, N: int, grad_a=None, grad_sigs=None, workspace=None):
    """Gradients `(grad_a [B, S], grad_sigs [B, group, S])` of a loss with respect to the arguments of
    `sig_combine_grouped(a, sigs, d, N)`, given its gradient `grad_out` `[B, group, S]` with respect to the result.
    `workspace` (uint8, GPU) is allocated through torch if not given."""
    import torch

    _check_grouped("sig_combine_grouped_backward", a, sigs, d, N)
    if not isinstance(grad_out, torch.Tensor) or grad_out.dtype != a.dtype or grad_out.device != a.device or \
            grad_out.shape != sigs.shape or not grad_out.is_contiguous():
        raise ValueError("grad_out must match sigs and be contiguous")
    outs = []
    for t, like in ((grad_a, a), (grad_sigs, sigs)):
        if t is None:
            t = torch.empty_like(like)
        elif t.dtype != like.dtype or t.device != like.device or t.shape != like.shape or not t.is_contiguous():
            raise ValueError("grad_a must match a and grad_sigs must match sigs")
        outs.append(t)
    lib = load_library()
    dtype = _dtype_of(a)
    with _on_device(a.device):
        need = int(lib.sig_combine_grouped_backward_workspace_bytes(sigs.shape[0], sigs.shape[1], d, N, dtype))
        if need < 0:
            raise SigError(SIG_ERR_UNSUPPORTED, "no workspace size for this shape")
        if workspace is None:
            workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=a.device)
        status = int(lib.sig_combine_grouped_backward(a.data_ptr(), sigs.data_ptr(), grad_out.data_ptr(), sigs.shape[0],
                                                      sigs.shape[1], d, N, dtype, outs[0].data_ptr(), outs[1].data_ptr(),
                                                      workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                                      _current_stream()))
    if status != SIG_OK:
        raise SigError(status, sig_status_string(status))
    return outs[0], outs[1]
