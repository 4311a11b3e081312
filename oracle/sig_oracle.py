"""ctypes front end of the fp64 CPU oracle (`sig_oracle.c`).  TEST INFRASTRUCTURE ONLY.

Only the tests, `__graft_entry__.smoke()` and the benchmark's cpu_baseline leg may import
this module.  It never touches the HIP library or the product package.

The C file is compiled on demand with the host gcc (`build`); building the checker is not
using it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import threading

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sig_oracle.c")
_LIB = os.path.join(_HERE, "libsig_oracle.so")
_lock = threading.Lock()
_lib = None


def _compile(out_path: str, src: str = _SRC, extra=()) -> None:
    tmp = out_path + f".tmp{os.getpid()}"
    cmd = ["gcc", "-std=c99", "-O2", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared",
           "-Wall", "-Wextra", "-I", _HERE, *extra, "-o", tmp, src]
    subprocess.run(cmd, check=True)
    os.replace(tmp, out_path)


def build(force: bool = False) -> str:
    """Compile `sig_oracle.c` into `libsig_oracle.so` next to it; returns the library path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        _compile(_LIB)
    return _LIB


def _declare(lib):
    i64, i32 = ctypes.c_int64, ctypes.c_int
    dp = ctypes.POINTER(ctypes.c_double)
    lib.sig_oracle_channels.restype = i64
    lib.sig_oracle_channels.argtypes = [i32, i32]
    lib.sig_oracle_exp.restype = None
    lib.sig_oracle_exp.argtypes = [dp, i32, i32, dp]
    lib.sig_oracle_mul.restype = None
    lib.sig_oracle_mul.argtypes = [dp, dp, i32, i32, dp]
    lib.sig_oracle_mul_backward.restype = None
    lib.sig_oracle_mul_backward.argtypes = [dp, dp, dp, i32, i32, dp, dp]
    lib.sig_oracle_forward_f64.restype = i32
    lib.sig_oracle_forward_f64.argtypes = [dp, i64, i64, i32, i32, i32, i32, dp, i32]
    lib.sig_oracle_backward_f64.restype = i32
    lib.sig_oracle_backward_f64.argtypes = [dp, dp, i64, i64, i32, i32, i32, i32, dp, i32]
    lib.sig_oracle_log.restype = i32
    lib.sig_oracle_log.argtypes = [dp, i32, i32, dp]
    lib.sig_oracle_log_backward.restype = i32
    lib.sig_oracle_log_backward.argtypes = [dp, dp, i32, i32, dp]
    lib.sig_oracle_max_threads.restype = i32
    lib.sig_oracle_max_threads.argtypes = []
    return lib


def compile_copy(out_path: str, extra=()) -> str:
    """Compiles `sig_oracle.c` as it stands into `out_path` with extra compiler flags (e.g. sanitizers)."""
    _compile(out_path, _SRC, extra)
    return out_path


def source_text() -> str:
    """The text of `sig_oracle.c` (for tests that build altered copies of it)."""
    with open(_SRC) as fh:
        return fh.read()


class use_source:
    """Context manager for tests of the checker itself: inside it, every function of this module runs a library
    compiled from `text` (a copy of `sig_oracle.c`, e.g. with a mistake planted by the mutation tests, or the original
    built with sanitizers through `extra` compiler flags) into `workdir`."""

    def __init__(self, text: str, workdir: str, tag: str = "alt", extra=()):
        src = os.path.join(workdir, f"sig_oracle_{tag}.c")
        with open(src, "w") as fh:
            fh.write(text)
        self.path = os.path.join(workdir, f"libsig_oracle_{tag}.so")
        _compile(self.path, src, extra)

    def __enter__(self):
        global _lib
        _load()
        with _lock:
            self.saved, _lib = _lib, _declare(ctypes.CDLL(self.path))
        return self

    def __exit__(self, *exc):
        global _lib
        with _lock:
            _lib = self.saved
        return False


def _load():
    global _lib
    with _lock:
        if _lib is None:
            # SIG_ORACLE_LIB names another build of this same source (the sanitizer leg of the tests sets it)
            lib = _declare(ctypes.CDLL(os.environ.get("SIG_ORACLE_LIB") or build()))
            _lib = lib
    return _lib


def _dptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def channels(d: int, N: int) -> int:
    """sum_{k=1..N} d^k, the number of scalars in a depth-N signature (section 2.4)."""
    return int(_load().sig_oracle_channels(d, N))


def max_threads() -> int:
    return int(_load().sig_oracle_max_threads())


def level_slices(d: int, N: int):
    """Slices of levels 1..N inside a flat signature vector."""
    out, off = [], 0
    for k in range(1, N + 1):
        out.append(slice(off, off + d ** k))
        off += d ** k
    return out


def tensor_exp(z, N: int) -> np.ndarray:
    """exp(z) = (z, z^{(x)2}/2!, ..., z^{(x)N}/N!) as a flat vector (section 2.2)."""
    z = np.ascontiguousarray(z, dtype=np.float64)
    d = z.shape[0]
    E = np.empty(channels(d, N), dtype=np.float64)
    _load().sig_oracle_exp(_dptr(z), d, N, _dptr(E))
    return E


def group_mul(A, B, d: int, N: int) -> np.ndarray:
    """A [x] B of two flat depth-N elements (section 2.2)."""
    A = np.ascontiguousarray(A, dtype=np.float64)
    B = np.ascontiguousarray(B, dtype=np.float64)
    S = channels(d, N)
    assert A.shape == (S,) and B.shape == (S,)
    C = np.empty(S, dtype=np.float64)
    _load().sig_oracle_mul(_dptr(A), _dptr(B), d, N, _dptr(C))
    return C


def group_mul_backward(A, B, gC, d: int, N: int):
    """(gA, gB): gradients with respect to the two factors of `group_mul(A, B, d, N)`, given the gradient gC with
    respect to the product (section 5.3)."""
    A = np.ascontiguousarray(A, dtype=np.float64)
    B = np.ascontiguousarray(B, dtype=np.float64)
    gC = np.ascontiguousarray(gC, dtype=np.float64)
    S = channels(d, N)
    assert A.shape == (S,) and B.shape == (S,) and gC.shape == (S,)
    gA, gB = np.empty(S), np.empty(S)
    _load().sig_oracle_mul_backward(_dptr(A), _dptr(B), _dptr(gC), d, N, _dptr(gA), _dptr(gB))
    return gA, gB


def signature(path, N: int, stream: bool = False, basepoint: bool = False,
              num_threads: int = 0) -> np.ndarray:
    """fp64 signatures of a batch of paths.

    path: array `[B, L, d]` (any float dtype; widened exactly to float64).
    Returns `[B, S]`, or `[B, n_inc, S]` in stream mode (entry j = signature after the
    (j+1)-th increment), S = channels(d, N), n_inc = L - 1 (L with basepoint).
    """
    x = np.ascontiguousarray(path, dtype=np.float64)
    if x.ndim != 3:
        raise ValueError("path must have shape [B, L, d]")
    B, L, d = x.shape
    S = channels(d, N)
    if S < 0:
        raise ValueError("bad d or N")
    n_inc = L if basepoint else L - 1
    if n_inc < 1:
        raise ValueError("a path needs at least two points (one with basepoint)")
    shape = (B, n_inc, S) if stream else (B, S)
    out = np.empty(shape, dtype=np.float64)
    rc = _load().sig_oracle_forward_f64(_dptr(x), B, L, d, N, int(stream), int(basepoint),
                                        _dptr(out), int(num_threads))
    if rc != 0:
        raise RuntimeError(f"sig_oracle_forward_f64 failed with code {rc}")
    return out


def signature_backward(path, grad_out, N: int, stream: bool = False, basepoint: bool = False,
                       num_threads: int = 0) -> np.ndarray:
    """fp64 gradient with respect to the path of a loss whose gradient with respect to
    `signature(path, N, stream, basepoint)` is `grad_out` (section 5.3, appendix C).

    path `[B, L, d]`, grad_out `[B, S]` or `[B, n_inc, S]`; returns `[B, L, d]`.
    """
    x = np.ascontiguousarray(path, dtype=np.float64)
    g = np.ascontiguousarray(grad_out, dtype=np.float64)
    if x.ndim != 3:
        raise ValueError("path must have shape [B, L, d]")
    B, L, d = x.shape
    S = channels(d, N)
    if S < 0:
        raise ValueError("bad d or N")
    n_inc = L if basepoint else L - 1
    if n_inc < 1:
        raise ValueError("a path needs at least two points (one with basepoint)")
    want = (B, n_inc, S) if stream else (B, S)
    if g.shape != want:
        raise ValueError(f"grad_out has shape {g.shape}, expected {want}")
    gx = np.empty_like(x)
    rc = _load().sig_oracle_backward_f64(_dptr(x), _dptr(g), B, L, d, N, int(stream), int(basepoint),
                                         _dptr(gx), int(num_threads))
    if rc != 0:
        raise RuntimeError(f"sig_oracle_backward_f64 failed with code {rc}")
    return gx


def tensor_log(sig, d: int, N: int) -> np.ndarray:
    """log of signatures `[..., S]` in the truncated tensor algebra (section 2.3): same shape, all words kept."""
    a = np.ascontiguousarray(sig, dtype=np.float64)
    S = channels(d, N)
    if a.shape[-1] != S:
        raise ValueError(f"last dimension must be {S}")
    flat = a.reshape(-1, S)
    out = np.empty_like(flat)
    lib = _load()
    for r in range(flat.shape[0]):
        rc = lib.sig_oracle_log(_dptr(flat[r]), d, N, _dptr(out[r]))
        if rc != 0:
            raise RuntimeError(f"sig_oracle_log failed with code {rc}")
    return out.reshape(a.shape)


def tensor_log_backward(sig, grad_log, d: int, N: int) -> np.ndarray:
    """Gradient with respect to `sig` `[..., S]` of a loss whose gradient with respect to `tensor_log(sig)` is `grad_log`."""
    a = np.ascontiguousarray(sig, dtype=np.float64)
    g = np.ascontiguousarray(grad_log, dtype=np.float64)
    S = channels(d, N)
    if a.shape[-1] != S or g.shape != a.shape:
        raise ValueError(f"sig and grad_log must both end in {S} channels and agree in shape")
    flat, gflat = a.reshape(-1, S), g.reshape(-1, S)
    out = np.empty_like(flat)
    lib = _load()
    for r in range(flat.shape[0]):
        rc = lib.sig_oracle_log_backward(_dptr(flat[r]), _dptr(gflat[r]), d, N, _dptr(out[r]))
        if rc != 0:
            raise RuntimeError(f"sig_oracle_log_backward failed with code {rc}")
    return out.reshape(a.shape)


def lyndon_words(d: int, N: int):
    """All Lyndon words over d letters of length 1..N as tuples of 0-based letters, by length and then
    lexicographically: a word is Lyndon when it is strictly earlier than each of its proper rotations
    (appendix A.2.1).  Straight from that definition, every word tried."""
    import itertools
    out = []
    for k in range(1, N + 1):
        for w in itertools.product(range(d), repeat=k):
            if all(w < w[i:] + w[:i] for i in range(1, k)):
                out.append(w)
    return out


def lyndon_indices(d: int, N: int) -> np.ndarray:
    """Offsets, inside a flat depth-N element, of the coefficients of the Lyndon words (in the order of
    `lyndon_words`)."""
    offs = [sl.start for sl in level_slices(d, N)]
    idx = []
    for w in lyndon_words(d, N):
        flat = 0
        for letter in w:
            flat = flat * d + letter
        idx.append(offs[len(w) - 1] + flat)
    return np.asarray(idx, dtype=np.int64)


def logsignature(path, N: int, stream: bool = False, basepoint: bool = False) -> np.ndarray:
    """psi(log(Sig(path))): the coefficients of the Lyndon words in the logarithm of the signature, the basis of
    appendix A.2.4.  Shape `[B, w]` or `[B, n_inc, w]`, w = number of Lyndon words of length <= N."""
    x = np.ascontiguousarray(path, dtype=np.float64)
    d = x.shape[2]
    full = tensor_log(signature(x, N, stream, basepoint), d, N)
    return full[..., lyndon_indices(d, N)]


def logsignature_backward(path, grad_out, N: int, stream: bool = False, basepoint: bool = False) -> np.ndarray:
    """Gradient with respect to the path of a loss whose gradient with respect to `logsignature(path, ...)` is
    `grad_out`: the selection of Lyndon words, the logarithm and the signature transposed in turn."""
    x = np.ascontiguousarray(path, dtype=np.float64)
    d = x.shape[2]
    g = np.ascontiguousarray(grad_out, dtype=np.float64)
    sig = signature(x, N, stream, basepoint)
    g_log = np.zeros_like(sig)
    g_log[..., lyndon_indices(d, N)] = g
    return signature_backward(x, tensor_log_backward(sig, g_log, d, N), N, stream, basepoint)
