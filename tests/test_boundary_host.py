"""Host-side checks of the C ABI: exported symbols, size helpers, argument validation.

None of these launches a kernel, so they run without a GPU.
"""
import ctypes
import os
import re

import pytest

import paper_2001_00706_amd as sig
from paper_2001_00706_amd import binding
from paper_2001_00706_amd.inputs import WORKLOADS

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2001_00706_amd.build import build_lib
        build_lib()
    return sig.load_library()


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "sig.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sig_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(lib):
    declared = _declared_functions()
    assert declared == sorted(binding.EXPORTED_SYMBOLS)
    for name in declared:
        assert getattr(lib, name) is not None


def _declared(header, prefix):
    text = open(header).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(" + prefix + r"[a-z0-9_]+)\s*\(", text)))


def test_oracle_library_exports_every_symbol_its_header_declares():
    # the checker's own boundary (host pointers, fp64); nothing is computed here
    from oracle import sig_oracle
    declared = _declared(os.path.join(ROOT, "oracle", "sig_oracle.h"), "sig_oracle_")
    assert "sig_oracle_forward_f64" in declared and len(declared) == 9
    olib = ctypes.CDLL(sig_oracle.build())
    for name in declared:
        assert getattr(olib, name) is not None


def test_peaks_library_exports_every_symbol_its_header_declares():
    # the device-limit microbenchmarks bench.py times beside the kernels; loading needs no GPU
    from paper_2001_00706_amd.build import PEAKS_LIB_PATH, build_peaks_lib
    if not os.path.exists(PEAKS_LIB_PATH):
        build_peaks_lib()
    declared = _declared(os.path.join(ROOT, "include", "sig_peaks.h"), "sig_peak_")
    assert len(declared) == 6
    plib = ctypes.CDLL(PEAKS_LIB_PATH)
    for name in declared:
        assert getattr(plib, name) is not None


def test_channels(lib):
    assert sig.sig_signature_channels(2, 4) == 30
    assert sig.sig_signature_channels(4, 6) == 5460
    assert sig.sig_signature_channels(16, 4) == 69904
    assert sig.sig_signature_channels(1, 32) == 32
    assert sig.sig_signature_channels(0, 3) == -1
    assert sig.sig_signature_channels(3, 0) == -1
    assert sig.sig_signature_channels(1, 33) == -1
    assert sig.sig_signature_channels(2, 32) == 2 ** 33 - 2
    assert sig.sig_signature_channels(1024, 5) == -1          # beyond 2^40
    for w in WORKLOADS:
        assert sig.sig_signature_channels(w.d, w.N) == w.channels


def test_output_elems(lib):
    assert sig.sig_output_elems(32, 16, 2, 4, False, False) == 32 * 30
    # stream mode: one entry per increment (section 5.5: prefixes of length 2..L)
    assert sig.sig_output_elems(128, 256, 4, 5, True, False) == 128 * 255 * 1364
    assert sig.sig_output_elems(128, 256, 4, 5, True, True) == 128 * 256 * 1364
    assert sig.sig_output_elems(0, 2, 3, 3, False, False) == 0
    assert sig.sig_output_elems(4, 1, 3, 3, False, False) == -1   # a single point is no path
    assert sig.sig_output_elems(4, 1, 3, 3, False, True) == 4 * 39
    assert sig.sig_output_elems(-1, 4, 3, 3, False, False) == -1
    assert sig.sig_output_elems(2 ** 40, 2 ** 30, 2, 20, True, False) == -1


def _F_closed_form(d, N):
    # appendix A.1.3, closed form of F(d, N) for d >= 2
    return (d ** (N + 2) - d ** 3 - (N - 1) * d ** 2 + (N - 1) * d) // ((d - 1) ** 2)


@pytest.mark.parametrize("d,N", [(2, 4), (4, 6), (8, 5), (4, 5), (16, 4), (3, 3), (7, 7), (2, 1)])
def test_fused_fma_count_matches_the_papers_multiplication_count(lib, d, N):
    # appendix A.1.2: F(d, N) = d(N-1) + sum_{k=1..N} sum_{i=2..k} d^i; M = F - d(N-1)
    M = sig.sig_fused_fmas(d, N)
    assert M == sum(sum(d ** i for i in range(2, k + 1)) for k in range(1, N + 1))
    assert M + d * (N - 1) == _F_closed_form(d, N)


def test_fused_fma_count_of_the_benchmark_shapes(lib):
    got = [sig.sig_fused_fmas(w.d, w.N) for w in WORKLOADS]
    assert got == [44, 7248, 42752, 1792, 74496]


def test_status_strings(lib):
    texts = [sig.sig_status_string(s) for s in range(6)]
    assert texts[0] == "ok" and len(set(texts)) == 6 and "scratch" in texts[sig.SIG_ERR_TOO_LARGE]
    assert sig.sig_status_string(99) == "unknown status"


def test_validation_happens_before_any_device_work(lib):
    raw = sig.sig_forward_raw
    dummy = 0x1000  # never dereferenced: every call below fails validation or has B == 0
    assert raw(dummy, -1, 4, 2, 2, 0, 0, sig.SIG_F32, dummy, 0) == sig.SIG_ERR_INVALID_ARG
    assert raw(dummy, 2, 1, 2, 2, 0, 0, sig.SIG_F32, dummy, 0) == sig.SIG_ERR_INVALID_ARG
    assert raw(dummy, 2, 0, 2, 2, 0, 1, sig.SIG_F32, dummy, 0) == sig.SIG_ERR_INVALID_ARG
    assert raw(dummy, 2, 4, 0, 2, 0, 0, sig.SIG_F32, dummy, 0) == sig.SIG_ERR_INVALID_ARG
    assert raw(dummy, 2, 4, 2, 0, 0, 0, sig.SIG_F32, dummy, 0) == sig.SIG_ERR_INVALID_ARG
    assert raw(dummy, 2, 4, 2, 33, 0, 0, sig.SIG_F32, dummy, 0) == sig.SIG_ERR_INVALID_ARG
    assert raw(dummy, 2, 4, 2, 2, 0, 0, 7, dummy, 0) == sig.SIG_ERR_INVALID_ARG
    assert raw(0, 2, 4, 2, 2, 0, 0, sig.SIG_F32, dummy, 0) == sig.SIG_ERR_INVALID_ARG
    assert raw(dummy, 2, 4, 2, 2, 0, 0, sig.SIG_F32, 0, 0) == sig.SIG_ERR_INVALID_ARG
    assert raw(dummy, 2, 4, 1024, 5, 0, 0, sig.SIG_F32, dummy, 0) == sig.SIG_ERR_OVERFLOW
    assert raw(dummy, 2 ** 40, 2 ** 30, 2, 20, 1, 0, sig.SIG_F32, dummy, 0) == sig.SIG_ERR_OVERFLOW
    assert raw(dummy, 2, 4, 2, 2, 0, 0, sig.SIG_F32, dummy, 0, variant=99) == sig.SIG_ERR_INVALID_ARG
    # the matrix-core family is fp32 only
    assert raw(dummy, 2, 4, 4, 3, 0, 0, sig.SIG_F64, dummy, 0, variant=sig.SIG_VARIANT_MFMA) \
        == sig.SIG_ERR_UNSUPPORTED
    # an empty batch is fine and enqueues nothing, even with null pointers
    assert raw(0, 0, 4, 2, 2, 0, 0, sig.SIG_F32, 0, 0) == sig.SIG_OK


def test_combine_validation(lib):
    f = lib.sig_combine
    dummy = 0x1000
    assert f(dummy, dummy, -1, 2, 2, sig.SIG_F32, dummy, 0) == sig.SIG_ERR_INVALID_ARG
    assert f(dummy, dummy, 2, 0, 2, sig.SIG_F32, dummy, 0) == sig.SIG_ERR_INVALID_ARG
    assert f(dummy, dummy, 2, 2, 0, sig.SIG_F32, dummy, 0) == sig.SIG_ERR_INVALID_ARG
    assert f(dummy, dummy, 2, 2, 2, 5, dummy, 0) == sig.SIG_ERR_INVALID_ARG
    assert f(0, dummy, 2, 2, 2, sig.SIG_F32, dummy, 0) == sig.SIG_ERR_INVALID_ARG
    assert f(dummy, dummy, 2, 1024, 5, sig.SIG_F32, dummy, 0) == sig.SIG_ERR_OVERFLOW
    assert f(dummy, dummy, 2, 2, 32, sig.SIG_F32, dummy, 0) == sig.SIG_ERR_UNSUPPORTED
    assert f(0, 0, 0, 2, 2, sig.SIG_F32, 0, 0) == sig.SIG_OK


def test_backward_validation(lib):
    f = lib.sig_backward
    p = 0x1000
    args = lambda **kw: [kw.get("path", p), kw.get("sig", p), kw.get("gout", p), kw.get("B", 2), kw.get("L", 4),
                         kw.get("d", 2), kw.get("N", 2), 0, kw.get("basepoint", 0), kw.get("bpv", 0),
                         kw.get("dtype", sig.SIG_F32), kw.get("gpath", p), kw.get("gbp", 0), 0, 0, 0]
    assert f(*args(B=-1)) == sig.SIG_ERR_INVALID_ARG
    assert f(*args(d=0)) == sig.SIG_ERR_INVALID_ARG
    assert f(*args(N=33)) == sig.SIG_ERR_INVALID_ARG
    assert f(*args(L=1)) == sig.SIG_ERR_INVALID_ARG
    assert f(*args(dtype=7)) == sig.SIG_ERR_INVALID_ARG
    for name in ("path", "sig", "gout", "gpath"):
        assert f(*args(**{name: 0})) == sig.SIG_ERR_INVALID_ARG
    assert f(*args(d=1024, N=5)) == sig.SIG_ERR_OVERFLOW
    assert f(*args(d=65, N=1)) == sig.SIG_ERR_UNSUPPORTED          # more than 64 channels
    assert f(*args(d=2, N=31)) == sig.SIG_ERR_UNSUPPORTED          # 2^32 scalars per signature
    assert f(*args(B=0, path=0, sig=0, gout=0, gpath=0)) == sig.SIG_OK
    # a basepoint value or its gradient without the basepoint flag
    assert f(*args(bpv=p)) == sig.SIG_ERR_INVALID_ARG
    assert f(*args(gbp=p)) == sig.SIG_ERR_INVALID_ARG
    assert sig.sig_backward_workspace_bytes(2, 1, 2, 2, False, False) == -1
    assert sig.sig_backward_workspace_bytes(2, 4, 65, 1, False, False) == -1
    assert sig.sig_backward_workspace_bytes(0, 4, 2, 2, False, False) == 0
    # fp32, d <= 8, N <= 9: the partial gradients of the prefix-tree kernels, one per workgroup (7^5 words in 66
    # workgroups), increment and channel
    assert sig.sig_backward_workspace_bytes(32, 128, 7, 7, False, False) == 32 * 66 * 127 * 7 * 4


def test_signature_invert_and_strided_combine_validation(lib):
    p = 0x1000
    f = lib.sig_signature
    # path, B, L, d, N, stream, basepoint, basepoint_value, initial, inverse, dtype, out, hip_stream
    assert f(p, 2, 4, 2, 2, 0, 0, 0, 0, 0, sig.SIG_F32, 0, 0) == sig.SIG_ERR_INVALID_ARG      # null out
    assert f(p, 2, 4, 2, 2, 0, 0, p, 0, 0, sig.SIG_F32, p, 0) == sig.SIG_ERR_INVALID_ARG      # value without the flag
    assert f(p, 2, 1, 2, 2, 0, 0, 0, 0, 0, sig.SIG_F32, p, 0) == sig.SIG_ERR_INVALID_ARG      # one point
    assert f(p, 2, 4, 2, 2, 0, 0, 0, 0, 0, 9, p, 0) == sig.SIG_ERR_INVALID_ARG
    assert f(p, 2, 4, 2, 31, 0, 0, 0, p, 0, sig.SIG_F32, p, 0) == sig.SIG_ERR_UNSUPPORTED     # S >= 2^31 with initial
    assert f(0, 0, 4, 2, 2, 0, 0, 0, 0, 1, sig.SIG_F32, 0, 0) == sig.SIG_OK
    g = lib.sig_invert
    assert g(p, -1, 2, 2, sig.SIG_F32, p, 0) == sig.SIG_ERR_INVALID_ARG
    assert g(0, 3, 2, 2, sig.SIG_F32, p, 0) == sig.SIG_ERR_INVALID_ARG
    assert g(p, 3, 2, 32, sig.SIG_F32, p, 0) == sig.SIG_ERR_UNSUPPORTED
    assert g(0, 0, 2, 2, sig.SIG_F64, 0, 0) == sig.SIG_OK
    h = lib.sig_combine_strided
    # a, a_stride, b, b_stride, B, d, N, dtype, out, out_stride, hip_stream
    assert h(p, 6, p, 6, 2, 2, 2, sig.SIG_F32, p, 5, 0) == sig.SIG_ERR_INVALID_ARG            # out rows would overlap
    assert h(p, -1, p, 6, 2, 2, 2, sig.SIG_F32, p, 6, 0) == sig.SIG_ERR_INVALID_ARG
    assert h(p, 0, 0, 6, 2, 2, 2, sig.SIG_F32, p, 6, 0) == sig.SIG_ERR_INVALID_ARG
    assert h(0, 0, 0, 0, 0, 2, 2, sig.SIG_F32, 0, 6, 0) == sig.SIG_OK
    cb, cbw = lib.sig_combine_backward, lib.sig_combine_backward_workspace_bytes
    # a, b, grad_out, B, d, N, dtype, grad_a, grad_b, workspace, workspace_bytes, hip_stream
    assert cbw(3, 2, 1, sig.SIG_F32) == 0 and cbw(3, 2, 4, sig.SIG_F64) > 0 and cbw(-1, 2, 4, sig.SIG_F32) == -1
    assert cb(p, p + 64, p + 128, 2, 2, 3, sig.SIG_F32, p + 192, p + 192, p, 1 << 20, 0) == sig.SIG_ERR_INVALID_ARG
    assert cb(p, p + 64, p + 128, 2, 2, 3, sig.SIG_F32, p, p + 256, p, 1 << 20, 0) == sig.SIG_ERR_INVALID_ARG
    assert cb(p, p + 64, p + 128, 2, 2, 3, sig.SIG_F32, p + 192, p + 256, 0, 0, 0) == sig.SIG_ERR_INVALID_ARG
    assert cb(p, p + 64, 0, 2, 2, 3, sig.SIG_F32, p + 192, p + 256, p, 1 << 20, 0) == sig.SIG_ERR_INVALID_ARG
    assert cb(0, 0, 0, 0, 2, 3, sig.SIG_F32, 0, 0, 0, 0, 0) == sig.SIG_OK
    cg, cgb, cgw = lib.sig_combine_grouped, lib.sig_combine_grouped_backward, lib.sig_combine_grouped_backward_workspace_bytes
    # a, sigs, B, group, d, N, dtype, out, hip_stream
    assert cg(p, p + 64, 2, 0, 2, 3, sig.SIG_F32, p + 64, 0) == sig.SIG_ERR_INVALID_ARG
    assert cg(p, 0, 2, 3, 2, 3, sig.SIG_F32, p + 64, 0) == sig.SIG_ERR_INVALID_ARG
    assert cg(p, p + 64, 2, 3, 2, 3, sig.SIG_F32, p, 0) == sig.SIG_ERR_INVALID_ARG           # out is the left factor
    assert cg(p, p + 64, 2, 1 << 62, 2, 3, sig.SIG_F32, p + 64, 0) == sig.SIG_ERR_INVALID_ARG  # B * group overflows
    assert cg(p, p + 64, 2, 3, 2, 32, sig.SIG_F32, p + 64, 0) == sig.SIG_ERR_UNSUPPORTED
    assert cg(0, 0, 0, 3, 2, 3, sig.SIG_F32, 0, 0) == sig.SIG_OK
    # the plain gradient's workspace for all B * group products, rounded up, plus one signature per product
    plain = cbw(6, 2, 3, sig.SIG_F32)
    assert cgw(2, 3, 2, 3, sig.SIG_F32) == (plain + 255) // 256 * 256 + 6 * 14 * 4
    assert cgw(2, 0, 2, 3, sig.SIG_F32) == -1 and cgw(2, 3, 2, 3, 9) == -1 and cgw(-1, 3, 2, 3, sig.SIG_F32) == -1
    # a, sigs, grad_out, B, group, d, N, dtype, grad_a, grad_sigs, workspace, workspace_bytes, hip_stream
    assert cgb(p, p + 64, p + 128, 2, 3, 2, 3, sig.SIG_F32, p + 192, p + 192, p, 1 << 20, 0) == sig.SIG_ERR_INVALID_ARG
    assert cgb(p, p + 64, p + 128, 2, 3, 2, 3, sig.SIG_F32, p + 192, p + 256, 0, 0, 0) == sig.SIG_ERR_INVALID_ARG
    assert cgb(p, p + 64, p + 128, 2, 3, 2, 3, sig.SIG_F32, p + 192, p + 256, p + 8, 1 << 20, 0) == sig.SIG_ERR_INVALID_ARG
    assert cgb(p, p + 64, p + 128, 2, 0, 2, 3, sig.SIG_F32, p + 192, p + 256, p, 1 << 20, 0) == sig.SIG_ERR_INVALID_ARG
    assert cgb(0, 0, 0, 0, 3, 2, 3, sig.SIG_F32, 0, 0, 0, 0, 0) == sig.SIG_OK
    m, mb = lib.sig_combine_many, lib.sig_combine_many_workspace_bytes
    # sigs, B, n, d, N, dtype, out, workspace, workspace_bytes, hip_stream
    assert mb(3, 1, 2, 2, sig.SIG_F32) == 0 and mb(3, 2, 2, 2, sig.SIG_F32) == 0
    assert mb(3, 3, 2, 2, sig.SIG_F32) == 3 * 2 * 6 * 4                       # one round of 2 per row
    assert mb(3, 9, 2, 2, sig.SIG_F64) == 3 * (5 + 3) * 6 * 8                 # rounds of 5 and 3, then reuse
    assert mb(3, 0, 2, 2, sig.SIG_F32) == -1 and mb(3, 3, 2, 2, 9) == -1
    assert m(p, 3, 0, 2, 2, sig.SIG_F32, p, 0, 0, 0) == sig.SIG_ERR_INVALID_ARG
    assert m(p, 3, 3, 2, 2, sig.SIG_F32, p, 0, 0, 0) == sig.SIG_ERR_INVALID_ARG   # workspace missing
    assert m(p, 3, 3, 2, 2, sig.SIG_F32, p, p, 100, 0) == sig.SIG_ERR_INVALID_ARG  # workspace short
    assert m(0, 3, 2, 2, 2, sig.SIG_F32, p, 0, 0, 0) == sig.SIG_ERR_INVALID_ARG
    assert m(p, 3, 2, 2, 32, sig.SIG_F32, p, 0, 0, 0) == sig.SIG_ERR_UNSUPPORTED
    assert m(0, 0, 5, 2, 2, sig.SIG_F32, 0, 0, 0, 0) == sig.SIG_OK


def test_chunk_hint(lib):
    h = lib.sig_forward_chunks_hint
    # B, L, d, N, basepoint, dtype
    assert h(1, 65536, 4, 6, 0, sig.SIG_F32) == 512          # 65535 increments: 1024 chunks would be 63 each
    assert h(1, 65537, 4, 6, 0, sig.SIG_F32) == 1024
    assert h(1, 65536, 4, 6, 1, sig.SIG_F32) == 1024         # the basepoint adds an increment
    assert h(32, 128, 8, 5, 0, sig.SIG_F32) == 1             # the cfg3 shape: short
    assert h(1024, 128, 4, 6, 0, sig.SIG_F32) == 1 and h(65, 100000, 4, 6, 0, sig.SIG_F32) == 1
    assert h(1, 512, 4, 6, 0, sig.SIG_F32) == 1 and h(1, 513, 4, 6, 0, sig.SIG_F32) == 8
    assert h(1, 2049, 8, 4, 0, sig.SIG_F32) == 1 and h(1, 4097, 8, 4, 0, sig.SIG_F32) == 64
    assert h(1, 2049, 8, 4, 0, sig.SIG_F64) == 32            # no 64-wavefront kernels in fp64
    assert h(64, 65537, 4, 6, 0, sig.SIG_F32) == 16          # 1024 stretches at most
    assert h(64, 65537, 16, 4, 0, sig.SIG_F32) == 8          # 256 MiB of signatures at most
    assert h(1, 1, 4, 6, 0, sig.SIG_F32) == 0 and h(1, 4096, 4, 6, 0, 9) == 0 and h(1, 4096, 0, 6, 0, sig.SIG_F32) == 0
    assert h(0, 4096, 4, 6, 0, sig.SIG_F32) == 1
    # depth 2, a plain sum over the increments: from 24 staged tiles on, stretches of at least 128 increments, 2048 at most
    assert h(1, 3072, 4, 2, 0, sig.SIG_F32) == 1 and h(1, 3073, 4, 2, 0, sig.SIG_F32) == 16
    assert h(1, 131073, 8, 2, 0, sig.SIG_F64) == 1024 and h(64, 131073, 8, 2, 0, sig.SIG_F32) == 32
    assert h(1, 1513, 64, 2, 0, sig.SIG_F32) == 8 and h(1, 1512, 64, 2, 0, sig.SIG_F32) == 1
    assert h(1024, 8193, 2, 2, 0, sig.SIG_F32) == 2 and h(1025, 8193, 2, 2, 0, sig.SIG_F32) == 1


def test_backward_chunk_hint_and_workspace(lib):
    h = lib.sig_backward_chunks_hint
    # B, L, d, N, basepoint, dtype: about sqrt(n_inc) / 2 stretches for small signatures, fewer for larger ones
    assert h(1, 4097, 4, 4, 0, sig.SIG_F32) == 32 and h(1, 65537, 4, 6, 0, sig.SIG_F32) == 64
    assert h(1, 2049, 5, 7, 0, sig.SIG_F32) == 8               # signatures beyond the LDS: a launch per stretch
    assert h(1, 512, 4, 4, 0, sig.SIG_F32) == 1 and h(1, 513, 4, 4, 0, sig.SIG_F32) == 8
    assert h(1, 512, 4, 4, 1, sig.SIG_F32) == 8                # the basepoint adds an increment
    assert h(128, 100001, 3, 4, 0, sig.SIG_F32) == 8 and h(129, 100001, 3, 4, 0, sig.SIG_F32) == 1   # 1024 rows at most
    assert h(1, 100001, 4, 2, 0, sig.SIG_F32) == 1             # depth 2 walks nothing
    assert h(1024, 128, 4, 6, 0, sig.SIG_F32) == 1
    assert h(1, 1, 4, 6, 0, sig.SIG_F32) == 0 and h(1, 4096, 4, 6, 0, 9) == 0 and h(1, 4096, 0, 6, 0, sig.SIG_F32) == 0
    w = lib.sig_backward_chunked_workspace_bytes
    # 10 increments in 4 stretches of 3: 8 rows of 4 points (256-byte pieces: points, 3 x signatures, point gradients)
    S = 3 + 9 + 27
    piece = lambda n: (n + 255) // 256 * 256
    inner = lib.sig_backward_workspace_bytes(8, 4, 3, 3, 0, 0, sig.SIG_F32)
    assert w(2, 11, 3, 3, 0, 4, sig.SIG_F32) == 2 * piece(8 * 4 * 3 * 4) + 3 * piece(8 * S * 4) + piece(inner)
    assert w(2, 11, 3, 3, 0, 1, sig.SIG_F32) == -1 and w(2, 11, 3, 3, 0, 65537, sig.SIG_F32) == -1
    assert w(70000, 11, 3, 3, 0, 4, sig.SIG_F32) == -1 and w(0, 11, 3, 3, 0, 4, sig.SIG_F32) == 0


def test_lyndon_table_is_built_on_the_host(lib):
    # appendix A.2.1; d = 2, N = 4: a, b, ab, aab, abb, aaab, aabb, abbb at offsets 0,1 | 2+1 | 6+1, 6+3 | 14+1, 14+3, 14+7
    assert sig.sig_lyndon_indices(2, 4) == [0, 1, 3, 7, 9, 15, 17, 21]
    assert sig.sig_logsignature_channels(2, 4) == 8
    assert sig.sig_logsignature_channels(4, 6) == 964        # Witt's formula (section 2.3): 4 + 6 + 20 + 60 + 204 + 670
    assert sig.sig_logsignature_channels(3, 1) == 3
    assert sig.sig_logsignature_channels(0, 3) == -1
    assert sig.sig_logsignature_channels(2, 32) == -1
    import ctypes
    buf = (ctypes.c_int64 * 4)()
    assert lib.sig_lyndon_indices(2, 4, buf, 4) == sig.SIG_ERR_INVALID_ARG      # room for 4 of 8
    assert lib.sig_lyndon_indices(2, 4, None, 8) == sig.SIG_ERR_INVALID_ARG
    p = 0x1000
    assert lib.sig_log(p, 2, 2, 2, sig.SIG_F32, p, 0) == sig.SIG_ERR_INVALID_ARG   # in place
    assert lib.sig_log(p, -2, 2, 2, sig.SIG_F32, p + 64, 0) == sig.SIG_ERR_INVALID_ARG
    assert lib.sig_lyndon_gather(p, 2, 2, 2, p, 7, sig.SIG_F32, p, 0) == sig.SIG_ERR_INVALID_ARG   # more entries than S
    assert lib.sig_lyndon_gather(p, 2, 2, 2, 0, 3, sig.SIG_F32, p, 0) == sig.SIG_ERR_INVALID_ARG
    assert lib.sig_lyndon_gather(0, 0, 2, 2, 0, 3, sig.SIG_F32, 0, 0) == sig.SIG_OK
    assert lib.sig_lyndon_scatter(p, 2, 2, 2, p, 7, sig.SIG_F32, p, 0) == sig.SIG_ERR_INVALID_ARG
    assert lib.sig_lyndon_scatter(0, 2, 2, 2, p, 3, sig.SIG_F32, p, 0) == sig.SIG_ERR_INVALID_ARG
    assert lib.sig_lyndon_scatter(0, 0, 2, 2, 0, 3, sig.SIG_F32, 0, 0) == sig.SIG_OK
    lb, lbw = lib.sig_log_backward, lib.sig_log_backward_workspace_bytes
    # sig, grad_log, rows, d, N, dtype, grad_sig, workspace, workspace_bytes, hip_stream
    # signatures that fit the LDS are served by a single launch that needs no workspace (at d = 2, 4, 8 whatever the
    # batch; otherwise mid-sized ones only in small batches); large ones need one
    assert lbw(3, 2, 1, sig.SIG_F32) == 0 and lbw(3, 2, 4, sig.SIG_F32) == 0 and lbw(3, 0, 4, sig.SIG_F32) == -1
    assert lbw(3, 4, 8, sig.SIG_F32) > 0 and lbw(1024, 4, 6, sig.SIG_F32) == 0 and lbw(8, 4, 6, sig.SIG_F32) == 0
    assert lbw(1024, 3, 7, sig.SIG_F32) > 0 and lbw(8, 3, 7, sig.SIG_F32) == 0
    assert lbw(3, 2, 4, 7) == -1
    assert lb(p, p + 64, 2, 2, 3, sig.SIG_F32, p, p, 1 << 20, 0) == sig.SIG_ERR_INVALID_ARG          # in place
    assert lb(p, p + 64, 2, 4, 8, sig.SIG_F32, p + 128, 0, 0, 0) == sig.SIG_ERR_INVALID_ARG          # no workspace
    assert lb(p, p + 64, 2, 4, 8, sig.SIG_F32, p + 128, p + 4, 1 << 30, 0) == sig.SIG_ERR_INVALID_ARG  # misaligned
    assert lb(p, 0, 2, 2, 3, sig.SIG_F32, p + 128, p, 1 << 20, 0) == sig.SIG_ERR_INVALID_ARG
    assert lb(p, p + 64, 2, 2, 32, sig.SIG_F32, p + 128, p, 1 << 20, 0) == sig.SIG_ERR_UNSUPPORTED
    assert lb(0, 0, 0, 2, 3, sig.SIG_F64, 0, 0, 0, 0) == sig.SIG_OK


def test_variant_names(lib):
    assert sig.sig_variant_name(32, 16, 2, 4, False, False, variant=sig.SIG_VARIANT_GENERIC) == "generic"
    assert sig.sig_variant_name(32, 1, 2, 4, False, False) == "invalid"
    assert sig.sig_variant_name(32, 16, 3, 4, False, False, variant=sig.SIG_VARIANT_MFMA) == "unsupported"
    assert sig.sig_variant_name(32, 16, 4, 4, False, False, variant=sig.SIG_VARIANT_MFMA) == "mfma_d4"
    assert sig.sig_variant_name(32, 16, 4, 7, False, False, variant=sig.SIG_VARIANT_MFMA) == "unsupported"
    assert sig.sig_variant_name(32, 16, 4, 7, False, False, variant=sig.SIG_VARIANT_MFMA_SHARD) == "mfma_d4_shard"
    assert sig.sig_variant_name(32, 16, 2, 4, True, True, sig.SIG_F64, sig.SIG_VARIANT_SMALL) == "small"
    assert sig.sig_variant_name(32, 16, 4, 6, True, False, variant=sig.SIG_VARIANT_MFMA) == "unsupported"
    # the row kernel: stream mode wherever a lane per word leaves one or two levels below it (two up to 8 channels) ...
    auto = lambda *a, **k: sig.sig_variant_name(*a, **k)
    assert auto(128, 256, 8, 3, True, False) == auto(128, 256, 8, 4, True, False, sig.SIG_F64) == "row_stream"
    assert auto(128, 256, 3, 5, True, False) == auto(128, 256, 2, 8, True, True) == auto(4, 9, 16, 2, True, False) == "row_stream"
    assert auto(128, 256, 8, 5, True, False) == auto(128, 256, 3, 6, True, False) == auto(128, 256, 12, 3, True, False) == "tree"
    assert auto(128, 256, 2, 3, True, False) == "small"                       # 4 lanes per row: left to the one-wavefront kernel
    assert auto(128, 256, 4, 5, True, False) == "mfma_d4_shard"               # the matrix-core stream kernels come first
    assert auto(128, 256, 12, 3, True, False, variant=sig.SIG_VARIANT_ROW_STREAM) == "unsupported"
    # ... and final mode where one level lies below the word and the state exceeds 64 scalars
    assert auto(32, 128, 8, 3, False, False) == auto(32, 128, 3, 4, False, True) == auto(32, 128, 2, 7, False, False) == "row_stream"
    assert auto(32, 128, 5, 4, False, False) == "tree" and auto(32, 128, 2, 5, False, False) == "small"
    assert auto(32, 128, 5, 4, False, False, variant=sig.SIG_VARIANT_ROW_STREAM) == "row_stream"


def test_python_binding_refuses_cpu_tensors(lib):
    import torch
    with pytest.raises(TypeError):
        sig.sig_forward(torch.zeros(2, 3, 2), 2)
    with pytest.raises(TypeError):
        sig.sig_forward([[0.0, 1.0]], 2)


def test_product_package_does_not_touch_the_oracle():
    pkg_dir = os.path.join(ROOT, "paper_2001_00706_amd")
    for dirpath, _, files in os.walk(pkg_dir):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "sig_oracle" not in text and "import oracle" not in text, f
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c", ".h")):
            text = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_2001_00706_amd" not in text and "libsig.so" not in text, f
