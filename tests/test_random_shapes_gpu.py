"""Seeded random sweep of shapes over the entry points of the HIP library, each case against the fp64 CPU oracle.

The other GPU test files pick their shapes by hand, around the limits of each kernel family.  This one draws them:
channel counts from 1 to 100, depths 1 to 9, 1 to 2500 paths, 1 to 3000 points, both modes, both precisions, with and
without the origin as basepoint, whatever kernel family `SIG_VARIANT_AUTO` picks for the draw.  The draws that first
showed a fault are kept as explicit cases in the hand-picked files; the seeds here are fixed, so the sweep is the same
on every run.

Bars as in the hand-picked files: relative L2 over the whole result 1e-4 (fp32) / 1e-9 (fp64) for the forward scans,
ten times that for the gradients of the scans; the gradients of the logarithm and of the product are measured against
the gradient of the same expression with every term taken by its absolute value (1e-5 / 1e-13), which is the size of
the sums the rounding errors come from.
"""
import numpy as np
import pytest

import paper_2001_00706_amd as sig
from oracle import sig_oracle as orc

pytestmark = pytest.mark.gpu


def rel(a, b):
    return np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-30)


def channels(d, N):
    return sum(d ** k for k in range(1, N + 1))


def draw_depth(rng, d, most):
    N = int(rng.integers(1, 10))
    while N > 1 and channels(d, N) > most:
        N -= 1
    return N


@pytest.mark.parametrize("seed", [101, 303, 505])
def test_scan_logarithm_product_and_their_gradients(seed):
    import torch
    rng = np.random.default_rng(seed)
    for _ in range(110):
        d = int(rng.choice([1, 2, 3, 4, 5, 6, 7, 8, 9, 11, 12, 13, 16, 17, 20, 24, 31, 32, 40, 49, 64, 70, 100]))
        N = draw_depth(rng, d, 60000)
        S = channels(d, N)
        B = int(rng.choice([1, 2, 3, 5, 17, 40, 300]))
        L = int(rng.choice([1, 2, 3, 7, 33, 65, 130, 300, 1100]))
        if B * L * S > 4e8:
            B = 2
        stream, bp = bool(rng.integers(0, 2)), bool(rng.integers(0, 2))
        dt = np.float32 if rng.integers(0, 2) else np.float64
        if L == 1:
            bp = True
        n_inc = L if bp else L - 1
        if stream and B * n_inc * S > 3e6:
            stream = False
        x = (rng.standard_normal((B, L, d)) * (0.3 if L < 200 else 0.05)).astype(dt)
        tol = 1e-4 if dt == np.float32 else 1e-9
        tag = f"seed {seed}: B={B} L={L} d={d} N={N} stream={stream} basepoint={bp} {dt.__name__}"
        xt = torch.from_numpy(x).to("cuda:0")
        want = orc.signature(x, N, stream, bp)
        got = sig.sig_forward(xt, N, stream=stream, basepoint=bp)
        assert rel(got.cpu().numpy(), want) <= tol, tag
        if d <= 64:
            g = rng.standard_normal(want.shape).astype(dt)
            gw = orc.signature_backward(x, g, N, stream, bp)
            gg = sig.sig_backward(xt, got, torch.from_numpy(g).to("cuda:0"), N, stream=stream, basepoint=bp)
            assert rel(gg.cpu().numpy(), gw) <= 10 * tol, tag
        rows = want.reshape(-1, S)[:50]
        lw = orc.tensor_log(rows, d, N)
        lg = sig.sig_log(got.reshape(-1, S)[:50].contiguous(), d, N).cpu().numpy()
        assert np.abs(lg - lw).max() <= 10 * tol * max(np.abs(want).max() ** N, np.abs(lw).max(), 1e-30), tag
        rows = rows[:6]
        gl = rng.standard_normal(rows.shape).astype(dt)
        glw = orc.tensor_log_backward(rows, gl, d, N)
        scale = orc.tensor_log_backward(-np.abs(rows.astype(np.float64)), np.abs(gl.astype(np.float64)), d, N)
        glg = sig.sig_log_backward(torch.from_numpy(rows.astype(dt)).to("cuda:0"), torch.from_numpy(gl).to("cuda:0"), d, N)
        bar = 1e-5 if dt == np.float32 else 1e-13
        assert np.linalg.norm(glg.cpu().numpy() - glw) <= bar * max(np.linalg.norm(scale), 1e-30), tag
        b2 = rows[::-1].copy()
        ga, gb = sig.sig_combine_backward(torch.from_numpy(rows.astype(dt)).to("cuda:0"), torch.from_numpy(b2.astype(dt)).to("cuda:0"),
                                          torch.from_numpy(gl).to("cuda:0"), d, N)
        for i in range(rows.shape[0]):
            wa, wb = orc.group_mul_backward(rows[i].astype(dt), b2[i].astype(dt), gl[i], d, N)
            sa, sb = orc.group_mul_backward(np.abs(rows[i]), np.abs(b2[i]), np.abs(gl[i]), d, N)
            assert np.linalg.norm(ga[i].cpu().numpy() - wa) <= bar * max(np.linalg.norm(sa), 1e-30), tag
            assert np.linalg.norm(gb[i].cpu().numpy() - wb) <= bar * max(np.linalg.norm(sb), 1e-30), tag


@pytest.mark.parametrize("seed", [1, 2])
def test_long_paths_in_stretches_and_many_short_paths(seed):
    import torch
    rng = np.random.default_rng(seed)
    for _ in range(60):
        many = bool(rng.integers(0, 2))
        d = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 11, 16, 17, 32, 64]))
        N = draw_depth(rng, d, 30000)
        N = min(N, 7)
        S = channels(d, N)
        dt = np.float32 if rng.integers(0, 2) else np.float64
        code = sig.SIG_F32 if dt == np.float32 else sig.SIG_F64
        tol = 1e-4 if dt == np.float32 else 1e-9
        bp = bool(rng.integers(0, 2))
        if not many:
            # few long paths: the scan and its gradient cut into stretches, and the entry point that allocates nothing
            B = int(rng.choice([1, 2, 5, 33]))
            L = int(rng.choice([2, 3, 9, 64, 257, 1000, 3001]))
            if B * L * S > 1.5e8:
                L = max(2, int(1.5e8 / (B * S)))
            chunks = int(rng.choice([2, 4, 8, 16, 64, 256]))
            stretches = int(rng.choice([2, 3, 7, 16, 64, 200]))
            x = (rng.standard_normal((B, L, d)) * (0.3 / np.sqrt(max(L, 10) / 10))).astype(dt)
            tag = f"seed {seed}: B={B} L={L} d={d} N={N} chunks={chunks} stretches={stretches} basepoint={bp} {dt.__name__}"
            xt = torch.from_numpy(x).to("cuda:0")
            want = orc.signature(x, N, False, bp)
            got = sig.sig_forward_chunked(xt, N, chunks, basepoint=bp)
            assert rel(got.cpu().numpy(), want) <= tol, tag
            if sig.sig_forward_chunked_workspace_bytes(B, L, d, N, bp, chunks, code) <= sig.sig_forward_chunked_static_max_bytes():
                assert torch.equal(got, sig.sig_forward_chunked_static(xt, N, chunks, basepoint=bp)), tag
            hint = sig.sig_forward_chunks_hint(B, L, d, N, bp, code)
            if hint > 1:
                assert rel(sig.sig_forward_chunked(xt, N, hint, basepoint=bp).cpu().numpy(), want) <= tol, tag
            if d <= 64 and sig.sig_backward_chunked_workspace_bytes(B, L, d, N, bp, stretches, code) >= 0:
                g = rng.standard_normal(want.shape).astype(dt)
                gw = orc.signature_backward(x, g, N, False, bp)
                gg = sig.sig_backward_chunked(xt, torch.from_numpy(g).to("cuda:0"), N, stretches, basepoint=bp)
                assert rel(gg.cpu().numpy(), gw) <= 10 * tol, tag
        else:
            # many short paths: the families picked from 512 and 1024 paths on, several wavefronts per SIMD
            B = int(rng.choice([513, 1024, 1300, 2500]))
            L = int(rng.choice([2, 5, 17, 65, 129]))
            stream = bool(rng.integers(0, 2))
            while B * (L if stream else 1) * S > 6e7 and L > 2:
                L = max(2, L // 2)
            if B * (L if stream else 1) * S > 6e7:
                stream = False
            if B * L * S > 4e8:
                continue
            x = (rng.standard_normal((B, L, d)) * 0.2).astype(dt)
            tag = f"seed {seed}: B={B} L={L} d={d} N={N} stream={stream} basepoint={bp} {dt.__name__}"
            xt = torch.from_numpy(x).to("cuda:0")
            want = orc.signature(x, N, stream, bp)
            got = sig.sig_forward(xt, N, stream=stream, basepoint=bp)
            assert rel(got.cpu().numpy(), want) <= tol, tag
            if d <= 64:
                g = rng.standard_normal(want.shape).astype(dt)
                gw = orc.signature_backward(x, g, N, stream, bp)
                gg = sig.sig_backward(xt, got, torch.from_numpy(g).to("cuda:0"), N, stream=stream, basepoint=bp)
                assert rel(gg.cpu().numpy(), gw) <= 10 * tol, tag
