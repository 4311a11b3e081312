"""Parity of `sig_backward_chunked` (the gradient of few long paths, walked back stretch by stretch) with the CPU oracle's
gradient, through the C ABI."""
import numpy as np
import pytest

import paper_2001_00706_amd as sig
from oracle import sig_oracle as orc
from paper_2001_00706_amd.inputs import brownian_paths, uniform_paths

pytestmark = pytest.mark.gpu

TOL = {np.float32: 1e-4, np.float64: 1e-9}


def dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def chunked(x, g, N, chunks, basepoint=False, grad_basepoint=None):
    import torch
    xt = dev(x)
    gp = torch.full_like(xt, float("nan"))
    sig.sig_backward_chunked(xt, dev(g), N, chunks, basepoint=basepoint, grad_path=gp, grad_basepoint=grad_basepoint)
    torch.cuda.synchronize()
    return gp.cpu().numpy()


def check(x, N, chunks, basepoint=False, seed=0):
    dt = x.dtype.type
    B, L, d = x.shape
    S = orc.channels(d, N)
    g = np.random.default_rng(seed + L + 7 * d + N).standard_normal((B, S)).astype(dt)
    got = chunked(x, g, N, chunks, basepoint)
    assert np.all(np.isfinite(got)), "gradient not fully written"
    want = orc.signature_backward(x, g, N, False, basepoint)
    err = np.linalg.norm(got.astype(np.float64) - want) / np.linalg.norm(want)
    assert err <= TOL[dt], err
    per_path = np.linalg.norm((got - want).reshape(B, -1), axis=1) / np.linalg.norm(want.reshape(B, -1), axis=1)
    assert per_path.max() <= 5 * TOL[dt], per_path.max()


# the stretches' shapes land on different gradient kernels: register-resident (d = 2, 4), prefix-tree (d = 3, 5, 6), the
# d = 4, N = 6 and d = 16, N = 4 kernels, many channels (d = 20), the generic one (d = 3, N = 10)
@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("B,L,d,N,chunks", [
    (2, 65, 3, 4, 4), (3, 64, 4, 4, 8), (1, 130, 2, 6, 16), (2, 41, 5, 3, 5), (1, 100, 4, 6, 7), (2, 50, 16, 4, 4),
    (1, 33, 20, 3, 3), (2, 30, 6, 5, 6), (1, 40, 3, 10, 4), (4, 20, 8, 3, 2), (1, 300, 4, 5, 32), (2, 19, 3, 3, 18),
    # depth 2 (a stretch is not a path of its own: the closed form of the depth-2 gradient must step aside) and depth 1
    (1, 64, 4, 2, 2), (2, 300, 32, 2, 16), (5, 9, 64, 2, 4), (33, 64, 16, 2, 7), (2, 100, 1, 2, 8), (3, 50, 48, 2, 5),
    (2, 40, 5, 1, 4), (1, 30, 1, 1, 3),
])
def test_stretches_walked_back_side_by_side(B, L, d, N, chunks, dtype):
    check(brownian_paths(B, L, d, seed=L + d).astype(dtype), N, chunks)


@pytest.mark.parametrize("B,L,d,N,chunks", [(2, 64, 3, 4, 4), (1, 65, 4, 4, 8), (3, 30, 5, 3, 7), (2, 9, 2, 5, 9)])
def test_with_the_origin_as_basepoint(B, L, d, N, chunks):
    check(brownian_paths(B, L, d, seed=3).astype(np.float64) + 0.3, N, chunks, basepoint=True)
    check(brownian_paths(B, L, d, seed=4) + np.float32(0.3), N, chunks, basepoint=True)


def test_with_a_basepoint_value_and_its_gradient():
    import torch
    B, L, d, N = 3, 45, 3, 4
    x = brownian_paths(B, L, d, seed=5).astype(np.float64) + 0.1
    bp = uniform_paths(B, 1, d, seed=6)[:, 0].astype(np.float64)
    g = np.random.default_rng(1).standard_normal((B, orc.channels(d, N)))
    bt = dev(bp)
    gb = torch.full_like(bt, float("nan"))
    got = chunked(x, g, N, 6, basepoint=bt, grad_basepoint=gb)
    want = orc.signature_backward(np.concatenate([bp[:, None], x], axis=1), g, N)
    np.testing.assert_allclose(got, want[:, 1:], rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(gb.cpu().numpy(), want[:, 0], rtol=1e-9, atol=1e-11)


def test_more_stretches_than_increments_and_stretches_that_do_not_divide_the_path():
    # 10 increments: 4 stretches of 3, 3, 3, 1; 64 asked for: 10 stretches of one increment
    for chunks in (4, 64, 3, 2):
        check(brownian_paths(2, 11, 3, seed=chunks).astype(np.float64), 4, chunks)
    check(brownian_paths(1, 2, 4, seed=9).astype(np.float64), 3, 2)   # a single increment


def test_the_hinted_count_on_a_long_path():
    B, L, d, N = 1, 4097, 4, 4
    chunks = sig.sig_backward_chunks_hint(B, L, d, N)
    assert chunks > 1
    check(brownian_paths(B, L, d, seed=12), N, chunks)
    check(brownian_paths(B, L, d, seed=13).astype(np.float64), N, chunks)
    assert sig.sig_backward_chunks_hint(1024, 128, 4, 6) == 1 and sig.sig_backward_chunks_hint(1, 100000, 4, 2) == 1


def test_autograd_takes_the_stretches_for_a_long_path():
    import torch
    B, L, d, N = 2, 1025, 3, 4
    assert sig.sig_backward_chunks_hint(B, L, d, N) > 1
    x = brownian_paths(B, L, d, seed=8).astype(np.float64)
    w = np.random.default_rng(9).standard_normal((B, orc.channels(d, N)))
    xt = dev(x).requires_grad_(True)
    (sig.signature(xt, N) * dev(w)).sum().backward()
    want = orc.signature_backward(x, w, N)
    np.testing.assert_allclose(xt.grad.cpu().numpy(), want, rtol=1e-8, atol=1e-10)


def test_same_result_twice_and_inputs_untouched():
    import torch
    x = dev(brownian_paths(2, 200, 4, seed=2))
    g = dev(np.random.default_rng(3).standard_normal((2, orc.channels(4, 5))).astype(np.float32))
    x0, g0 = x.clone(), g.clone()
    a = sig.sig_backward_chunked(x, g, 5, 8).clone()
    b = sig.sig_backward_chunked(x, g, 5, 8)
    torch.cuda.synchronize()
    assert torch.equal(a, b) and torch.equal(x, x0) and torch.equal(g, g0)


def test_invalid_arguments_and_short_workspace():
    import torch
    x = dev(brownian_paths(2, 50, 3, seed=1))
    g = dev(np.zeros((2, orc.channels(3, 4)), dtype=np.float32))
    for chunks in (0, 1, 70000):
        with pytest.raises(sig.SigError):
            sig.sig_backward_chunked(x, g, 4, chunks)
        assert sig.sig_backward_chunked_workspace_bytes(2, 50, 3, 4, False, chunks) == -1
    need = sig.sig_backward_chunked_workspace_bytes(2, 50, 3, 4, False, 4)
    assert need > 0
    with pytest.raises(sig.SigError):
        sig.sig_backward_chunked(x, g, 4, 4, workspace=torch.empty(need - 1, dtype=torch.uint8, device="cuda:0"))
    assert sig.sig_backward_chunks_hint(2, 1, 3, 4) == 0
