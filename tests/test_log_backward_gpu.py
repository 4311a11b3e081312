"""GPU parity of `sig_log_backward`, `sig_lyndon_scatter` and the differentiable `logsignature` with the fp64
oracle (paper sections 2.3, 4.3, 5.3).

The gradient of the logarithm is, like the logarithm, an alternating sum of products that largely cancel, so its
rounding error is measured against the size of the terms summed.  That size comes from the oracle too: at -|x|
with cotangent |g| every term of the series has the same sign, so the oracle's gradient there is, scalar by scalar,
the sum of the absolute values of the terms.
"""
import numpy as np
import pytest

import paper_2001_00706_amd as sig
from oracle import sig_oracle as orc
from paper_2001_00706_amd.inputs import WORKLOADS, brownian_paths, workload_paths

pytestmark = pytest.mark.gpu

TOL = {np.float32: 1e-5, np.float64: 1e-13}


def dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def host(t):
    import torch
    torch.cuda.synchronize()
    return t.cpu().numpy()


def assert_grad_close(got, want, scale, d, N, dt):
    got = np.asarray(got, dtype=np.float64)
    for sl in orc.level_slices(d, N):
        err = np.linalg.norm(got[..., sl] - want[..., sl])
        bound = np.linalg.norm(scale[..., sl])
        assert err <= TOL[dt] * (bound if bound > 0 else 1.0), (err, bound)


# rows, d, N: matrices of at most 256 columns only (2^8, 3^5, 5^3, 9^2), wider ones (2^9, 4^5, 7^3, 8^3), a single
# letter, depths 1 and 2, and a channel count without a compiled-in divisor
SHAPES = [(3, 2, 9), (2, 2, 10), (5, 3, 6), (2, 4, 6), (3, 5, 4), (2, 7, 4), (4, 1, 5), (3, 6, 1), (3, 4, 2),
          (2, 8, 4), (3, 9, 3), (1, 3, 7), (7, 2, 3)]


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("rows,d,N", SHAPES)
def test_gradient_of_the_logarithm(rows, d, N, dtype):
    x = orc.signature(1.5 * brownian_paths(rows, 8, d, seed=rows + 10 * d + N), N).astype(dtype)
    g = np.random.default_rng(N * 100 + d).standard_normal(x.shape).astype(dtype)
    got = host(sig.sig_log_backward(dev(x), dev(g), d, N))
    want = orc.tensor_log_backward(x, g, d, N)
    scale = orc.tensor_log_backward(-np.abs(x.astype(np.float64)), np.abs(g.astype(np.float64)), d, N)
    assert_grad_close(got, want, scale, d, N, dtype)


def test_gradient_of_the_logarithm_of_arbitrary_elements_and_leading_dimensions():
    # not only signatures; leading dimensions are flattened into rows
    d, N = 3, 5
    S = orc.channels(d, N)
    rng = np.random.default_rng(1)
    x, g = 0.5 * rng.standard_normal((2, 3, S)), rng.standard_normal((2, 3, S))
    got = host(sig.sig_log_backward(dev(x), dev(g), d, N))
    scale = orc.tensor_log_backward(-np.abs(x), np.abs(g), d, N)
    assert got.shape == x.shape
    assert_grad_close(got, orc.tensor_log_backward(x, g, d, N), scale, d, N, np.float64)


def test_two_calls_give_identical_bits():
    d, N = 4, 6
    x = orc.signature(brownian_paths(6, 9, d, seed=2), N).astype(np.float32)
    g = np.random.default_rng(0).standard_normal(x.shape).astype(np.float32)
    a = host(sig.sig_log_backward(dev(x), dev(g), d, N))
    b = host(sig.sig_log_backward(dev(x), dev(g), d, N))
    assert np.array_equal(a, b)


def test_scatter_is_the_transpose_of_gather():
    d, N = 3, 5
    idx = orc.lyndon_indices(d, N)
    g = np.random.default_rng(3).standard_normal((4, 2, len(idx)))
    got = host(sig.sig_lyndon_scatter(dev(g), d, N))
    want = np.zeros((4, 2, orc.channels(d, N)))
    want[..., idx] = g
    assert np.array_equal(got, want)


def test_workspace_is_checked():
    import torch
    d, N = 4, 7     # 21 844 scalars per signature: the chain of launches, which needs a workspace
    x = dev(orc.signature(brownian_paths(2, 5, d, seed=1), N))
    need = sig.sig_log_backward_workspace_bytes(2, d, N, sig.SIG_F64)
    assert need > 0
    short = torch.empty(need - 1, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(sig.SigError):
        sig.sig_log_backward(x, x.clone(), d, N, workspace=short)
    assert sig.sig_log_backward_workspace_bytes(2, d, 1, sig.SIG_F64) == 0
    assert sig.sig_log_backward_workspace_bytes(2, 2, 4, sig.SIG_F64) == 0      # single launch, everything in LDS


@pytest.mark.parametrize("dtype", [np.float32, np.float64], ids=["float32", "float64"])
def test_both_routes_agree_on_the_same_shape(dtype):
    # d = 3, N = 7 (3279 scalars): 8 signatures go through the single-launch kernel (no workspace), 300 through the
    # chain of launches (workspace); in fp64 the working set of a signature exceeds the LDS and both take the chain
    d, N = 3, 7
    code = sig.SIG_F32 if dtype == np.float32 else sig.SIG_F64
    assert sig.sig_log_backward_workspace_bytes(300, d, N, code) > 0
    assert (sig.sig_log_backward_workspace_bytes(8, d, N, code) == 0) == (dtype == np.float32)
    x = orc.signature(brownian_paths(300, 6, d, seed=12), N).astype(dtype)
    g = np.random.default_rng(4).standard_normal(x.shape).astype(dtype)
    many = host(sig.sig_log_backward(dev(x), dev(g), d, N))
    few = host(sig.sig_log_backward(dev(x[:8]), dev(g[:8]), d, N))
    want = orc.tensor_log_backward(x[:8], g[:8], d, N)
    scale = orc.tensor_log_backward(-np.abs(x[:8].astype(np.float64)), np.abs(g[:8].astype(np.float64)), d, N)
    assert_grad_close(few, want, scale, d, N, dtype)
    assert_grad_close(many[:8], want, scale, d, N, dtype)
    want = orc.tensor_log_backward(x, g, d, N)
    scale = orc.tensor_log_backward(-np.abs(x.astype(np.float64)), np.abs(g.astype(np.float64)), d, N)
    assert_grad_close(many, want, scale, d, N, dtype)


@pytest.mark.parametrize("dtype", [np.float32, np.float64], ids=["float32", "float64"])
@pytest.mark.parametrize("rows,d,N", [(5, 2, 2), (300, 2, 9), (3, 2, 10), (70, 4, 3), (9, 4, 6), (2, 8, 2), (40, 8, 3), (3, 8, 4)])
def test_power_of_two_channels_take_one_launch_at_any_batch_size(rows, d, N, dtype):
    # d = 2, 4, 8: the gather form of the single-launch kernel whenever a signature's working set fits the LDS (all of
    # these do, in both precisions: the largest, d = 4, N = 6 in fp64, takes 140 KB)
    code = sig.SIG_F32 if dtype == np.float32 else sig.SIG_F64
    assert sig.sig_log_backward_workspace_bytes(rows, d, N, code) == 0
    x = orc.signature(1.3 * brownian_paths(rows, 7, d, seed=rows + d + N), N).astype(dtype)
    g = np.random.default_rng(rows + N).standard_normal(x.shape).astype(dtype)
    got = host(sig.sig_log_backward(dev(x), dev(g), d, N))
    want = orc.tensor_log_backward(x, g, d, N)
    scale = orc.tensor_log_backward(-np.abs(x.astype(np.float64)), np.abs(g.astype(np.float64)), d, N)
    assert_grad_close(got, want, scale, d, N, dtype)
    for r in range(0, rows, 17):
        assert_grad_close(got[r:r + 1], want[r:r + 1], scale[r:r + 1], d, N, dtype)


@pytest.mark.parametrize("dtype", [np.float32, np.float64], ids=["float32", "float64"])
@pytest.mark.parametrize("rows", [1024, 256])
def test_benchmark_shape_every_row(rows, dtype):
    """d = 4, N = 6 at 1024 rows is what `bench.py --op logsignature_backward` times: one launch, with 61 KB of LDS per
    signature in fp32 and 140 KB in fp64.  Every row against the oracle, batch-wide and row by row."""
    w = WORKLOADS[1]
    code = sig.SIG_F32 if dtype == np.float32 else sig.SIG_F64
    need = sig.sig_log_backward_workspace_bytes(rows, w.d, w.N, code)
    assert need == 0
    x = orc.signature(workload_paths(w)[:rows], w.N).astype(dtype)
    g = np.random.default_rng(w.seed).standard_normal(x.shape).astype(dtype)
    got = host(sig.sig_log_backward(dev(x), dev(g), w.d, w.N))
    want = orc.tensor_log_backward(x, g, w.d, w.N)
    scale = orc.tensor_log_backward(-np.abs(x.astype(np.float64)), np.abs(g.astype(np.float64)), w.d, w.N)
    assert_grad_close(got, want, scale, w.d, w.N, dtype)
    for r in range(0, rows, 29):
        assert_grad_close(got[r:r + 1], want[r:r + 1], scale[r:r + 1], w.d, w.N, dtype)


def test_logsignature_gradient_on_the_benchmark_shape():
    """The whole gradient of the logsignature (scatter, logarithm, signature) with respect to the path on all 1024
    paths of d = 4, N = 6, L = 128, in fp32, against the oracle's."""
    import torch
    w = WORKLOADS[1]
    x = workload_paths(w)
    n_words = len(orc.lyndon_indices(w.d, w.N))
    g = np.random.default_rng(w.seed + 1).standard_normal((w.B, n_words)).astype(np.float32)
    p = dev(x).requires_grad_(True)
    sig.logsignature(p, w.N).backward(dev(g))
    got = host(p.grad).astype(np.float64)
    want = orc.logsignature_backward(x, g, w.N)
    err = np.linalg.norm((got - want).reshape(w.B, -1), axis=1)
    den = np.linalg.norm(want.reshape(w.B, -1), axis=1)
    assert np.linalg.norm(err) <= 1e-4 * np.linalg.norm(den), np.linalg.norm(err) / np.linalg.norm(den)
    assert np.max(err / den) <= 5e-4, np.max(err / den)


@pytest.mark.parametrize("stream", [False, True])
@pytest.mark.parametrize("B,L,d,N", [(3, 7, 2, 5), (2, 6, 3, 4), (2, 9, 4, 4)])
def test_logsignature_is_differentiable_in_the_path(B, L, d, N, stream):
    import torch
    x = brownian_paths(B, L, d, seed=L + N).astype(np.float64)
    n_inc = L - 1
    w = len(orc.lyndon_indices(d, N))
    g = np.random.default_rng(5).standard_normal((B, n_inc, w) if stream else (B, w))
    p = dev(x).requires_grad_(True)
    out = sig.logsignature(p, N, stream=stream)
    np.testing.assert_allclose(host(out.detach()), orc.logsignature(x, N, stream=stream), rtol=0, atol=1e-11)
    out.backward(dev(g))
    want = orc.logsignature_backward(x, g, N, stream=stream)
    np.testing.assert_allclose(host(p.grad), want, rtol=1e-9, atol=1e-10)


def test_gradcheck_through_the_logsignature_in_both_modes():
    import torch
    x = dev(brownian_paths(2, 5, 2, seed=9).astype(np.float64)).requires_grad_(True)
    assert torch.autograd.gradcheck(lambda p: sig.logsignature(p, 4), (x,), eps=1e-6, atol=1e-7, rtol=1e-6)
    assert torch.autograd.gradcheck(lambda p: sig.logsignature(p, 3, stream=True, mode="expand"), (x,), eps=1e-6,
                                    atol=1e-7, rtol=1e-6)
    s = dev(orc.signature(brownian_paths(2, 5, 2, seed=9), 3)).requires_grad_(True)
    assert torch.autograd.gradcheck(lambda t: sig.signature_to_logsignature(t, 2, 3), (s,), eps=1e-6, atol=1e-7,
                                    rtol=1e-6)
