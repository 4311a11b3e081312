"""Parity of `sig_backward` (HIP, through the C ABI) with the fp64 CPU oracle's gradient.

Error measure: e = ||g_gpu - g_oracle||_2 / ||g_oracle||_2 over the whole gradient tensor (and the
worst single path).  Bars: fp32 1e-4, fp64 1e-9: the backward pass first undoes the forward increments
one by one in the working precision (appendix C.1, reversibility), so its rounding error is that of
two scans of the path; measured values are around 1e-6 and 1e-15.
"""
import numpy as np
import pytest

import paper_2001_00706_amd as sig
from oracle import sig_oracle as orc
from paper_2001_00706_amd.inputs import WORKLOADS, brownian_paths, uniform_paths, workload_paths

pytestmark = pytest.mark.gpu

TOL = {np.float32: 1e-4, np.float64: 1e-9}
TOL_SINGLE = {np.float32: 5e-4, np.float64: 5e-9}


def out_shape(B, L, d, N, stream, basepoint):
    S = sig.sig_signature_channels(d, N)
    n_inc = L if basepoint else L - 1
    return (B, n_inc, S) if stream else (B, S)


def gpu_backward(x, g, N, stream, basepoint, misalign=False):
    import torch
    xt = torch.from_numpy(np.ascontiguousarray(x)).to("cuda:0")
    gt = torch.from_numpy(np.ascontiguousarray(g)).to("cuda:0")
    if misalign:   # an output gradient that starts 4 bytes off a 16-byte boundary: the vector-loading kernels step aside
        holder = torch.empty(gt.numel() + 1, dtype=gt.dtype, device=gt.device)
        holder[1:].copy_(gt.reshape(-1))
        gt = holder[1:].view(gt.shape)
    st = sig.sig_forward(xt, N, stream=stream, basepoint=basepoint)
    gp = torch.full_like(xt, float("nan"))
    sig.sig_backward(xt, st, gt, N, stream=stream, basepoint=basepoint, grad_path=gp)
    torch.cuda.synchronize()
    return gp.cpu().numpy()


def check(x, N, stream=False, basepoint=False, sample=None, seed=0, misalign=False):
    dt = x.dtype.type
    B, L, d = x.shape
    rng = np.random.default_rng(seed + 31 * L + d + N)
    g = rng.standard_normal(out_shape(B, L, d, N, stream, basepoint)).astype(dt)
    got = gpu_backward(x, g, N, stream, basepoint, misalign)
    assert np.all(np.isfinite(got)), "gradient not fully written"
    idx = np.arange(B) if sample is None else np.asarray(sample)
    want = orc.signature_backward(x[idx], g[idx], N, stream, basepoint)
    diff = got[idx].astype(np.float64) - want
    den = np.linalg.norm(want)
    assert np.linalg.norm(diff) <= TOL[dt] * (den if den > 0 else 1.0), np.linalg.norm(diff) / den
    dens = np.linalg.norm(want.reshape(len(idx), -1), axis=1)
    dens[dens == 0] = 1.0
    single = np.linalg.norm(diff.reshape(len(idx), -1), axis=1) / dens
    assert single.max() <= TOL_SINGLE[dt], single.max()
    return got


SWEEP = [
    # (B, L, d, N)
    (1, 2, 1, 1), (3, 2, 1, 5), (2, 40, 1, 3), (2, 5, 2, 1), (5, 3, 2, 2), (4, 17, 3, 4), (2, 9, 5, 3), (3, 6, 7, 3),
    (2, 33, 2, 7), (1, 4, 6, 4), (7, 12, 4, 4), (2, 5, 9, 2), (3, 20, 3, 5), (2, 11, 4, 6), (5, 9, 8, 3),
    (2, 7, 16, 3), (1, 3, 33, 2), (2, 4, 64, 1), (2, 3, 64, 2), (1, 5, 22, 2), (2, 6, 17, 3),
]


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("B,L,d,N", SWEEP)
def test_shape_sweep(B, L, d, N, dtype):
    x = uniform_paths(B, L, d, seed=2000 + 7 * L + d, lo=-0.5, hi=0.5).astype(dtype)
    for stream in (False, True):
        for basepoint in (False, True):
            check(x, N, stream=stream, basepoint=basepoint)


POW2 = [(2, N) for N in range(2, 10)] + [(8, N) for N in range(2, 6)] + [(4, 4), (4, 5), (4, 6)]


@pytest.mark.parametrize("d,N", POW2)
def test_register_resident_kernels_every_depth(d, N):
    # fp32, d = 2, 4, 8: a thread per word, cotangents summed over siblings with lane exchanges
    x = brownian_paths(3, 70, d, seed=10 * d + N)      # 69 increments: two tiles, the first one ragged
    for stream in (False, True):
        for basepoint in (False, True):
            check(x, N, stream=stream, basepoint=basepoint)


def test_final_mode_families_on_both_sides_of_their_batch_thresholds():
    # with one gradient per path the prefix-tree kernels serve every shape but d = 4 at N >= 5 below 512 paths
    check(brownian_paths(520, 6, 2, seed=3), 9, sample=[0, 1, 255, 519])
    check(brownian_paths(8, 6, 2, seed=4), 9)
    check(brownian_paths(515, 7, 4, seed=5), 5, sample=[0, 300, 514])
    check(brownian_paths(515, 5, 4, seed=6), 6, basepoint=True, sample=[1, 2, 513])
    check(brownian_paths(5, 70, 4, seed=7), 6)


@pytest.mark.parametrize("B,L,d,N", [
    (2, 6, 7, 7),      # 16 807 threads per path over 66 workgroups, 960 799 scalars per signature
    (2, 8, 4, 9), (2, 10, 4, 8), (2, 9, 4, 7), (3, 40, 3, 7), (2, 12, 5, 7), (2, 9, 6, 7), (2, 70, 5, 4),
    (37, 6, 3, 4),     # 9 threads per path: 16 paths share a workgroup, the last workgroup is ragged
    (5, 5, 7, 2), (3, 7, 6, 3), (4, 9, 3, 2),
    # 9 to 16 channels (one level per thread below its word), depths 2..6
    (3, 9, 9, 2), (20, 7, 16, 2), (2, 40, 16, 3), (3, 9, 10, 4), (2, 6, 16, 4), (2, 5, 11, 5), (1, 4, 9, 6), (2, 70, 13, 3),
])
def test_prefix_tree_kernels(B, L, d, N):
    # fp32 shapes that neither the d = 4 nor the power-of-two register kernels serve
    x = brownian_paths(B, L, d, seed=B + L + d + N)
    for stream in (False, True):
        if stream and d ** N > 100000:
            continue   # the stream output of the largest shapes would only slow the oracle down
        for basepoint in (False, True):
            check(x, N, stream=stream, basepoint=basepoint)


@pytest.mark.parametrize("d,N", [(2, 3), (2, 9), (4, 5), (4, 6), (8, 3), (8, 5)])
def test_prefix_tree_kernels_on_unaligned_buffers(d, N):
    # the same shapes the register kernels serve, pushed to the prefix-tree kernels by a misaligned buffer
    x = brownian_paths(3, 40, d, seed=d + N)
    for stream in (False, True):
        check(x, N, stream=stream, basepoint=stream, misalign=True)


def test_prefix_tree_kernels_wide_in_fp64():
    for B, L, d, N in [(2, 9, 16, 3), (3, 6, 10, 4), (5, 7, 12, 2)]:
        x = brownian_paths(B, L, d, seed=B + d).astype(np.float64)
        check(x, N)
        check(x, N, stream=True, basepoint=True)


def tree_gradient_shapes(max_scalars):
    """Every (d, N) the prefix-tree gradient kernels are instantiated for (d = 2..8 to depth 9, d = 9..16 to depth
    6), up to signatures of `max_scalars` scalars."""
    return [(d, N) for d in range(2, 17) for N in range(2, (9 if d <= 8 else 6) + 1)
            if sig.sig_signature_channels(d, N) <= max_scalars]


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("stream", [False, True], ids=["final", "stream"])
def test_tree_gradient_every_shape(dtype, stream):
    """One instantiation of the prefix-tree gradient kernels per (d, N), mode and precision, some at 350 and more
    registers per lane: every one of them on two paths of three points (two increments: the last one and the first
    one, which in stream mode takes the identity for the signature before it), misaligned so that no other family
    takes the call.  In fp64 stream mode at d = 4, N = 8; d = 5, N = 7; d = 6, N = 6 and d = 8, N = 6 the first
    increment once lost the cotangent of the levels above a thread's word."""
    for d, N in tree_gradient_shapes(3_000_000):
        x = uniform_paths(2, 3, d, seed=100 * d + N, lo=-0.4, hi=0.4).astype(dtype)
        check(x, N, stream=stream, misalign=True)


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_more_paths_than_compute_units(dtype):
    x = brownian_paths(515, 9, 3, seed=77).astype(dtype)
    check(x, 4, sample=[0, 1, 100, 513, 514])
    check(x, 3, stream=True, basepoint=True, sample=[0, 255, 514])


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_working_set_in_global_memory(dtype):
    # d = 9, N = 5: 66 429 scalars per signature; the generic kernel's arena does not fit on chip and lives in the
    # workspace
    B, L, d, N = 3, 6, 9, 5
    dt = sig.SIG_F32 if dtype == np.float32 else sig.SIG_F64
    assert sig.sig_backward_workspace_bytes(B, L, d, N, False, False, dt) > 0
    x = brownian_paths(B, L, d, seed=5).astype(dtype)
    check(x, N)
    check(x, N, stream=True)


def test_more_paths_than_persistent_workgroups_in_global_memory():
    # 1030 paths over 1024 workgroups: some workgroups scan two paths with the same arena
    B, L, d, N = 1030, 3, 16, 4   # the generic kernel (d > 8)
    assert sig.sig_backward_workspace_bytes(B, L, d, N, False, False, sig.SIG_F32) > 0
    x = brownian_paths(B, L, d, seed=6)
    check(x, N, sample=[0, 5, 1023, 1024, 1029])


def test_large_lds_arena_fp64_depth_six():
    # d = 4, N = 6 in fp64 needs about 118 KB of LDS per workgroup (above the 64 KB default) when it fits at all
    x = brownian_paths(4, 20, 4, seed=9).astype(np.float64)
    check(x, 6)
    check(x, 6, stream=True, basepoint=True)


def test_missing_or_short_workspace_is_refused():
    import torch
    B, L, d, N = 2, 4, 9, 5
    need = sig.sig_backward_workspace_bytes(B, L, d, N, False, False, sig.SIG_F32)
    assert need > 0
    x = torch.zeros((B, L, d), device="cuda:0")
    s = sig.sig_forward(x, N)
    g = torch.zeros_like(s)
    small = torch.empty(need - 1, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(sig.SigError) as e:
        sig.sig_backward(x, s, g, N, workspace=small)
    assert e.value.status == sig.SIG_ERR_INVALID_ARG
    exact = torch.empty(need, dtype=torch.uint8, device="cuda:0")
    out = sig.sig_backward(x, s, g, N, workspace=exact)
    torch.cuda.synchronize()
    assert torch.all(out == 0)


def test_short_workspace_of_the_prefix_tree_kernels_is_refused():
    import torch
    B, L, d, N = 3, 12, 3, 5
    need = sig.sig_backward_workspace_bytes(B, L, d, N, False, False, sig.SIG_F32)
    assert need == B * 27 * (L - 1) * d * 4          # one partial sum per thread (27 three-letter words), increment, channel
    x = torch.from_numpy(brownian_paths(B, L, d, seed=1)).to("cuda:0")
    s = sig.sig_forward(x, N)
    with pytest.raises(sig.SigError) as e:
        sig.sig_backward(x, s, torch.ones_like(s), N, workspace=torch.empty(need - 4, dtype=torch.uint8, device="cuda:0"))
    assert e.value.status == sig.SIG_ERR_INVALID_ARG


# ---- depth 2 in final mode: the closed form (no scan), any channel count up to 122 (85 in fp64)
@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("B,L,d", [(3, 2, 5), (2, 3, 1), (4, 40, 32), (1, 300, 7), (2, 9, 100), (5, 17, 16), (2, 130, 64), (3, 5, 85),
                                   (2, 260, 3),
                                   # fp32 from 8 channels on: the matrix-core kernel; two points only, several workgroups
                                   # per path, several rounds per workgroup, rounds of 16 points
                                   (3, 2, 24), (2, 700, 40), (1200, 200, 9), (2, 50, 112), (3, 3, 8)])
def test_depth_two_gradient_by_its_closed_form(B, L, d, dtype):
    import torch
    if d >= 100 and dtype == np.float64:   # 100 x 101 doubles do not fit the LDS, and no other fp64 gradient kernel takes them
        assert sig.sig_backward_workspace_bytes(B, L, d, 2, False, False, sig.SIG_F64) == -1
        return
    x = (brownian_paths(B, L, d, seed=L + d) + 0.3).astype(dtype)
    for basepoint in (False, True):
        check(x, 2, basepoint=basepoint, seed=d)
    # a basepoint given by value, and its own gradient
    bp = uniform_paths(B, 1, d, seed=d + 1)[:, 0].astype(dtype)
    g = np.random.default_rng(d).standard_normal((B, d + d * d)).astype(dtype)
    to_dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")
    xt, bt = to_dev(x), to_dev(bp)
    st = sig.sig_signature(xt, 2, basepoint=bt)
    gb = torch.full_like(bt, float("nan"))
    gp = sig.sig_backward(xt, st, to_dev(g), 2, basepoint=bt, grad_basepoint=gb)
    torch.cuda.synchronize()
    want = orc.signature_backward(np.concatenate([bp[:, None], x], axis=1).astype(np.float64), g.astype(np.float64), 2)
    tol = 1e-4 if dtype == np.float32 else 1e-9
    assert np.linalg.norm(gp.cpu().numpy() - want[:, 1:]) <= tol * np.linalg.norm(want)
    assert np.linalg.norm(gb.cpu().numpy() - want[:, 0]) <= tol * np.linalg.norm(want)


@pytest.mark.parametrize("B,L,d", [(3, 200, 3), (2, 150, 12), (2, 100, 64)])
def test_depth_two_gradient_far_from_the_origin(B, L, d):
    # as for the forward pass: only differences of points may enter, a path around 10 000 loses nothing
    x = (brownian_paths(B, L, d, seed=L + d) + 10000.0).astype(np.float32)
    check(x, 2, seed=d)


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("B,L,d,N", [
    (2, 9, 17, 3), (1, 40, 20, 3),    # a last block of one letter; three tiles of increments
    (3, 5, 33, 2), (1, 6, 70, 2),     # depth 2 (stream mode; final mode has its closed form): 3 and 5 blocks of letters
    (2, 7, 40, 3), (1, 4, 18, 4),     # 75 and 365 wavefronts per path
    (3, 20, 12, 3), (2, 6, 9, 4),     # final mode from 9 channels on at few paths: picked over the prefix-tree kernels
    (2, 5, 17, 5), (1, 3, 9, 7),      # deeper
    (1, 4, 14, 5),                    # final mode at depths 5 and 6 from 13 channels on: picked over the prefix-tree kernels
])
def test_many_channels_at_low_depth(B, L, d, N, dtype):
    x = uniform_paths(B, L, d, seed=4000 + L + d, lo=-0.4, hi=0.4).astype(dtype)
    code = sig.SIG_F32 if dtype == np.float32 else sig.SIG_F64
    for stream in (False, True):
        assert sig.sig_backward_workspace_bytes(B, L, d, N, stream, False, code) >= 0
        for basepoint in (False, True):
            check(x, N, stream=stream, basepoint=basepoint)


def test_unsupported_and_invalid_arguments():
    import torch
    x = torch.zeros((1, 3, 65), device="cuda:0")
    s = sig.sig_forward(x, 1)
    with pytest.raises(sig.SigError) as e:
        sig.sig_backward(x, s, torch.zeros_like(s), 1)
    assert e.value.status == sig.SIG_ERR_UNSUPPORTED
    assert sig.sig_backward_workspace_bytes(1, 3, 65, 1, False, False, sig.SIG_F32) == -1
    assert sig.sig_backward_workspace_bytes(1, 1, 2, 2, False, False, sig.SIG_F32) == -1   # one point, no basepoint
    assert sig.sig_backward_workspace_bytes(0, 5, 2, 2, False, False, sig.SIG_F32) == 0


def test_empty_batch_and_single_point_with_basepoint():
    import torch
    x = torch.zeros((0, 4, 3), device="cuda:0")
    s = sig.sig_forward(x, 3)
    assert sig.sig_backward(x, s, torch.zeros_like(s), 3).shape == (0, 4, 3)
    xs = uniform_paths(3, 1, 2, seed=1).astype(np.float64)
    check(xs, 4, basepoint=True)
    check(xs, 4, basepoint=True, stream=True)


def test_zero_increments_and_repeated_points():
    x = brownian_paths(2, 8, 3, seed=12).astype(np.float64)
    x[:, 3] = x[:, 2]
    x[:, 6] = x[:, 5]
    check(x, 4)
    check(np.zeros((2, 5, 3)), 3, stream=True)


@pytest.mark.parametrize("B,L,d,N", [(6, 30, 4, 5), (3, 40, 20, 3)])   # the second: sums through LDS atomic adds
def test_deterministic_and_inputs_untouched(B, L, d, N):
    import torch
    x = torch.from_numpy(brownian_paths(B, L, d, seed=3)).to("cuda:0")
    s = sig.sig_forward(x, N)
    g = torch.randn_like(s)
    x0, s0, g0 = x.clone(), s.clone(), g.clone()
    a = sig.sig_backward(x, s, g, N).clone()
    for _ in range(3):
        b = sig.sig_backward(x, s, g, N)
        torch.cuda.synchronize()
        assert torch.equal(a, b)
    assert torch.equal(x, x0) and torch.equal(s, s0) and torch.equal(g, g0)


@pytest.mark.parametrize("dtype", [np.float32, np.float64], ids=["float32", "float64"])
@pytest.mark.parametrize("w", WORKLOADS[:4], ids=lambda w: w.name)
def test_benchmark_workloads_full_size_every_path(w, dtype):
    """The shapes of the first four forward workloads at full size, as `bench.py --op backward` launches them: the
    gradient of every path is compared with the oracle's, element by element."""
    check(workload_paths(w).astype(dtype), w.N, stream=w.stream, basepoint=w.basepoint)


@pytest.mark.parametrize("dtype", [np.float32, np.float64], ids=["float32", "float64"])
def test_largest_workload_full_size(dtype):
    """d = 16, N = 4, 256 paths of 1024 points (1023 increments undone one after the other, appendix C.1).  The
    oracle's stored-forward gradient of this shape costs about 1.5 core-minutes per path, so it recomputes 16 whole
    paths spread over the launch; EVERY path is then checked through a property that holds at any size: the
    derivative of <g, Sig(x + t u)> at t = 0, which is <grad, u>, against central differences of the oracle's
    (pinned) forward pass in fp64."""
    w = WORKLOADS[4]
    x = workload_paths(w).astype(dtype)
    sample = np.unique(np.concatenate([[0, 1, w.B // 2, w.B - 2, w.B - 1],
                                       np.random.default_rng(w.seed).choice(w.B, size=11, replace=False)]))
    got = check(x, w.N, sample=sample).astype(np.float64)
    rng = np.random.default_rng(31 * w.L + w.d + w.N)          # the output gradient `check` drew
    g = rng.standard_normal(out_shape(w.B, w.L, w.d, w.N, False, False)).astype(dtype).astype(np.float64)
    u = brownian_paths(w.B, w.L, w.d, seed=w.seed + 1000).astype(np.float64)
    h = 1e-3
    x64 = x.astype(np.float64)
    hi = np.einsum("bs,bs->b", g, orc.signature(x64 + h * u, w.N))
    lo = np.einsum("bs,bs->b", g, orc.signature(x64 - h * u, w.N))
    want = (hi - lo) / (2 * h)
    have = np.einsum("bld,bld->b", got, u)
    scale = np.sqrt(np.mean(want ** 2))
    assert np.max(np.abs(have - want)) <= 2e-3 * scale, (np.max(np.abs(have - want)), scale)


def test_long_path_reversibility_error_stays_small():
    # 1023 increments undone one after the other in fp32
    x = brownian_paths(2, 1024, 3, seed=21)
    check(x, 4)


@pytest.mark.parametrize("stream,basepoint", [(False, False), (True, False), (False, True), (True, True)])
def test_autograd_function_passes_gradcheck(stream, basepoint):
    # finite differences of the HIP forward against the HIP backward, in fp64, on the GPU
    import torch
    x = torch.from_numpy(uniform_paths(2, 5, 3, seed=4).astype(np.float64)).to("cuda:0").requires_grad_(True)
    assert torch.autograd.gradcheck(lambda p: sig.signature(p, 3, stream, basepoint), (x,), eps=1e-6, atol=1e-7, rtol=1e-6)


def test_autograd_sum_backward_as_in_the_papers_example():
    # the usage pattern of the code-example section (section 3): signature(path, depth).sum().backward()
    import torch
    x_host = brownian_paths(4, 12, 3, seed=8)
    x = torch.from_numpy(x_host).to("cuda:0").requires_grad_(True)
    sig.signature(x, 4).sum().backward()
    torch.cuda.synchronize()
    want = orc.signature_backward(x_host, np.ones((4, sig.sig_signature_channels(3, 4))), 4)
    got = x.grad.cpu().numpy()
    assert np.linalg.norm(got - want) <= 1e-4 * np.linalg.norm(want)


def test_a_training_step_can_be_captured_in_a_graph_and_replayed():
    # forward, logarithm, group product and all three gradients in one HIP graph: none of the calls allocates,
    # synchronises or memsets; every replay is checked against the same calls made eagerly
    import torch
    x_host = brownian_paths(8, 40, 4, seed=17)
    x = torch.from_numpy(x_host).to("cuda:0")
    N = 5
    S = sig.sig_signature_channels(4, N)
    s = torch.empty((8, S), device="cuda:0")
    lg = torch.empty_like(s)
    prod = torch.empty_like(s)
    g = torch.from_numpy(np.random.default_rng(2).standard_normal((8, S)).astype(np.float32)).to("cuda:0")
    gp = torch.empty_like(x)
    g_words = torch.from_numpy(np.random.default_rng(3).standard_normal((8, sig.sig_logsignature_channels(4, N)))
                               .astype(np.float32)).to("cuda:0")
    g_log, g_sig, g_a, g_b = (torch.empty_like(s) for _ in range(4))
    ws = torch.empty(max(sig.sig_log_backward_workspace_bytes(8, 4, N), sig.sig_combine_backward_workspace_bytes(8, 4, N)),
                     dtype=torch.uint8, device="cuda:0")

    def step():
        sig.sig_forward(x, N, out=s)
        sig.sig_log(s, 4, N, out=lg)
        sig.sig_backward(x, s, g, N, grad_path=gp)
        sig.sig_combine(s, s, 4, N, out=prod)
        sig.sig_lyndon_scatter(g_words, 4, N, out=g_log)
        sig.sig_log_backward(s, g_log, 4, N, out=g_sig, workspace=ws)
        sig.sig_combine_backward(s, lg, g, 4, N, grad_a=g_a, grad_b=g_b, workspace=ws)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                   # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(3):
        x.copy_(torch.from_numpy(x_host * (1.0 + 0.5 * rep)).to("cuda:0"))
        for t in (s, lg, gp, prod, g_log, g_sig, g_a, g_b):
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = [t.clone() for t in (s, lg, gp, prod, g_log, g_sig, g_a, g_b)]
        step()
        torch.cuda.synchronize()
        for a, b in zip(got, (s, lg, gp, prod, g_log, g_sig, g_a, g_b)):
            assert torch.equal(a, b), rep
