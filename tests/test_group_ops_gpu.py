"""GPU parity of the options built on top of the scan (paper sections 4.2, 5.4, 5.5): a basepoint
given by value, `initial`, `inverse`, inverses of stored signatures, strided products and `Path`.

Every expected value comes from the fp64 oracle applied to a path that spells the option out:
the basepoint prepended as a point, the earlier data concatenated in front, the path reversed.
"""
import numpy as np
import pytest

import paper_2001_00706_amd as sig
from oracle import sig_oracle as orc
from paper_2001_00706_amd.inputs import brownian_paths, uniform_paths

pytestmark = pytest.mark.gpu

TOL = {np.float32: 1e-4, np.float64: 1e-10}


def dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def host(t):
    import torch
    torch.cuda.synchronize()
    return t.cpu().numpy()


def assert_levels_close(got, want, d, N, dt):
    got = np.asarray(got, dtype=np.float64)
    for sl in orc.level_slices(d, N):
        den = np.linalg.norm(want[..., sl])
        err = np.linalg.norm(got[..., sl] - want[..., sl]) / (den if den > 0 else 1.0)
        assert err <= TOL[dt], err


def reversed_prefix_signatures(x, N):
    """Inverted signature of every prefix = signature of the prefix traversed backwards (section 5.4)."""
    B, L, d = x.shape
    out = np.empty((B, L - 1, orc.channels(d, N)))
    for j in range(2, L + 1):
        out[:, j - 2] = orc.signature(x[:, :j][:, ::-1], N)
    return out


# shapes chosen to reach every kernel family: d=4 N=6 (one wavefront per path), d=4 N=5 stream and N=7 (four
# per path), d=8 N=5, d=16 N=4, a small state, and the fallback
FAMILY_SHAPES = [(5, 9, 4, 6), (3, 20, 4, 7), (2, 7, 8, 5), (2, 5, 16, 4), (4, 11, 2, 5), (3, 8, 5, 4), (2, 6, 3, 6)]


@pytest.mark.parametrize("stream", [False, True])
@pytest.mark.parametrize("B,L,d,N", FAMILY_SHAPES)
def test_basepoint_given_by_value(B, L, d, N, stream):
    x = brownian_paths(B, L, d, seed=L + d) + 0.25
    bp = uniform_paths(B, 1, d, seed=N)[:, 0]
    got = host(sig.sig_signature(dev(x), N, stream=stream, basepoint=dev(bp)))
    want = orc.signature(np.concatenate([bp[:, None], x], axis=1), N, stream=stream)
    assert_levels_close(got, want, d, N, np.float32)


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("stream", [False, True])
@pytest.mark.parametrize("B,L,d,N", [(3, 9, 4, 5), (2, 6, 3, 4), (2, 5, 8, 4), (4, 7, 2, 6)])
def test_initial_continues_an_earlier_signature(B, L, d, N, stream, dtype):
    # earlier data y (ending where x begins) then x: initial = Sig(y); the result is the signature of everything
    whole = brownian_paths(B, L + 5, d, seed=3 * L + d).astype(dtype)
    y, x = whole[:, :6], whole[:, 5:]
    initial = orc.signature(y, N).astype(dtype)
    got = host(sig.sig_signature(dev(x), N, stream=stream, initial=dev(initial)))
    if stream:
        want = orc.signature(whole, N, stream=True)[:, 5:]
    else:
        want = orc.signature(whole, N)
    assert_levels_close(got, want, d, N, dtype)
    # the same through a basepoint: x without its first point, that point given as the basepoint
    got = host(sig.sig_signature(dev(x[:, 1:]), N, stream=stream, basepoint=dev(x[:, 0]), initial=dev(initial)))
    assert_levels_close(got, want, d, N, dtype)


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("B,L,d,N", [(3, 9, 4, 5), (2, 6, 3, 4), (2, 5, 7, 3), (4, 7, 2, 7), (2, 4, 1, 5), (3, 5, 6, 1)])
def test_inverse_is_the_signature_of_the_reversed_path(B, L, d, N, dtype):
    x = uniform_paths(B, L, d, seed=L * d + N).astype(dtype)
    got = host(sig.sig_signature(dev(x), N, inverse=True))
    assert_levels_close(got, orc.signature(x[:, ::-1], N), d, N, dtype)
    got = host(sig.sig_signature(dev(x), N, stream=True, inverse=True))
    assert_levels_close(got, reversed_prefix_signatures(x.astype(np.float64), N), d, N, dtype)
    # with a basepoint (the origin) the reversed path ends there
    got = host(sig.sig_signature(dev(x), N, basepoint=True, inverse=True))
    x0 = np.concatenate([np.zeros((B, 1, d), dtype=dtype), x], axis=1)
    assert_levels_close(got, orc.signature(x0[:, ::-1], N), d, N, dtype)


def test_invert_in_place_out_of_place_and_twice():
    import torch
    x = brownian_paths(6, 12, 3, seed=4)
    s = sig.sig_forward(dev(x), 5)
    inv = sig.sig_invert(s, 3, 5)
    assert_levels_close(host(inv), orc.signature(x[:, ::-1], 5), 3, 5, np.float32)
    again = sig.sig_invert(inv, 3, 5)
    assert torch.equal(again, s)                      # a signed permutation: exact
    t = s.clone()
    sig.sig_invert(t, 3, 5, out=t)
    assert torch.equal(t, inv)
    # inverse [x] signature = identity (all zeros, the constant term being implicit)
    prod = host(sig.sig_combine(inv, s, 3, 5))
    assert np.abs(prod).max() <= 1e-5


def test_strided_combine_reads_rows_of_stream_outputs():
    x = brownian_paths(4, 10, 4, seed=2).astype(np.float64)
    N, S = 4, orc.channels(4, 4)
    st = sig.sig_forward(dev(x), N, stream=True)           # [4, 9, S]
    inv = sig.sig_invert(st, 4, N)
    import torch
    out = torch.full((4, S + 3), float("nan"), dtype=torch.float64, device="cuda:0")
    # Sig(x_3..x_8) = Sig(x_0..x_3)^{-1} [x] Sig(x_0..x_8): rows 2 and 7 of every path
    sig.sig_combine_strided(inv.reshape(-1)[2 * S:], 9 * S, st.reshape(-1)[7 * S:], 9 * S, 4, 4, N, out, S + 3)
    got = host(out)
    assert_levels_close(got[:, :S], orc.signature(x[:, 3:9], N), 4, N, np.float64)
    assert np.all(np.isnan(got[:, S:]))                      # the gap between output rows is left alone
    # stride 0 repeats one left factor
    one = dev(orc.signature(x[:1, :4], N))
    out2 = torch.empty((4, S), dtype=torch.float64, device="cuda:0")
    sig.sig_combine_strided(one, 0, st.reshape(-1)[7 * S:], 9 * S, 4, 4, N, out2, S)
    want = np.stack([orc.group_mul(orc.signature(x[:1, :4], N)[0], orc.signature(x[b:b + 1, :9], N)[0], 4, N)
                     for b in range(4)])
    assert_levels_close(host(out2), want, 4, N, np.float64)


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("B,n,d,N", [(3, 1, 3, 3), (4, 2, 4, 4), (3, 3, 2, 5), (2, 5, 4, 5), (5, 8, 3, 4), (2, 11, 8, 3),
                                     (1, 37, 5, 3)])
def test_combine_many_joins_adjacent_intervals(B, n, d, N, dtype):
    """Signatures of n consecutive pieces of a path, pieces of different lengths sharing their end points,
    multiplied in order give the signature of the whole path (section 5.5)."""
    rng = np.random.default_rng(B * 100 + n)
    cuts = np.concatenate([[0], np.cumsum(rng.integers(1, 4, size=n))])
    x = brownian_paths(B, int(cuts[-1]) + 1, d, seed=n + d).astype(np.float64)
    pieces = np.stack([orc.signature(x[:, cuts[i]:cuts[i + 1] + 1], N) for i in range(n)], axis=1)   # [B, n, S]
    got = host(sig.sig_combine_many(dev(pieces.astype(dtype)), d, N))
    assert_levels_close(got, orc.signature(x, N), d, N, dtype)


def test_combine_many_keeps_the_order_of_the_factors():
    # the product does not commute: reversing the pieces must change the result
    x = brownian_paths(2, 7, 3, seed=5).astype(np.float64)
    N = 4
    pieces = np.stack([orc.signature(x[:, 2 * i:2 * i + 3], N) for i in range(3)], axis=1)
    fwd = host(sig.sig_combine_many(dev(pieces), 3, N))
    rev = host(sig.sig_combine_many(dev(pieces[:, ::-1]), 3, N))
    want_rev = np.stack([orc.group_mul(orc.group_mul(pieces[b, 2], pieces[b, 1], 3, N), pieces[b, 0], 3, N)
                         for b in range(2)])
    assert_levels_close(rev, want_rev, 3, N, np.float64)
    assert np.linalg.norm(fwd - rev) > 1e-3 * np.linalg.norm(fwd)


def assert_query_close(got, x, i, j, N, dt):
    """A query is a product of two long-prefix signatures whose terms largely cancel (section 4.2 ends with a
    warning about exactly this), so its rounding error scales with the factors, not with the result: per level,
    |error| <= c * sum_m |Sig(x_0..x_i)^{-1}|_m |Sig(x_0..x_j)|_{k-m}, c a few roundings of the working precision."""
    d = x.shape[2]
    want = orc.signature(x[:, i:j + 1], N)
    if i == 0:
        return assert_levels_close(got, want, d, N, dt)
    sl = orc.level_slices(d, N)
    left = orc.signature(x[:, :i + 1][:, ::-1], N)
    right = orc.signature(x[:, :j + 1], N)
    norm = lambda a, k: 1.0 if k == 0 else np.linalg.norm(a[:, sl[k - 1]])
    c = 4e-6 if dt == np.float32 else 1e-14
    for k in range(1, N + 1):
        scale = sum(norm(left, m) * norm(right, k - m) for m in range(k + 1))
        err = np.linalg.norm(np.asarray(got, dtype=np.float64)[:, sl[k - 1]] - want[:, sl[k - 1]])
        assert err <= c * scale, (k, err, scale)


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_path_queries_and_update(dtype):
    B, L, d, N = 3, 14, 3, 4
    x = brownian_paths(B, L + 6, d, seed=11).astype(dtype)
    p = sig.Path(dev(x[:, :L]), N)
    assert p.length == L
    for i, j in [(0, L - 1), (0, 1), (3, 4), (2, 9), (L - 2, L - 1), (5, L - 1)]:
        assert_query_close(host(p.signature(i, j)), x, i, j, N, dtype)
    p.update(dev(x[:, L:L + 4]))
    p.update(dev(x[:, L + 4:]))
    assert p.length == L + 6
    for i, j in [(0, L + 5), (4, L + 2), (L - 1, L), (L + 1, L + 5)]:
        assert_query_close(host(p.signature(i, j)), x, i, j, N, dtype)
    with pytest.raises(ValueError):
        p.signature(5, 5)


@pytest.mark.parametrize("stream", [False, True])
def test_backward_with_a_basepoint_value_and_its_gradient(stream):
    import torch
    B, L, d, N = 3, 7, 3, 4
    x = brownian_paths(B, L, d, seed=5).astype(np.float64) + 0.1
    bp = uniform_paths(B, 1, d, seed=6)[:, 0].astype(np.float64)
    S = orc.channels(d, N)
    g = np.random.default_rng(1).standard_normal((B, L, S) if stream else (B, S))
    xt, bt = dev(x), dev(bp)
    s = sig.sig_signature(xt, N, stream=stream, basepoint=bt)
    gb = torch.empty_like(bt)
    gp = sig.sig_backward(xt, s, dev(g), N, stream=stream, basepoint=bt, grad_basepoint=gb)
    want = orc.signature_backward(np.concatenate([bp[:, None], x], axis=1), g, N, stream=stream)
    np.testing.assert_allclose(host(gp), want[:, 1:], rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(host(gb), want[:, 0], rtol=1e-9, atol=1e-11)


def test_autograd_through_inverse_and_basepoint_value():
    import torch
    x = dev(uniform_paths(2, 5, 2, seed=9).astype(np.float64)).requires_grad_(True)
    bp = dev(uniform_paths(2, 1, 2, seed=10)[:, 0].astype(np.float64)).requires_grad_(True)
    assert torch.autograd.gradcheck(lambda p, q: sig.signature(p, 3, True, q, True), (x, bp), eps=1e-6, atol=1e-7, rtol=1e-6)
    assert torch.autograd.gradcheck(lambda p: sig.signature(p, 4, False, False, True), (x,), eps=1e-6, atol=1e-7, rtol=1e-6)


# ---- gradient of the group product ---------------------------------------------------------------------------------

@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("B,d,N", [(3, 2, 9), (2, 2, 10), (4, 3, 6), (5, 4, 5), (2, 7, 4), (3, 1, 4), (2, 5, 1), (3, 4, 2),
                                   (2, 8, 4), (2, 9, 3)])
def test_gradient_of_the_group_product(B, d, N, dtype):
    rng = np.random.default_rng(B + 10 * d + 100 * N)
    a = orc.signature(brownian_paths(B, 6, d, seed=d + N), N).astype(dtype)
    b = orc.signature(brownian_paths(B, 7, d, seed=d * N), N).astype(dtype)
    g = rng.standard_normal(a.shape).astype(dtype)
    ga, gb = sig.sig_combine_backward(dev(a), dev(b), dev(g), d, N)
    want = [orc.group_mul_backward(a[i], b[i], g[i], d, N) for i in range(B)]
    # every term of the gradient is a product of one cotangent with one factor: the yardstick is that sum with
    # absolute values
    scale = [orc.group_mul_backward(np.abs(a[i]), np.abs(b[i]), np.abs(g[i]), d, N) for i in range(B)]
    tol = 1e-5 if dtype == np.float32 else 1e-13
    for got, k in ((host(ga), 0), (host(gb), 1)):
        w = np.stack([t[k] for t in want])
        sc = np.stack([t[k] for t in scale])
        for sl in orc.level_slices(d, N):
            assert np.linalg.norm(got[:, sl] - w[:, sl]) <= tol * np.linalg.norm(sc[:, sl])


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("B,group,d,N", [(3, 5, 2, 6), (2, 9, 4, 5), (4, 1, 3, 4), (1, 37, 4, 6), (2, 3, 8, 4), (3, 4, 5, 1),
                                         (2, 6, 7, 2), (130, 2, 2, 3)])
def test_one_left_factor_for_a_group_of_right_factors_and_its_gradient(B, group, d, N, dtype):
    # what `initial` does to a stream-mode output: row (b, s) is a[b] [x] sigs[b, s]; the oracle does every product
    # on its own and the gradients of the shared factor are added up here
    rng = np.random.default_rng(B + 10 * d + 100 * N + group)
    S = orc.channels(d, N)
    a = orc.signature(brownian_paths(B, 6, d, seed=d + N), N).astype(dtype)
    sigs = orc.signature(brownian_paths(B * group, 5, d, seed=d * N + 1), N).astype(dtype).reshape(B, group, S)
    g = rng.standard_normal(sigs.shape).astype(dtype)
    got = host(sig.sig_combine_grouped(dev(a), dev(sigs), d, N))
    want = np.stack([np.stack([orc.group_mul(a[b], sigs[b, s], d, N) for s in range(group)]) for b in range(B)])
    assert_levels_close(got, want, d, N, dtype)
    # in place
    buf = dev(sigs.copy())
    assert sig.sig_combine_grouped(dev(a), buf, d, N, out=buf) is buf
    np.testing.assert_array_equal(host(buf), got)

    ga, gs = sig.sig_combine_grouped_backward(dev(a), dev(sigs), dev(g), d, N)
    ga, gs = host(ga), host(gs)
    tol = 1e-5 if dtype == np.float32 else 1e-13
    want_a, want_s = np.zeros((B, S)), np.zeros((B, group, S))
    scale_a, scale_s = np.zeros((B, S)), np.zeros((B, group, S))
    for b in range(B):
        for s in range(group):
            wa, ws = orc.group_mul_backward(a[b], sigs[b, s], g[b, s], d, N)
            sa, ss = orc.group_mul_backward(np.abs(a[b]), np.abs(sigs[b, s]), np.abs(g[b, s]), d, N)
            want_a[b] += wa
            scale_a[b] += sa
            want_s[b, s], scale_s[b, s] = ws, ss
    for sl in orc.level_slices(d, N):
        assert np.linalg.norm(ga[:, sl] - want_a[:, sl]) <= tol * np.linalg.norm(scale_a[:, sl])
        assert np.linalg.norm(gs[..., sl] - want_s[..., sl]) <= tol * np.linalg.norm(scale_s[..., sl])


def test_grouped_product_argument_errors():
    import torch
    d, N = 3, 3
    S = orc.channels(d, N)
    a = torch.zeros(2, S, device="cuda:0")
    sigs = torch.zeros(2, 4, S, device="cuda:0")
    lib = sig.binding.load_library()
    f, fb = lib.sig_combine_grouped, lib.sig_combine_grouped_backward
    assert f(a.data_ptr(), sigs.data_ptr(), 2, 0, d, N, sig.SIG_F32, sigs.data_ptr(), 0) == sig.SIG_ERR_INVALID_ARG
    assert f(0, sigs.data_ptr(), 2, 4, d, N, sig.SIG_F32, sigs.data_ptr(), 0) == sig.SIG_ERR_INVALID_ARG
    assert f(a.data_ptr(), sigs.data_ptr(), 2, 4, d, N, 7, sigs.data_ptr(), 0) == sig.SIG_ERR_INVALID_ARG
    assert f(a.data_ptr(), sigs.data_ptr(), 0, 4, d, N, sig.SIG_F32, sigs.data_ptr(), 0) == sig.SIG_OK
    need = sig.sig_combine_grouped_backward_workspace_bytes(2, 4, d, N)
    assert need >= 2 * 4 * S * 4
    assert sig.sig_combine_grouped_backward_workspace_bytes(2, 0, d, N) == -1
    ga, gs, g = torch.full_like(a, 7.0), torch.full_like(sigs, 7.0), torch.ones_like(sigs)
    ws = torch.empty(need, dtype=torch.uint8, device="cuda:0")
    # a short workspace, a missing one, outputs that alias: refused, outputs untouched
    args = (a.data_ptr(), sigs.data_ptr(), g.data_ptr(), 2, 4, d, N, sig.SIG_F32)
    assert fb(*args, ga.data_ptr(), gs.data_ptr(), ws.data_ptr(), need - 1, 0) == sig.SIG_ERR_INVALID_ARG
    assert fb(*args, ga.data_ptr(), gs.data_ptr(), 0, need, 0) == sig.SIG_ERR_INVALID_ARG
    assert fb(*args, ga.data_ptr(), g.data_ptr(), ws.data_ptr(), need, 0) == sig.SIG_ERR_INVALID_ARG
    torch.cuda.synchronize()
    assert bool((ga == 7).all()) and bool((gs == 7).all())
    assert fb(*args, ga.data_ptr(), gs.data_ptr(), ws.data_ptr(), need, 0) == sig.SIG_OK
    torch.cuda.synchronize()


@pytest.mark.parametrize("inverse", [False, True])
def test_initial_is_differentiable_in_stream_mode(inverse):
    import torch
    d, N = 2, 3
    x = dev(brownian_paths(2, 5, d, seed=12).astype(np.float64)).requires_grad_(True)
    init = dev(orc.signature(brownian_paths(2, 4, d, seed=3), N)).requires_grad_(True)
    bp = dev(uniform_paths(2, 1, d, seed=10)[:, 0].astype(np.float64)).requires_grad_(True)
    assert torch.autograd.gradcheck(lambda p, i: sig.signature(p, N, stream=True, initial=i, inverse=inverse), (x, init),
                                    eps=1e-6, atol=1e-7, rtol=1e-6)
    assert torch.autograd.gradcheck(lambda p, i, q: sig.signature(p, N, stream=True, basepoint=q, initial=i, inverse=inverse),
                                    (x, init, bp), eps=1e-6, atol=1e-7, rtol=1e-6)
    # the differentiable route and the single call that applies `initial` in place give the same values
    with torch.no_grad():
        direct = sig.signature(x, N, stream=True, initial=init, inverse=inverse)
    np.testing.assert_allclose(host(sig.signature(x, N, stream=True, initial=init, inverse=inverse).detach()), host(direct),
                               rtol=1e-13, atol=1e-15)


def test_stream_gradient_through_initial_against_the_oracle():
    # loss = sum of g * (initial [x] Sig(prefixes of x)): with y the earlier data whose signature is `initial`, the
    # oracle's gradient of the stream signature of the joined path, taken at the points of x after the junction, is
    # the path gradient; the gradient of `initial` is checked through the oracle's product gradient
    import torch
    B, L, d, N = 3, 9, 4, 5
    S = orc.channels(d, N)
    x = brownian_paths(B, L, d, seed=31).astype(np.float64)
    init = orc.signature(brownian_paths(B, 6, d, seed=32).astype(np.float64), N)
    g = np.random.default_rng(5).standard_normal((B, L - 1, S))
    xt, it = dev(x).requires_grad_(True), dev(init).requires_grad_(True)
    out = sig.signature(xt, N, stream=True, initial=it)
    out.backward(dev(g))
    plain = orc.signature(x, N, stream=True)
    want_i, want_plain = np.zeros((B, S)), np.zeros((B, L - 1, S))
    for b in range(B):
        for s in range(L - 1):
            wa, ws = orc.group_mul_backward(init[b], plain[b, s], g[b, s], d, N)
            want_i[b] += wa
            want_plain[b, s] = ws
    want_x = orc.signature_backward(x, want_plain, N, stream=True)
    np.testing.assert_allclose(host(it.grad), want_i, rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(host(xt.grad), want_x, rtol=1e-9, atol=1e-11)


@pytest.mark.parametrize("B,L,d,N,basepoint", [(2, 700, 3, 4, False), (1, 5000, 4, 6, True), (3, 4200, 8, 4, False)])
def test_differentiable_signature_chunks_few_long_paths_by_itself(B, L, d, N, basepoint):
    # final mode with at most 64 long paths goes through sig_forward_chunked (the hint says how many chunks); values
    # and gradients are those of the plain scan
    import torch
    for dtype in (np.float32, np.float64):
        code = sig.SIG_F32 if dtype == np.float32 else sig.SIG_F64
        assert sig.sig_forward_chunks_hint(B, L, d, N, basepoint, code) > 1
        x = (brownian_paths(B, L, d, seed=L) + 0.5).astype(dtype)
        g = np.random.default_rng(L).standard_normal((B, orc.channels(d, N))).astype(dtype)
        xt = dev(x).requires_grad_(True)
        out = sig.signature(xt, N, basepoint=basepoint)
        out.backward(dev(g))
        full = np.concatenate([np.zeros((B, 1, d)), x], axis=1) if basepoint else x
        assert_levels_close(host(out.detach()), orc.signature(full, N), d, N, dtype)
        want = orc.signature_backward(full, g, N)[:, 1 if basepoint else 0:]
        err = np.linalg.norm(host(xt.grad) - want) / np.linalg.norm(want)
        assert err <= (1e-4 if dtype == np.float32 else 1e-9), err


def test_gradcheck_through_products_and_initial():
    import torch
    d, N = 2, 3
    sigs = [dev(orc.signature(brownian_paths(2, 4, d, seed=s), N)).requires_grad_(True) for s in range(5)]
    assert torch.autograd.gradcheck(lambda p, q: sig.signature_combine(p, q, d, N), tuple(sigs[:2]), eps=1e-6,
                                    atol=1e-7, rtol=1e-6)
    assert torch.autograd.gradcheck(lambda *t: sig.multi_signature_combine(list(t), d, N), tuple(sigs), eps=1e-6,
                                    atol=1e-7, rtol=1e-6)
    x = dev(brownian_paths(2, 5, d, seed=11).astype(np.float64)).requires_grad_(True)
    assert torch.autograd.gradcheck(lambda p, i: sig.signature(p, N, initial=i), (x, sigs[0]), eps=1e-6, atol=1e-7,
                                    rtol=1e-6)
    assert torch.autograd.gradcheck(lambda p, i: sig.signature(p, N, initial=i, inverse=True, basepoint=True),
                                    (x, sigs[1]), eps=1e-6, atol=1e-7, rtol=1e-6)


def test_multi_signature_combine_equals_the_signature_of_the_whole_path():
    import torch
    d, N = 3, 4
    x = brownian_paths(3, 13, d, seed=4).astype(np.float64)
    cuts = [0, 3, 4, 9, 12]
    pieces = [dev(orc.signature(x[:, cuts[i]:cuts[i + 1] + 1], N)) for i in range(4)]
    got = host(sig.multi_signature_combine(pieces, d, N))
    assert_levels_close(got, orc.signature(x, N), d, N, np.float64)
    # `initial` in final mode: the signature of everything so far
    first = dev(orc.signature(x[:, :6], N))
    got = host(sig.signature(dev(x[:, 5:]), N, initial=first))
    assert_levels_close(got, orc.signature(x, N), d, N, np.float64)


def test_path_logsignature_queries():
    x = brownian_paths(3, 12, 3, seed=21).astype(np.float64)
    N = 4
    p = sig.Path(dev(x), N)
    for i, j in ((0, 11), (2, 9), (5, 6)):
        got = host(p.logsignature(i, j))
        np.testing.assert_allclose(got, orc.logsignature(x[:, i:j + 1], N), rtol=0, atol=1e-10)
    assert host(p.logsignature(1, 4, mode="expand")).shape == (3, orc.channels(3, N))
