"""Pins for the logarithm / logsignature part of the fp64 CPU oracle (sections 2.3, 4.3, appendix A.2)."""
import itertools
import math

import numpy as np
import pytest

from oracle import sig_oracle as orc
from paper_2001_00706_amd.inputs import brownian_paths, uniform_paths
from tests.test_oracle_pins import join_levels, np_group_mul, split_levels


def np_exp_of_element(y_levels):
    """exp(y) = sum_{m>=0} y^{[x] m} / m! for an element y without constant term, as level lists with the
    constant term dropped again (numpy outer products, independent of the oracle)."""
    N = len(y_levels)
    zero = [np.zeros_like(a) for a in y_levels]
    total = [a.copy() for a in y_levels]
    power = [a.copy() for a in y_levels]
    for m in range(2, N + 1):
        nxt = [z.copy() for z in zero]
        for k in range(2, N + 1):
            for j in range(1, k):
                nxt[k - 1] = nxt[k - 1] + np.multiply.outer(power[j - 1], y_levels[k - j - 1])
        power = nxt
        total = [t + p / math.factorial(m) for t, p in zip(total, power)]
    return total


def bracket(a, b):
    return np.multiply.outer(a, b) - np.multiply.outer(b, a)


def mobius(n):
    result, p = 1, 2
    while p * p <= n:
        if n % p == 0:
            n //= p
            if n % p == 0:
                return 0
            result = -result
        p += 1
    return -result if n > 1 else result


def witt(d, N):
    # section 2.3: w(d, N) = sum_{k=1..N} (1/k) sum_{i | k} mu(k/i) d^i
    return sum(sum(mobius(k // i) * d ** i for i in range(1, k + 1) if k % i == 0) // k for k in range(1, N + 1))


@pytest.mark.parametrize("d,N", [(2, 5), (3, 4), (5, 3)])
def test_log_of_a_single_exponential_is_the_increment(d, N):
    # log is the inverse of exp (section 2.3): log(exp(z)) = (z, 0, ..., 0)
    z = np.random.default_rng(d + N).standard_normal(d)
    got = orc.tensor_log(orc.tensor_exp(z, N), d, N)
    want = np.zeros_like(got)
    want[:d] = z
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-14)


@pytest.mark.parametrize("L,d,N", [(6, 2, 5), (5, 3, 4), (9, 4, 3)])
def test_exp_of_log_returns_the_signature(L, d, N):
    x = brownian_paths(2, L, d, seed=L + d)
    s = orc.signature(x, N)
    lg = orc.tensor_log(s, d, N)
    for b in range(2):
        back = join_levels(np_exp_of_element(split_levels(lg[b], d, N)))
        np.testing.assert_allclose(back, s[b], rtol=1e-12, atol=1e-14)


def test_baker_campbell_hausdorff_to_depth_three():
    # two segments a, b: log(exp(a) [x] exp(b)) = a + b + [a,b]/2 + ([a,[a,b]] + [b,[b,a]])/12 + (depth >= 4)
    rng = np.random.default_rng(2)
    d = 3
    a, b = rng.standard_normal((2, d))
    x = np.stack([np.zeros(d), a, a + b])[None]
    got = split_levels(orc.tensor_log(orc.signature(x, 3), d, 3)[0], d, 3)
    ab = bracket(a, b)
    np.testing.assert_allclose(got[0], a + b, atol=1e-14)
    np.testing.assert_allclose(got[1], ab / 2, atol=1e-14)
    np.testing.assert_allclose(got[2], (bracket(a, ab) + bracket(b, -ab)) / 12, atol=1e-14)


def test_level_two_of_the_log_is_the_levy_area():
    # log_2 = S_2 - S_1 (x) S_1 / 2: the antisymmetric part of level 2
    x = brownian_paths(3, 12, 4, seed=7)
    s = orc.signature(x, 2)
    lg = orc.tensor_log(s, 4, 2)
    for b in range(3):
        S1, S2 = split_levels(s[b], 4, 2)
        L1, L2 = split_levels(lg[b], 4, 2)
        np.testing.assert_allclose(L1, S1, atol=1e-15)
        np.testing.assert_allclose(L2, (S2 - S2.T) / 2, atol=1e-14)


def test_log_turns_the_group_product_of_commuting_elements_into_a_sum():
    # collinear segments commute: log(exp(s z) [x] exp(t z)) = (s + t) z; and log(g^{-1}) = -log(g)
    z = np.array([0.3, -1.1, 0.7])
    x = np.stack([np.zeros(3), 0.4 * z, 1.5 * z])[None]
    lg = orc.tensor_log(orc.signature(x, 4), 3, 4)[0]
    want = np.zeros_like(lg)
    want[:3] = 1.5 * z
    np.testing.assert_allclose(lg, want, atol=1e-14)
    y = brownian_paths(1, 8, 3, seed=3)
    np.testing.assert_allclose(orc.tensor_log(orc.signature(y[:, ::-1], 4), 3, 4),
                               -orc.tensor_log(orc.signature(y, 4), 3, 4), rtol=1e-11, atol=1e-14)


def test_lyndon_words_examples_of_the_paper_and_witt_dimension():
    # appendix A.2.1: a2 a2 a3 a4 is a Lyndon word, a2 a2 is not (0-based letters below)
    words = orc.lyndon_words(4, 4)
    assert (1, 1, 2, 3) in words
    assert (1, 1) not in words
    assert words[:4] == [(0,), (1,), (2,), (3,)]
    assert orc.lyndon_words(2, 4) == [(0,), (1,), (0, 1), (0, 0, 1), (0, 1, 1), (0, 0, 0, 1), (0, 0, 1, 1), (0, 1, 1, 1)]
    for d, N in [(2, 8), (3, 5), (4, 4), (7, 3), (1, 5)]:
        assert len(orc.lyndon_words(d, N)) == witt(d, N)          # Witt's formula, section 2.3


def test_lyndon_indices_point_at_the_words():
    d, N = 3, 4
    idx = orc.lyndon_indices(d, N)
    flat = np.arange(orc.channels(d, N))
    levels = split_levels(flat, d, N)
    for w, i in zip(orc.lyndon_words(d, N), idx):
        assert levels[len(w) - 1][w] == i


def test_logsignature_determines_the_log_through_the_lyndon_basis_at_depth_two_and_three():
    # a Lie element of depth 2 is sum_i a_i e_i + sum_{i<j} c_ij [e_i, e_j]; its coefficient on the Lyndon word ij (i<j) is c_ij,
    # and on the Lyndon words iij, ijj, ijk (depth 3) the coefficients of the brackets' leading words (appendix A.2.4)
    d, N = 3, 3
    x = brownian_paths(1, 7, d, seed=13)
    lg = split_levels(orc.tensor_log(orc.signature(x, N), d, N)[0], d, N)
    ls = orc.logsignature(x, N)[0]
    words = orc.lyndon_words(d, N)
    assert ls.shape == (len(words),)
    for w, v in zip(words, ls):
        assert v == lg[len(w) - 1][w]
    # level 2 of a Lie element is antisymmetric, so the Lyndon coefficients ij (i<j) rebuild it completely
    L2 = np.zeros((d, d))
    for w, v in zip(words, ls):
        if len(w) == 2:
            L2[w] = v
            L2[w[::-1]] = -v
    np.testing.assert_allclose(L2, lg[1], atol=1e-14)


def test_stream_and_basepoint_logsignatures_are_logs_of_the_prefix_signatures():
    x = uniform_paths(2, 6, 2, seed=5).astype(np.float64)
    ls = orc.logsignature(x, 4, stream=True, basepoint=True)
    idx = orc.lyndon_indices(2, 4)
    for j in range(6):
        want = orc.tensor_log(orc.signature(x[:, :j + 1], 4, basepoint=True), 2, 4)[:, idx]
        np.testing.assert_allclose(ls[:, j], want, rtol=1e-13, atol=1e-15)


# ---- gradient of the logarithm ------------------------------------------------------------------------------------

@pytest.mark.parametrize("d,N", [(2, 2), (2, 5), (3, 4), (4, 3), (1, 4)])
def test_log_gradient_matches_finite_differences_of_the_pinned_log(d, N):
    # any element x (not only signatures): the adjoint must reproduce <g, d log(1 + x)[v]> for every direction v
    rng = np.random.default_rng(10 * d + N)
    S = orc.channels(d, N)
    x, g = 0.6 * rng.standard_normal(S), rng.standard_normal(S)
    gx = orc.tensor_log_backward(x, g, d, N)
    h = 1e-6
    for _ in range(6):
        v = rng.standard_normal(S)
        fd = np.dot(g, orc.tensor_log(x + h * v, d, N) - orc.tensor_log(x - h * v, d, N)) / (2 * h)
        assert abs(np.dot(gx, v) - fd) <= 1e-8 * (1 + abs(fd))
    # and coordinate by coordinate at the lowest and the highest level
    for i in list(range(min(d, 3))) + [S - 1]:
        e = np.zeros(S)
        e[i] = h
        fd = np.dot(g, orc.tensor_log(x + e, d, N) - orc.tensor_log(x - e, d, N)) / (2 * h)
        assert abs(gx[i] - fd) <= 1e-8 * (1 + abs(fd))


def test_log_gradient_closed_form_at_depth_two():
    # log(1 + x) = (x_1, x_2 - x_1 (x) x_1 / 2)  =>  gx_2 = g_2,  gx_1 = g_1 - (g_2 x_1 + g_2^T x_1) / 2
    d = 3
    rng = np.random.default_rng(4)
    x, g = rng.standard_normal(d + d * d), rng.standard_normal(d + d * d)
    g2 = g[d:].reshape(d, d)
    want = np.concatenate([g[:d] - 0.5 * (g2 @ x[:d] + g2.T @ x[:d]), g[d:]])
    np.testing.assert_allclose(orc.tensor_log_backward(x, g, d, 2), want, rtol=0, atol=1e-14)


def test_logsignature_gradient_of_a_single_segment_sees_only_level_one():
    # log Sig of a straight segment is (z, 0, ..., 0) for every z, so only the cotangent of the letters reaches the
    # two end points, with opposite signs; the cotangents of all longer Lyndon words are annihilated
    d, N = 3, 4
    rng = np.random.default_rng(8)
    path = rng.standard_normal((2, 2, d))
    g = rng.standard_normal((2, len(orc.lyndon_indices(d, N))))
    got = orc.logsignature_backward(path, g, N)
    np.testing.assert_allclose(got[:, 1], g[:, :d], rtol=0, atol=1e-13)
    np.testing.assert_allclose(got[:, 0], -g[:, :d], rtol=0, atol=1e-13)


def test_logsignature_gradient_matches_finite_differences():
    d, N = 2, 4
    x = brownian_paths(2, 6, d, seed=3).astype(np.float64) * 2.0
    rng = np.random.default_rng(2)
    g = rng.standard_normal((2, 5, len(orc.lyndon_indices(d, N))))
    got = orc.logsignature_backward(x, g, N, stream=True)
    h = 1e-6
    for _ in range(5):
        v = rng.standard_normal(x.shape)
        fd = np.sum(g * (orc.logsignature(x + h * v, N, stream=True) - orc.logsignature(x - h * v, N, stream=True))) / (2 * h)
        assert abs(np.sum(got * v) - fd) <= 1e-8 * (1 + abs(fd))
