"""Pins for the fp64 CPU oracle: it is checked against what the paper and the mathematics
fix, never against itself and never against the HIP path.

Each test names the passage of the paper it rests on.  The helpers below are written
independently of `oracle/` (numpy outer products, itertools brute force).
"""
import itertools
import math
import os
from collections import Counter
from fractions import Fraction

import numpy as np
import pytest

from oracle import sig_oracle as orc
from paper_2001_00706_amd.inputs import brownian_paths, uniform_paths

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------------------- helpers
def split_levels(flat, d, N):
    """Flat signature -> list of N tensors, level k of shape (d,)*k (lexicographic order)."""
    out, off = [], 0
    for k in range(1, N + 1):
        out.append(np.asarray(flat[off:off + d ** k]).reshape((d,) * k))
        off += d ** k
    assert off == len(flat)
    return out


def join_levels(levels):
    return np.concatenate([np.asarray(a).reshape(-1) for a in levels])


def np_group_mul(A, B):
    """(A [x] B)_k = sum_{j=0..k} A_j (x) B_{k-j}, A_0 = B_0 = 1 (section 2.2), on level lists."""
    N = len(A)
    C = []
    for k in range(1, N + 1):
        acc = A[k - 1] + B[k - 1]
        for j in range(1, k):
            acc = acc + np.multiply.outer(A[j - 1], B[k - j - 1])
        C.append(acc)
    return C


def brute_force_exact(x, N):
    """Integral definition (section 2.1) evaluated segment by segment for a piecewise-linear
    path: the ordered simplex splits into cells indexed by non-decreasing segment tuples
    s_1 <= ... <= s_k; on a cell the integrand is the constant z_{s_1} (x) ... (x) z_{s_k}
    and the cell's volume is prod over runs of equal indices of 1/(run length)!."""
    x = np.asarray(x, dtype=np.float64)
    z = np.diff(x, axis=0)
    n, d = z.shape
    levels = []
    for k in range(1, N + 1):
        acc = np.zeros((d,) * k)
        for tup in itertools.combinations_with_replacement(range(n), k):
            vol = 1.0
            for m in Counter(tup).values():
                vol /= math.factorial(m)
            term = z[tup[0]]
            for s in tup[1:]:
                term = np.multiply.outer(term, z[s])
            acc += vol * term
        levels.append(acc)
    return levels


def riemann_levels(x, N, m):
    """Strict-order Riemann sum of the iterated integrals: every segment cut into m equal
    pieces with increments D_t, level k ~= sum_{t_1 < ... < t_k} D_{t_1} (x) ... (x) D_{t_k}.
    Accumulated as P_k(t) = P_k(t-1) + P_{k-1}(t-1) (x) D_t."""
    x = np.asarray(x, dtype=np.float64)
    z = np.diff(x, axis=0)
    d = x.shape[1]
    P = [np.zeros((d,) * k) for k in range(1, N + 1)]
    for seg in z:
        D = seg / m
        for _ in range(m):
            for k in range(N, 1, -1):
                P[k - 1] = P[k - 1] + np.multiply.outer(P[k - 2], D)
            P[0] = P[0] + D
    return P


def riemann_levels_literal(x, N, m):
    x = np.asarray(x, dtype=np.float64)
    z = np.diff(x, axis=0)
    d = x.shape[1]
    D = np.repeat(z / m, m, axis=0)
    out = []
    for k in range(1, N + 1):
        acc = np.zeros((d,) * k)
        for tup in itertools.combinations(range(len(D)), k):
            term = D[tup[0]]
            for t in tup[1:]:
                term = np.multiply.outer(term, D[t])
            acc += term
        out.append(acc)
    return out


def sig1(x, N, **kw):
    """Oracle signature of a single path [L, d] -> flat vector."""
    return orc.signature(np.asarray(x)[None], N, **kw)[0]


def rel(a, b):
    a, b = np.asarray(a, dtype=np.float64), np.asarray(b, dtype=np.float64)
    den = np.linalg.norm(b.reshape(-1))
    return np.linalg.norm((a - b).reshape(-1)) / (den if den > 0 else 1.0)


def rand_path(L, d, seed):
    return uniform_paths(1, L, d, seed)[0].astype(np.float64)


# --------------------------------------------------------------------- sizes and layout
@pytest.mark.parametrize("d,N", [(1, 1), (1, 5), (2, 4), (3, 3), (4, 6), (8, 5), (16, 4)])
def test_channels_is_sum_of_powers(d, N):
    # section 2.4: output has sum_{k=1..N} d^k channels
    assert orc.channels(d, N) == sum(d ** k for k in range(1, N + 1))


def test_channels_of_the_benchmark_shapes():
    assert [orc.channels(d, N) for d, N in [(2, 4), (4, 6), (8, 5), (4, 5), (16, 4)]] == \
        [30, 5460, 37448, 1364, 69904]


def test_channels_rejects_bad_arguments():
    assert orc.channels(0, 3) == -1
    assert orc.channels(3, 0) == -1
    assert orc.channels(1000, 30) == -1


def test_output_shapes():
    x = brownian_paths(3, 7, 2, seed=1)
    assert orc.signature(x, 3).shape == (3, 14)
    # section 5.5 ("expanding intervals"): prefixes of length 2..L -> L-1 entries
    assert orc.signature(x, 3, stream=True).shape == (3, 6, 14)
    assert orc.signature(x, 3, stream=True, basepoint=True).shape == (3, 7, 14)


# ----------------------------------------------------------- P1: single segment = exp
@pytest.mark.parametrize("d,N", [(1, 6), (2, 5), (3, 4), (5, 3)])
def test_single_segment_is_tensor_exponential(d, N):
    # section 2.2: Sig((x1, x2)) = exp(x2 - x1), level k = v^{(x)k} / k!
    x = rand_path(2, d, seed=10 + d)
    v = x[1] - x[0]
    got = split_levels(sig1(x, N), d, N)
    pw = v
    for k in range(1, N + 1):
        if k > 1:
            pw = np.multiply.outer(pw, v)
        np.testing.assert_allclose(got[k - 1], pw / math.factorial(k), rtol=1e-14, atol=1e-300)
    np.testing.assert_allclose(orc.tensor_exp(v, N), sig1(x, N), rtol=1e-15)


def test_scalar_path_gives_monomials():
    # section 2.5: for d = 1 the signature terms are the monomials Delta^k / k!
    x = np.array([[0.3], [1.1], [-0.4], [2.0], [1.25]])
    delta = x[-1, 0] - x[0, 0]
    got = sig1(x, 7)
    want = [delta ** k / math.factorial(k) for k in range(1, 8)]
    np.testing.assert_allclose(got, want, rtol=1e-11)  # cancellation between large up/down moves


# ----------------------------------------------------------------- P9: hand examples
def _read_golden(name):
    with open(os.path.join(GOLDEN, name)) as fh:
        rows = [ln.split() for ln in fh if ln.strip()]
    d, N, L = (int(t) for t in rows[0])
    path = np.array([[float(Fraction(t)) for t in r] for r in rows[1:1 + L]])
    levels = [np.array([float(Fraction(t)) for t in r]) for r in rows[1 + L:1 + L + N]]
    assert path.shape == (L, d) and all(len(lv) == d ** (k + 1) for k, lv in enumerate(levels))
    return d, N, path, np.concatenate(levels)


@pytest.mark.parametrize("name", ["axis_path_d2_N3.txt", "axis_path_d3_N3.txt"])
def test_hand_computed_axis_paths(name):
    # section 2.1 (integral definition), worked by hand; see tests/golden/README.md
    d, N, path, want = _read_golden(name)
    np.testing.assert_allclose(sig1(path, N), want, rtol=1e-15, atol=1e-15)


def test_word_order_is_lexicographic_with_first_letter_slowest():
    # x moves, then y: word 12 (offset 1 of level 2) carries the mass, word 21 (offset 2) none.
    s = sig1(np.array([[0.0, 0.0], [1.0, 0.0], [1.0, 1.0]]), 2)
    assert s[2 + 1] == 1.0 and s[2 + 2] == 0.0
    s = sig1(np.array([[0.0, 0.0], [0.0, 1.0], [1.0, 1.0]]), 2)
    assert s[2 + 1] == 0.0 and s[2 + 2] == 1.0


# ------------------------------------------------- P7 / P8: brute force from the definition
@pytest.mark.parametrize("L,d,N,seed", [(2, 2, 4, 0), (3, 2, 4, 1), (4, 3, 3, 2), (6, 2, 4, 3),
                                        (5, 3, 4, 4), (6, 1, 4, 5)])
def test_brute_force_cells_of_the_ordered_simplex(L, d, N, seed):
    x = rand_path(L, d, seed)
    want = brute_force_exact(x, N)
    got = split_levels(sig1(x, N), d, N)
    for k in range(N):
        np.testing.assert_allclose(got[k], want[k], rtol=1e-12, atol=1e-13)


def test_riemann_recursion_matches_literal_ordered_sum():
    x = rand_path(3, 2, 7)
    a, b = riemann_levels(x, 3, 3), riemann_levels_literal(x, 3, 3)
    for k in range(3):
        np.testing.assert_allclose(a[k], b[k], rtol=1e-12, atol=1e-14)


@pytest.mark.parametrize("L,d,N,seed", [(3, 2, 4, 11), (5, 3, 3, 12)])
def test_riemann_quadrature_converges_to_the_oracle(L, d, N, seed):
    # section 2.1: the signature is the iterated integral; first-order quadrature converges
    # like 1/m, so the error must halve when m doubles and be small at large m.
    x = rand_path(L, d, seed)
    got = split_levels(sig1(x, N), d, N)
    errs = []
    for m in (64, 128, 256):
        q = riemann_levels(x, N, m)
        errs.append([rel(q[k], got[k]) for k in range(N)])
    errs = np.array(errs)
    assert np.all(errs[:, 0] < 1e-12)                      # level 1 is exact
    assert np.all(errs[2, 1:] < 2e-2)
    ratio = errs[0, 1:] / errs[1, 1:]
    assert np.all((ratio > 1.8) & (ratio < 2.2)), ratio
    ratio = errs[1, 1:] / errs[2, 1:]
    assert np.all((ratio > 1.8) & (ratio < 2.2)), ratio


# ------------------------------------------------------------------------ P2: Chen
@pytest.mark.parametrize("L,d,N,seed", [(5, 2, 5, 21), (7, 3, 4, 22), (4, 4, 4, 23)])
def test_chen_identity_at_every_interior_point(L, d, N, seed):
    # section 2.2, eq. "grouplike": Sig(x_1..x_L) = Sig(x_1..x_j) [x] Sig(x_j..x_L)
    x = rand_path(L, d, seed)
    whole = sig1(x, N)
    for j in range(1, L - 1):
        a, b = sig1(x[:j + 1], N), sig1(x[j:], N)
        via_np = join_levels(np_group_mul(split_levels(a, d, N), split_levels(b, d, N)))
        via_c = orc.group_mul(a, b, d, N)
        assert rel(via_np, whole) < 1e-13
        assert rel(via_c, whole) < 1e-13


def test_group_mul_is_not_commutative_and_matches_numpy():
    d, N = 3, 4
    a, b = sig1(rand_path(4, d, 31), N), sig1(rand_path(3, d, 32), N)
    ab = orc.group_mul(a, b, d, N)
    ba = orc.group_mul(b, a, d, N)
    assert rel(ab, ba) > 1e-3
    want = join_levels(np_group_mul(split_levels(a, d, N), split_levels(b, d, N)))
    np.testing.assert_allclose(ab, want, rtol=1e-13, atol=1e-15)


# -------------------------------------------------- P3: reparametrisation invariance
def test_inserting_collinear_or_repeated_points_changes_nothing():
    # section 2.1 (remark after definition 4): the knots' positions in [0,1] do not matter,
    # so a point inserted on a segment, or a repeated point, leaves the signature unchanged.
    d, N = 3, 5
    x = rand_path(5, d, 41)
    base = sig1(x, N)
    for j, t in [(0, 0.25), (2, 0.5), (3, 0.9)]:
        mid = x[j] + t * (x[j + 1] - x[j])
        y = np.insert(x, j + 1, mid, axis=0)
        assert rel(sig1(y, N), base) < 1e-13
    y = np.insert(x, 2, x[2], axis=0)
    assert rel(sig1(y, N), base) < 1e-15
    y = np.concatenate([x[:1], x, x[-1:]], axis=0)
    assert rel(sig1(y, N), base) < 1e-15


# ------------------------------------------- P4: level 1 / level 2 closed forms, area
def test_level_one_is_total_displacement_and_level_two_closed_form():
    d, N = 4, 3
    x = rand_path(9, d, 51)
    z = np.diff(x, axis=0)
    lv = split_levels(sig1(x, N), d, N)
    np.testing.assert_allclose(lv[0], x[-1] - x[0], rtol=1e-13)
    want2 = np.zeros((d, d))
    for i in range(len(z)):
        want2 += 0.5 * np.outer(z[i], z[i])
        for j in range(i + 1, len(z)):
            want2 += np.outer(z[i], z[j])
    np.testing.assert_allclose(lv[1], want2, rtol=1e-12, atol=1e-14)
    # symmetric part = (1/2) S_1 (x) S_1
    np.testing.assert_allclose(0.5 * (lv[1] + lv[1].T), 0.5 * np.outer(lv[0], lv[0]),
                               rtol=1e-12, atol=1e-14)


def test_levy_area_of_a_closed_polygon_is_the_shoelace_area():
    # the antisymmetric part of level 2 is the signed area (section 1: "order and area")
    rng = np.random.default_rng(61)
    ang = np.sort(rng.uniform(0, 2 * np.pi, 7))
    rad = rng.uniform(0.5, 1.5, 7)
    pts = np.stack([rad * np.cos(ang), rad * np.sin(ang)], axis=1)
    poly = np.concatenate([pts, pts[:1]], axis=0)
    s2 = split_levels(sig1(poly, 2), 2, 2)[1]
    shoelace = 0.5 * np.sum(poly[:-1, 0] * poly[1:, 1] - poly[1:, 0] * poly[:-1, 1])
    assert abs(0.5 * (s2[0, 1] - s2[1, 0]) - shoelace) < 1e-13
    assert shoelace > 0
    # a closed loop has zero displacement, hence a purely antisymmetric level 2
    np.testing.assert_allclose(s2 + s2.T, 0, atol=1e-13)


# ------------------------------------------------------ P5: shuffle (group-like) identities
def test_shuffle_identities():
    d, N = 3, 4
    lv = split_levels(sig1(rand_path(6, d, 71), N), d, N)
    S1, S2, S3, S4 = lv
    for a in range(d):
        for b in range(d):
            assert abs(S1[a] * S1[b] - (S2[a, b] + S2[b, a])) < 1e-12
            for c in range(d):
                lhs = S1[a] * S2[b, c]
                rhs = S3[a, b, c] + S3[b, a, c] + S3[b, c, a]
                assert abs(lhs - rhs) < 1e-12
                for e in range(d):
                    lhs = S2[a, b] * S2[c, e]
                    rhs = (S4[a, b, c, e] + S4[a, c, b, e] + S4[a, c, e, b]
                           + S4[c, a, b, e] + S4[c, a, e, b] + S4[c, e, a, b])
                    assert abs(lhs - rhs) < 1e-12
        for k, Sk in enumerate(lv, start=1):
            assert abs(Sk[(a,) * k] - S1[a] ** k / math.factorial(k)) < 1e-12


# -------------------------------------------------------------- P6: inverse = reversal
def test_signature_of_reversed_path_is_the_group_inverse():
    # section 5.4: Sig(x_1..x_L)^{-1} = Sig(x_L..x_1); the identity is the all-zero vector
    d, N = 3, 5
    x = rand_path(6, d, 81)
    fwd, bwd = sig1(x, N), sig1(x[::-1], N)
    assert np.max(np.abs(orc.group_mul(fwd, bwd, d, N))) < 1e-12
    assert np.max(np.abs(orc.group_mul(bwd, fwd, d, N))) < 1e-12


# ------------------------------------- P10: scaling, translation, basepoint, stream mode
def test_scaling_and_translation():
    d, N = 2, 5
    x = rand_path(6, d, 91)
    base = split_levels(sig1(x, N), d, N)
    lam = -1.7
    scaled = split_levels(sig1(lam * x, N), d, N)
    for k in range(N):
        np.testing.assert_allclose(scaled[k], lam ** (k + 1) * base[k], rtol=1e-12, atol=1e-15)
    shifted = sig1(x + np.array([3.0, -2.0]), N)
    assert rel(shifted, join_levels(base)) < 1e-13


def test_basepoint_prepends_the_origin():
    d, N = 3, 4
    x = rand_path(5, d, 101) + 0.7
    with_flag = sig1(x, N, basepoint=True)
    by_hand = sig1(np.concatenate([np.zeros((1, d)), x], axis=0), N)
    np.testing.assert_array_equal(with_flag, by_hand)
    # a single point plus the basepoint is a one-segment path
    one = sig1(x[:1], N, basepoint=True)
    np.testing.assert_allclose(one, orc.tensor_exp(x[0], N), rtol=1e-15)


@pytest.mark.parametrize("basepoint", [False, True])
def test_stream_entries_are_prefix_signatures(basepoint):
    # section 5.5: (Sig(x1,x2), Sig(x1,x2,x3), ..., Sig(x1..xL))
    d, N = 2, 4
    x = brownian_paths(3, 9, d, seed=111).astype(np.float64)
    st = orc.signature(x, N, stream=True, basepoint=basepoint)
    fin = orc.signature(x, N, basepoint=basepoint)
    np.testing.assert_array_equal(st[:, -1], fin)
    first = 1 if basepoint else 2
    for j in range(st.shape[1]):
        pref = orc.signature(x[:, :first + j], N, basepoint=basepoint)
        np.testing.assert_array_equal(st[:, j], pref)


def test_batch_entries_are_independent_and_thread_count_does_not_matter():
    x = brownian_paths(9, 12, 3, seed=121)
    a = orc.signature(x, 4, num_threads=1)
    b = orc.signature(x, 4, num_threads=4)
    np.testing.assert_array_equal(a, b)
    for i in (0, 4, 8):
        np.testing.assert_array_equal(orc.signature(x[i:i + 1], 4)[0], a[i])


def test_bad_arguments_raise():
    with pytest.raises(ValueError):
        orc.signature(np.zeros((2, 1, 3)), 2)          # a single point is not a path
    with pytest.raises(ValueError):
        orc.signature(np.zeros((2, 3)), 2)
    assert orc.signature(np.zeros((0, 4, 3)), 2).shape == (0, 12)
    # zero increments are legal: the signature is the identity (all zeros)
    assert np.all(orc.signature(np.ones((2, 4, 3)), 3) == 0.0)
