"""Pins for the oracle's nodes and Berrut basis functions (no GPU).

Each test checks the oracle against something fixed by the paper's definitions or
by mathematics, not against the oracle's own formula.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import approxifer_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _exact_basis_product_form(z, x, s):
    """l_i(z) in the polynomial form obtained by multiplying numerator and
    denominator of eq. (2) by prod_k (z - x_k):
        l_i(z) = s_i prod_{k != i}(z - x_k) / sum_m s_m prod_{k != m}(z - x_k),
    in exact rational arithmetic.  It has no division by (z - x_i), so it is also
    valid at the nodes."""
    n = len(x)
    num = []
    for i in range(n):
        p = Fraction(s[i])
        for k in range(n):
            if k != i:
                p *= (z - x[k])
        num.append(p)
    den = sum(num)
    return [p / den for p in num]


def test_chebyshev_nodes_values():
    # Section 3, "ApproxIFER Encoding": alpha_j = cos((2j+1)pi/2K), beta_i = cos(i pi/N), N = W-1
    alpha, beta = orc.chebyshev_nodes(4, 7)
    for j in range(4):
        assert alpha[j] == pytest.approx(math.cos((2 * j + 1) * math.pi / 8), abs=1e-16)
    for i in range(7):
        assert beta[i] == pytest.approx(math.cos(i * math.pi / 6), abs=1e-16)
    # textbook values
    assert alpha[0] == pytest.approx(math.sqrt(2 + math.sqrt(2)) / 2, abs=1e-15)
    assert beta[0] == 1.0 and beta[-1] == pytest.approx(-1.0, abs=1e-15)
    assert beta[2] == pytest.approx(0.5, abs=1e-15)          # cos(pi/3)
    assert beta[3] == pytest.approx(0.0, abs=1e-15)
    # first-kind points are the roots of T_K, second-kind points the extrema of T_{W-1}
    T4 = np.polynomial.chebyshev.Chebyshev.basis(4)
    assert np.max(np.abs(T4(alpha))) < 1e-14
    T6 = np.polynomial.chebyshev.Chebyshev.basis(6)
    assert np.allclose(np.abs(T6(beta)), 1.0, atol=1e-14)
    # strictly descending, inside [-1, 1]
    assert np.all(np.diff(alpha) < 0) and np.all(np.diff(beta) < 0)


def test_golden_three_nodes_rational():
    rows = [l for l in open(os.path.join(GOLDEN, "berrut_three_nodes_rational.txt")) if not l.startswith("#")]
    x = np.array([1.0, 0.0, -1.0])
    s = np.array([1.0, -1.0, 1.0])
    for row in rows:
        left, right = row.split("|")
        zn, zd = (int(t) for t in left.split())
        want = [float(Fraction(t)) for t in right.split()]
        got = orc.berrut_weights([zn / zd], x, s)[0]
        assert np.allclose(got, want, rtol=0, atol=1e-15)


def test_golden_k2_w3_encoder_matrix():
    want = np.loadtxt(os.path.join(GOLDEN, "berrut_k2_w3.txt"))
    alpha, beta = orc.chebyshev_nodes(2, 3)
    got = orc.encode_weights(alpha, beta)
    assert got.shape == (3, 2)
    assert np.allclose(got, want, rtol=0, atol=2e-15)
    # the file's numbers are (1 +- sqrt 2)/2 and 1/2
    assert want[0, 0] == pytest.approx((1 + math.sqrt(2)) / 2, abs=1e-16)
    assert want[0, 1] == pytest.approx((1 - math.sqrt(2)) / 2, abs=1e-16)


@pytest.mark.parametrize("n", [2, 3, 4, 5, 7])
def test_weights_match_exact_rational_product_form(n):
    # rational nodes and evaluation points so that Fractions are exact
    rng = np.random.default_rng(100 + n)
    xs = sorted({Fraction(int(v), 16) for v in rng.integers(-16, 17, size=3 * n)}, reverse=True)[:n]
    assert len(xs) == n
    s = [(-1) ** i for i in range(n)]
    zs = [Fraction(int(v), 37) for v in rng.integers(-36, 37, size=6)]
    zs = [z for z in zs if z not in xs]
    got = orc.berrut_weights([float(z) for z in zs], [float(v) for v in xs], s)
    for m, z in enumerate(zs):
        want = [float(v) for v in _exact_basis_product_form(z, xs, s)]
        assert np.allclose(got[m], want, rtol=1e-12, atol=1e-13)


def test_two_nodes_is_linear_interpolation():
    # eq. (2) with two nodes: l_0 = (z - x_1)/(x_0 - x_1), l_1 = (x_0 - z)/(x_0 - x_1)
    x = np.array([0.8, -0.3])
    z = np.linspace(-1, 1, 9)
    L = orc.berrut_weights(z, x, [1, -1])
    assert np.allclose(L[:, 0], (z - x[1]) / (x[0] - x[1]), atol=1e-14)
    assert np.allclose(L[:, 1], (x[0] - z) / (x[0] - x[1]), atol=1e-14)


def test_single_node_is_replication():
    # K = 1: u(z) = X_0 for every z, so every coded query is the query itself
    alpha, beta = orc.chebyshev_nodes(1, 5)
    L = orc.encode_weights(alpha, beta)
    assert L.shape == (5, 1) and np.all(L == 1.0)


@pytest.mark.parametrize("K,W", [(4, 6), (8, 12), (12, 20), (8, 24), (16, 24), (32, 48), (3, 5)])
def test_rows_sum_to_one(K, W):
    alpha, beta = orc.chebyshev_nodes(K, W)
    L = orc.encode_weights(alpha, beta)
    assert L.shape == (W, K)
    assert np.max(np.abs(L.sum(axis=1) - 1.0)) < 1e-13


def test_one_hot_at_a_node_and_limit():
    x = np.array([0.9, 0.2, -0.5, -0.95])
    s = orc.alternating_signs(4)
    L = orc.berrut_weights(x, x, s)
    assert np.array_equal(L, np.eye(4))
    # the unit row is the limit of the formula: approach node 1
    near = orc.berrut_weights([x[1] + 1e-9], x, s)[0]
    assert np.allclose(near, [0, 1, 0, 0], atol=1e-7)
    # K=2, W=5: alpha_0 = cos(pi/4) coincides mathematically with beta_1 = cos(pi/4)
    alpha, beta = orc.chebyshev_nodes(2, 5)
    Lc = orc.encode_weights(alpha, beta)
    assert np.allclose(Lc[1], [1.0, 0.0], atol=1e-12) and np.allclose(Lc[3], [0.0, 1.0], atol=1e-12)


def test_invariance_to_order_and_global_sign():
    rng = np.random.default_rng(7)
    x = np.sort(rng.uniform(-1, 1, 6))
    s = orc.alternating_signs(6)
    z = rng.uniform(-1, 1, 5)
    L = orc.berrut_weights(z, x, s)
    # flipping every sign cancels in the ratio
    assert np.allclose(L, orc.berrut_weights(z, x, -s), atol=1e-15)
    # listing the nodes in descending order (as Chebyshev points come) permutes the columns only
    Lr = orc.berrut_weights(z, x[::-1], orc.alternating_signs(6))
    assert np.allclose(L, Lr[:, ::-1], atol=1e-13)


def test_no_real_pole_with_alternating_signs():
    # Section 3 (background): Berrut's interpolant has no pole on the real line; its
    # denominator sum_i (-1)^i/(z - x_i) keeps one sign between consecutive nodes, so
    # the weights stay bounded.  Probe densely between the nodes.
    alpha, _ = orc.chebyshev_nodes(12, 20)
    z = np.linspace(-0.999, 0.999, 4001)
    z = z[~np.isin(z, alpha)]
    L = orc.berrut_weights(z, alpha, orc.alternating_signs(12))
    assert np.all(np.isfinite(L))
    assert np.max(np.abs(L).sum(axis=1)) < 10.0        # Lebesgue function stays O(log n)
