"""Pins for the oracle's adversary locator (Algorithm 2) and Byzantine decoder (no GPU)."""
import itertools
from fractions import Fraction

import numpy as np
import pytest

from oracle import approxifer_oracle as orc
from paper_2109_09868_amd import synthetic as syn


def _rational_samples(rng, K, x):
    """y_i = p(x_i)/q(x_i) with deg p, deg q <= K-1 and q without zero on [-1, 1], q(0) = 1
    (the function class of Theorem 1, Appendix A)."""
    p = rng.standard_normal(K)
    q = np.concatenate([[1.0], 0.3 * rng.uniform(-1, 1, K - 1) / max(K - 1, 1)])
    P = np.polynomial.polynomial.polyval(x, p)
    Q = np.polynomial.polynomial.polyval(x, q)
    assert np.all(Q > 0.5)
    return P / Q


def _brute_force_adversaries(x, y, K, A):
    """The A-subset whose removal leaves points that lie exactly on some rational function of
    degree (K-1, K-1): smallest singular value of [V | -y V] (homogeneous, Appendix A
    eq. P(x_i) = y_i Q(x_i) with no error locator) is ~0 for that subset only."""
    n = len(x)
    best = None
    for sub in itertools.combinations(range(n), A):
        keep = np.setdiff1d(np.arange(n), sub)
        V = np.vander(x[keep], K, increasing=True)
        H = np.concatenate([V, -y[keep, None] * V], axis=1)
        H = H / np.linalg.norm(H, axis=0)
        smin = np.linalg.svd(H, compute_uv=False)[-1]
        if best is None or smin < best[0]:
            best = (smin, sub)
    return best


def test_system_shape_and_rows():
    # Algorithm 2 steps 1-2: 2(K+A)-1 unknowns, one equation per available worker
    K, A = 3, 2
    x = np.array([0.9, 0.5, 0.1, -0.2, -0.6, -0.8, -1.0, 0.3, 0.7, -0.4])
    y = np.arange(10.0) + 1
    Amat, rhs = orc.locator_system(x, y, K, A)
    M = K + A
    assert Amat.shape == (10, 2 * M - 1) and rhs.shape == (10,)
    i = 4
    # P part: x^0..x^{M-1}; Q part: -y x^1 .. -y x^{M-1}; rhs: y (the Q_0 = 1 term moved right)
    assert np.allclose(Amat[i, :M], [x[i] ** k for k in range(M)])
    assert np.allclose(Amat[i, M:], [-y[i] * x[i] ** k for k in range(1, M)])
    assert rhs[i] == y[i]
    # a (P, Q) pair that satisfies P(x_i) = y_i Q(x_i) exactly solves the system exactly
    rng = np.random.default_rng(0)
    Qc = np.concatenate([[1.0], rng.standard_normal(M - 1) * 0.1])
    Pc = rng.standard_normal(M)
    y2 = np.polynomial.polynomial.polyval(x, Pc) / np.polynomial.polynomial.polyval(x, Qc)
    A2, r2 = orc.locator_system(x, y2, K, A)
    assert np.allclose(A2 @ np.concatenate([Pc, Qc[1:]]), r2, atol=1e-12)


@pytest.mark.parametrize("K,A,S", [(2, 1, 0), (3, 1, 2), (3, 2, 0), (4, 2, 2)])
def test_theorem1_q_vanishes_at_adversaries(K, A, S):
    # Appendix A: Q = q * Lambda, Lambda(x) = prod_{adv}(1 - x/x_i) => Q(x_adv) = 0, and Q = q elsewhere
    rng = np.random.default_rng(11 * K + A)
    W = 2 * (K + A) + S
    _, beta = orc.chebyshev_nodes(K, W)
    for trial in range(20):
        avail = np.sort(rng.permutation(W)[: W - S])
        x = beta[avail]
        y = _rational_samples(rng, K, x)
        bad = np.sort(rng.permutation(avail.size)[:A])
        y_bad = y.copy()
        y_bad[bad] += rng.standard_normal(A) * 10 + 3
        a = orc.locator_values(x, y_bad, K, A)
        order = np.argsort(np.abs(a))
        assert set(order[:A]) == set(bad)
        assert np.abs(a[order[A - 1]]) < 1e-6 * np.abs(a[order[A]])          # clean separation
        picks = orc.pick_smallest(a, avail, A)
        assert set(picks) == set(avail[bad])


@pytest.mark.parametrize("K,A,W", [(2, 1, 6), (3, 1, 8), (2, 2, 8), (3, 2, 12)])
def test_locator_agrees_with_brute_force_subset_search(K, A, W):
    rng = np.random.default_rng(5 + K + 10 * A)
    _, beta = orc.chebyshev_nodes(K, W)
    avail = np.sort(rng.permutation(W)[: 2 * (K + A)])
    x = beta[avail]
    for trial in range(5):
        y = _rational_samples(rng, K, x)
        bad = np.sort(rng.permutation(avail.size)[:A])
        y[bad] += rng.choice([-1, 1], A) * rng.uniform(1, 5, A)
        smin, sub = _brute_force_adversaries(x, y, K, A)
        assert smin < 1e-10 and set(sub) == set(bad)
        a = orc.locator_values(x, y, K, A)
        assert set(np.argsort(np.abs(a))[:A]) == set(sub)
        a1 = orc.locator_values_homogeneous(x, y, K, A)
        assert set(np.argsort(np.abs(a1))[:A]) == set(sub)


def _exact_least_squares(rows, rhs):
    """argmin ||A s - b||_2 in exact rational arithmetic: the normal equations A^T A s = A^T b solved
    by Gauss-Jordan elimination over Fractions (A of full column rank)."""
    m = len(rows[0])
    N = [[sum(r[i] * r[j] for r in rows) for j in range(m)] + [sum(r[i] * b for r, b in zip(rows, rhs))]
         for i in range(m)]
    for i in range(m):
        piv = next(r for r in range(i, m) if N[r][i] != 0)
        N[i], N[piv] = N[piv], N[i]
        N[i] = [v / N[i][i] for v in N[i]]
        for r in range(m):
            if r != i and N[r][i] != 0:
                N[r] = [a - N[r][i] * b for a, b in zip(N[r], N[i])]
    return [N[i][m] for i in range(m)]


@pytest.mark.parametrize("K,A,n,seed", [(1, 1, 4, 0), (1, 1, 6, 1), (2, 1, 6, 2), (2, 1, 9, 3), (1, 2, 7, 4), (3, 1, 8, 5)])
def test_locator_values_are_the_exact_least_squares_solution_on_inconsistent_data(K, A, n, seed):
    # data that lie on no rational function: Algorithm 2's system is inconsistent and "solving" it means least
    # squares.  Rational nodes and values make the minimiser computable exactly (normal equations over Fractions);
    # the oracle's a_i = Q(x_i) must be that minimiser's, and so must the order of the |a_i|.
    rng = np.random.default_rng(seed)
    M = K + A
    xs = sorted({Fraction(int(v), 8) for v in rng.integers(-8, 9, size=4 * n) if v != 0}, reverse=True)[:n]
    assert len(xs) == n
    ys = [Fraction(int(v), 16) for v in rng.integers(-40, 41, size=n)]
    rows = [[x ** k for k in range(M)] + [-y * x ** k for k in range(1, M)] for x, y in zip(xs, ys)]
    sol = _exact_least_squares(rows, ys)
    Q = [Fraction(1)] + sol[M:]
    a_exact = [sum(q * x ** k for k, q in enumerate(Q)) for x in xs]
    a = orc.locator_values(np.array([float(x) for x in xs]), np.array([float(y) for y in ys]), K, A)
    want = np.array([float(v) for v in a_exact])
    assert np.max(np.abs(a - want)) <= 1e-9 * max(1.0, np.max(np.abs(want)))
    order_exact = sorted(range(n), key=lambda i: (abs(a_exact[i]), i))[:A]
    gaps = sorted(abs(v) for v in a_exact)
    if gaps[A] - gaps[A - 1] > Fraction(1, 10 ** 6):       # the pick is decided by more than rounding
        assert set(orc.pick_smallest(a, np.arange(n), A).tolist()) == set(order_exact)


@pytest.mark.parametrize("K,A,seed", [(2, 1, 0), (3, 1, 1), (2, 2, 2), (3, 2, 3), (4, 1, 4)])
def test_both_locators_return_q_times_the_error_locator_polynomial(K, A, seed):
    # Appendix A: with y_i = p(x_i)/q(x_i) off the adversaries, P = p Lambda and Q = q Lambda, Lambda(x) =
    # prod (1 - x/x_i) over the adversaries, satisfy every equation exactly, and at the minimum worker count
    # they are the only solution up to a factor.  So a_i = Q(x_i) is known in closed form: q(x_i) Lambda(x_i)
    # (divided by q(0) for Algorithm 2, whose Q(0) = 1; up to one factor for Algorithm 1).
    rng = np.random.default_rng(seed)
    M = K + A
    n = 2 * M
    xs = sorted({Fraction(int(v), 16) for v in rng.integers(-16, 17, size=6 * n) if v != 0}, reverse=True)[:n]
    assert len(xs) == n
    p = [Fraction(int(v), 4) for v in rng.integers(-8, 9, size=K)]
    q = [Fraction(1)] + [Fraction(int(v), 32) for v in rng.integers(-3, 4, size=K - 1)]
    ev = lambda c, x: sum(ck * x ** k for k, ck in enumerate(c))
    assert all(ev(q, x) > Fraction(1, 2) for x in xs)
    bad = sorted(rng.permutation(n)[:A].tolist())
    lam = lambda x: np.prod([1 - x / xs[i] for i in bad]) if bad else Fraction(1)
    ys = [ev(p, x) / ev(q, x) for x in xs]
    for i in bad:
        ys[i] += Fraction(int(rng.integers(1, 6)), 2) * (1 if rng.integers(0, 2) else -1)
    a_exact = np.array([float(ev(q, x) * lam(x) / q[0]) for x in xs])
    x_f = np.array([float(x) for x in xs])
    y_f = np.array([float(y) for y in ys])              # sixteenths and small rationals: a few are inexact in binary
    a2 = orc.locator_values(x_f, y_f, K, A)
    assert np.max(np.abs(a2 - a_exact)) <= 1e-7 * np.max(np.abs(a_exact))
    a1 = orc.locator_values_homogeneous(x_f, y_f, K, A)
    good = [i for i in range(n) if i not in bad]
    scale = a1[good[0]] / a_exact[good[0]]
    assert np.max(np.abs(a1 / scale - a_exact)) <= 1e-7 * np.max(np.abs(a_exact))
    assert np.all(np.abs(a_exact[bad]) == 0.0)


def test_zero_node_cannot_be_located_with_q0_fixed():
    # Algorithm 2 fixes Q(0) = 1 while the error locator Lambda(x) = prod (1 - x/x_i) of Appendix A
    # needs x_i != 0.  With an odd number of workers the middle node is 0: a_i = Q(0) = 1 there, so
    # an adversary sitting on it is never among the smallest |a_i|.  Algorithm 1 (Q_0 free) finds it.
    K, A, W = 3, 1, 9
    _, beta = orc.chebyshev_nodes(K, W)
    assert abs(beta[4]) < 1e-15
    rng = np.random.default_rng(2)
    x = beta[:8]
    y = _rational_samples(rng, K, x)
    y[4] += 5.0
    a2 = orc.locator_values(x, y, K, A)
    assert a2[4] == pytest.approx(1.0, abs=1e-12)
    a1 = orc.locator_values_homogeneous(x, y, K, A)
    assert np.argmin(np.abs(a1)) == 4


def test_algorithm1_null_vector_agrees():
    # Algorithm 1 (Q_0 free, null vector) locates the same workers as Algorithm 2 (Q_0 = 1)
    rng = np.random.default_rng(21)
    K, A, W = 4, 2, 14
    _, beta = orc.chebyshev_nodes(K, W)
    for trial in range(20):
        avail = np.sort(rng.permutation(W)[: 2 * (K + A)])
        x = beta[avail]
        y = _rational_samples(rng, K, x)
        bad = rng.permutation(avail.size)[:A]
        y[bad] += rng.standard_normal(A) * 4 + 2
        a2 = orc.locator_values(x, y, K, A)
        a1 = orc.locator_values_homogeneous(x, y, K, A)
        assert set(np.argsort(np.abs(a1))[:A]) == set(np.argsort(np.abs(a2))[:A]) == set(bad)
        # same polynomial up to the normalisation Q(0) = 1: a1 / a2 is one constant off the adversaries
        good = np.setdiff1d(np.arange(avail.size), bad)
        ratio = a1[good] / a2[good]
        assert np.allclose(ratio, ratio[0], rtol=1e-5)


def test_locator_invariant_to_scaling_predictions():
    rng = np.random.default_rng(22)
    K, A, W = 3, 2, 10
    _, beta = orc.chebyshev_nodes(K, W)
    x = beta
    y = _rational_samples(rng, K, x)
    y[[2, 7]] += [3.0, -2.0]
    a = orc.locator_values(x, y, K, A)
    a_scaled = orc.locator_values(x, 1000.0 * y, K, A)        # P scales, Q does not
    assert np.allclose(a, a_scaled, rtol=1e-6, atol=1e-9)


def test_pick_and_vote_conventions():
    # parity unpinned by the paper: ties -> smaller worker index first; output ascending
    avail = np.array([1, 3, 4, 8, 9])
    a = np.array([0.5, -0.1, 0.1, 2.0, -0.1])
    assert list(orc.pick_smallest(a, avail, 2)) == [3, 4]        # |a| ties at 0.1: workers 3, 4, 9 -> 3, 4
    assert list(orc.pick_smallest(a, avail, 3)) == [3, 4, 9]
    I = np.array([[7, 2], [2, 7], [5, 2], [7, 5], [1, 5]])        # counts: 2->3, 7->3, 5->3, 1->1
    adv, counts = orc.vote(I, 10, 2)
    assert list(adv) == [2, 5] and counts[2] == 3 and counts[7] == 3 and counts[1] == 1
    adv, _ = orc.vote(np.array([[9, 0], [9, 0], [9, 4]]), 10, 2)
    assert list(adv) == [0, 9]                                    # returned ascending
    assert adv.dtype == np.int32


def test_locate_and_decode_byzantine_on_linear_model_groups():
    # the "byzantine" workload at CPU size: linear hosted model => coded predictions are exactly
    # rational in beta, so the planted adversaries must be found in every group (Theorem 1),
    # even after the predictions are rounded to float32.
    w = syn.scaled(syn.WORKLOADS["byzantine"], G=48)
    alpha, beta = orc.chebyshev_nodes(w.K, w.W)
    X = syn.queries(w)
    params = syn.model_params(w)
    clean = syn.model_apply(w, params, orc.encode(X, alpha, beta))
    mask = syn.masks(w)
    adv_true = syn.adversaries(w, mask)
    Y = syn.corrupt(w, clean, adv_true)
    assert Y.dtype == np.float32
    out, adv, st = orc.decode_byzantine(Y, mask, alpha, beta, w.S, w.A)
    assert np.all(st == 0)
    assert np.array_equal(adv, adv_true)
    # decoding after exclusion equals plain decoding with the adversaries masked out as stragglers
    mask2 = mask.copy()
    for g in range(w.G):
        mask2[g, adv_true[g]] = 0
    out2, st2 = orc.decode(Y, mask2, alpha, beta, w.S + w.A)
    assert np.all(st2 == 0) and np.array_equal(out, out2)
    # and it is far closer to the true predictions than decoding with the adversaries left in
    truth = syn.model_apply(w, params, X)
    out_dirty, _ = orc.decode(Y, mask, alpha, beta, w.S)
    assert np.median(np.abs(out - truth)) < 0.25 * np.median(np.abs(out_dirty - truth))


def test_algorithm1_as_the_group_locator_on_linear_model_groups():
    # the same groups through Algorithm 1's homogeneous fit (per class, same picks and vote): on
    # exactly rational data its null vector is the error locator times q (Appendix A), so it finds
    # the same workers and the decoded group is the same
    w = syn.scaled(syn.WORKLOADS["byzantine"], G=24)
    alpha, beta = orc.chebyshev_nodes(w.K, w.W)
    clean = syn.model_apply(w, syn.model_params(w), orc.encode(syn.queries(w), alpha, beta))
    mask = syn.masks(w)
    adv_true = syn.adversaries(w, mask)
    Y = syn.corrupt(w, clean, adv_true)
    out1, adv1, st1 = orc.decode_byzantine(Y, mask, alpha, beta, w.S, w.A, locator=orc.LOCATOR_ALGORITHM_1)
    out2, adv2, st2 = orc.decode_byzantine(Y, mask, alpha, beta, w.S, w.A)
    assert np.all(st1 == 0) and np.array_equal(adv1, adv_true) and np.array_equal(adv2, adv_true)
    assert np.array_equal(out1, out2)
    # and per class: every class's picks are the planted workers
    for g in range(4):
        avail = np.nonzero(mask[g])[0]
        _, I, counts = orc.locate(Y[g], avail, beta, w.K, w.A, orc.LOCATOR_ALGORITHM_1)
        assert np.array_equal(np.sort(I, axis=1), np.tile(adv_true[g], (Y.shape[2], 1)))
        assert counts.sum() == Y.shape[2] * w.A


def test_algorithm1_is_invariant_to_scaling_predictions_and_coefficients():
    # a null vector is defined up to a factor: a_i = Q(x_i) may come back with either sign and any
    # length, the order of the |a_i| may not change; scaling the predictions rescales P only
    rng = np.random.default_rng(8)
    K, A, W = 3, 2, 12
    _, beta = orc.chebyshev_nodes(K, W)
    x = beta[np.sort(rng.permutation(W)[: 2 * (K + A)])]
    y = _rational_samples(rng, K, x)
    y[[1, 6]] += [3.0, -2.0]
    a = orc.locator_values_homogeneous(x, y, K, A)
    b = orc.locator_values_homogeneous(x, 64.0 * y, K, A)
    assert set(np.argsort(np.abs(a))[:A]) == set(np.argsort(np.abs(b))[:A]) == {1, 6}
    good = np.setdiff1d(np.arange(x.size), [1, 6])
    r = a[good] / b[good]
    assert np.allclose(r, r[0], rtol=1e-6)
    # the fit itself: P(x_i) - y_i Q(x_i) = 0 off the adversaries means Q(x_i) (y_i - r(x_i)) = 0, so on
    # the adversaries, where y_i != r(x_i), Q vanishes: |a| there is at rounding level of the rest
    assert np.max(np.abs(a[[1, 6]])) < 1e-8 * np.min(np.abs(a[good]))


def test_decode_byzantine_status():
    K, A, S = 2, 1, 1
    W = 2 * (K + A) + S
    alpha, beta = orc.chebyshev_nodes(K, W)
    Y = np.random.default_rng(3).standard_normal((2, W, 3))
    mask = np.ones((2, W), np.uint8)
    mask[0, 2] = 0                     # ok: W-S ones
    out, adv, st = orc.decode_byzantine(Y, mask, alpha, beta, S, A)
    assert list(st) == [0, 1] and np.all(out[1] == 0) and np.all(adv[1] == -1)
    assert adv[0, 0] != 2              # a straggler can never be named an adversary


def test_decode_byzantine_with_per_group_straggler_counts():
    # S = None: groups differ in how many workers returned; each needs 2(K+A) of them (eq. (3))
    K, A, W, C = 2, 1, 10, 4
    alpha, beta = orc.chebyshev_nodes(K, W)
    rng = np.random.default_rng(8)
    X = rng.uniform(0, 1, (4, K, 16))
    Mf = rng.standard_normal((16, C))
    Y = orc.encode(X, alpha, beta) @ Mf                    # exactly rational in beta
    mask = np.zeros((4, W), np.uint8)
    counts = [10, 6, 5, 8]                                 # 5 < 2(K+A) = 6: refused
    planted = []
    for g, n in enumerate(counts):
        avail = np.sort(rng.permutation(W)[:n])
        mask[g, avail] = 1
        bad = int(rng.permutation(avail)[0])
        planted.append(bad)
        Y[g, bad] += 5.0 * rng.standard_normal(C)
    out, adv, st = orc.decode_byzantine(Y, mask, alpha, beta, None, A)
    assert list(st) == [0, 0, 1, 0]
    assert np.all(out[2] == 0) and adv[2, 0] == -1
    for g in (0, 1, 3):
        assert adv[g, 0] == planted[g]
        one, adv1, st1 = orc.decode_byzantine(Y[g:g + 1], mask[g:g + 1], alpha, beta, W - counts[g], A)
        assert st1[0] == 0 and np.array_equal(out[g], one[0]) and np.array_equal(adv[g], adv1[0])


@pytest.mark.parametrize("real", [0, 1])
def test_fewer_real_adversaries_are_still_located(real):
    # Appendix A: Q = q * Lambda with Lambda vanishing at the corrupted nodes.  With fewer than A corrupted
    # workers the fit has a free factor, but every solution still vanishes at the real ones: they are
    # always among the A located, the other picks are innocent workers.
    K, A, S, W, C = 4, 2, 1, 13, 6
    alpha, beta = orc.chebyshev_nodes(K, W)
    rng = np.random.default_rng(31 + real)
    for trial in range(20):
        X = rng.uniform(0, 1, (1, K, 24))
        Mf = rng.standard_normal((24, C))
        Y = (orc.encode(X, alpha, beta) @ Mf)[0]
        avail = np.sort(rng.permutation(W)[: W - S])
        ok = avail[np.abs(beta[avail]) > 1e-9]
        bad = np.sort(rng.permutation(ok)[:real])
        Y[bad] += 3.0 * rng.standard_normal((real, C))
        adv, I, counts = orc.locate(Y, avail, beta, K, A)
        assert set(bad.tolist()) <= set(adv.tolist())
        assert len(set(adv.tolist())) == A and set(adv.tolist()) <= set(avail.tolist())


def test_algorithm3_is_exact_in_float64_and_fragile_on_float32_data():
    # Appendix A: r = P / Q reconstructs the rational function exactly (Theorem 2), and the paper's closing
    # remark: the division is prone to round-off.  With a linear model the coded predictions are exactly
    # rational in beta: from float64 data P/Q returns f(X_j) itself to ~1e-8; once the same data are rounded
    # to float32 (1e-7 relative), single groups are off by more than 1e-2 while the typical one is at 1e-5.
    # Locating and dropping the adversaries first, then Berrut, has no such tail: its error is the method's
    # own approximation error, the same for both precisions.
    K, A, S, N, C, G = 8, 2, 4, 24, 4, 50
    alpha, beta = orc.chebyshev_nodes(K, N)
    results = {}
    for single in (False, True):
        rng = np.random.default_rng(82)
        X = rng.uniform(0, 1, (G, K, 32))
        Mf = rng.standard_normal((32, C)) / 4
        truth = X @ Mf
        clean = orc.encode(X, alpha, beta) @ Mf
        e_div, e_ber = [], []
        for g in range(G):
            avail = np.sort(rng.permutation(N)[: N - S])
            bad = np.sort(rng.permutation(avail)[:A])
            Y = clean[g].copy()
            Y[bad] += 10 * clean.std() * rng.standard_normal((A, C))
            if single:
                Y = Y.astype(np.float32).astype(np.float64)
            r = np.stack([orc.rational_reconstruction(beta[avail], Y[avail, c], K, A, alpha) for c in range(C)], axis=1)
            mask = np.zeros((1, N), np.uint8)
            mask[0, avail] = 1
            out, located, _ = orc.decode_byzantine(Y[None], mask, alpha, beta, S, A, 1)
            assert np.array_equal(located[0], bad)
            scale = np.abs(truth[g]).max()
            e_div.append(np.abs(r - truth[g]).max() / scale)
            e_ber.append(np.abs(out[0] - truth[g]).max() / scale)
        results[single] = (np.array(e_div), np.array(e_ber))
    exact, _ = results[False]
    fragile, berrut32 = results[True]
    _, berrut64 = results[False]
    assert exact.max() < 1e-6
    assert np.median(fragile) < 1e-4 and fragile.max() > 1e-2 and fragile.max() > 1e3 * np.median(fragile)
    assert np.allclose(berrut32, berrut64, rtol=1e-3, atol=1e-6) and berrut32.max() < 1.0


def test_decode_rational_returns_the_hosted_function_on_exactly_rational_data():
    # Theorem 2: with a linear model and at most A lying workers P / Q is f o u itself, so reading it at the query
    # nodes returns f(X_j); float64 data, per-group masks, a refused group
    K, A, N, C, G = 3, 1, 12, 5, 6
    rng = np.random.default_rng(31)
    alpha, beta = orc.chebyshev_nodes(K, N)
    X = rng.uniform(0, 1, (G, K, 16))
    Mf = rng.standard_normal((16, C))
    truth = X @ Mf
    Y = orc.encode(X, alpha, beta) @ Mf
    mask = np.zeros((G, N), np.uint8)
    for g in range(G):
        cnt = 2 * (K + A) - 1 if g == 2 else int(rng.integers(2 * (K + A), N + 1))
        avail = np.sort(rng.permutation(N)[:cnt])
        mask[g, avail] = 1
        Y[g, rng.permutation(avail)[:A]] += 5.0 * rng.standard_normal((A, C))
    out, st = orc.decode_rational(Y, mask, alpha, beta, None, A)
    assert list(st) == [0, 0, 1, 0, 0, 0] and np.all(out[2] == 0.0)
    good = st == 0
    assert np.max(np.abs(out[good] - truth[good])) < 1e-8 * np.abs(truth).max()
    # fixed straggler count: a group with another count is refused
    out2, st2 = orc.decode_rational(Y, mask, alpha, beta, N - int(mask[0].sum()), A)
    assert st2[0] == 0 and np.array_equal(out2[0], out[0])
    assert np.all(st2[mask.sum(axis=1) != mask[0].sum()] == 1)
    # K = 1: replication, every honest worker returns f(X_0) and P / Q is that constant
    alpha1, beta1 = orc.chebyshev_nodes(1, 6)
    Y1 = np.full((1, 6, 2), 3.25)
    Y1[0, 4] = -7.0
    out1, _ = orc.decode_rational(Y1, np.ones((1, 6), np.uint8), alpha1, beta1, 0, 1)
    assert np.max(np.abs(out1 - 3.25)) < 1e-10

