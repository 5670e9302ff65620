"""Pins for the oracle's encoder and decoder (no GPU)."""
import itertools
import math
from fractions import Fraction

import numpy as np
import pytest

from oracle import approxifer_oracle as orc


def _berrut_eval_scalar(z, nodes, signs, values):
    """Direct evaluation of eq. (1)-(2) for one point with python floats, term by
    term, written independently of the oracle's vectorised routine."""
    num = 0.0
    den = 0.0
    for xi, si, fi in zip(nodes, signs, values):
        t = si / (z - xi)
        num += t * fi
        den += t
    return num / den


# ----------------------------------------------------------------------------
# encoder
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("K,W", [(4, 6), (12, 20)])
def test_encode_constant_queries_reproduce(K, W):
    # the basis functions sum to one, so identical queries give identical coded queries
    alpha, beta = orc.chebyshev_nodes(K, W)
    v = np.random.default_rng(0).uniform(0, 1, 33)
    X = np.broadcast_to(v, (2, K, 33)).copy()
    coded = orc.encode(X, alpha, beta)
    assert coded.shape == (2, W, 33)
    assert np.max(np.abs(coded - v)) < 1e-13


def test_encode_commutes_with_affine_model():
    # f(x) = Mx + b: f(u(beta_i)) = sum_j l_j(beta_i) f(X_j) because sum_j l_j = 1
    rng = np.random.default_rng(1)
    K, W, D, C = 5, 9, 40, 7
    alpha, beta = orc.chebyshev_nodes(K, W)
    X = rng.standard_normal((3, K, D))
    M, b = rng.standard_normal((D, C)), rng.standard_normal(C)
    lhs = orc.encode(X, alpha, beta) @ M + b
    rhs = orc.encode(X @ M + b, alpha, beta)
    assert np.allclose(lhs, rhs, atol=1e-11)


def test_encode_is_linear_and_elementwise_in_D():
    rng = np.random.default_rng(2)
    K, W, D = 4, 6, 10
    alpha, beta = orc.chebyshev_nodes(K, W)
    X1, X2 = rng.standard_normal((2, 1, K, D))
    assert np.allclose(orc.encode(2 * X1 - 3 * X2, alpha, beta),
                       2 * orc.encode(X1, alpha, beta) - 3 * orc.encode(X2, alpha, beta), atol=1e-12)
    # each feature is coded on its own: coding column d alone gives the same column
    full = orc.encode(X1, alpha, beta)
    for d in (0, 7):
        assert np.allclose(orc.encode(X1[:, :, d:d + 1], alpha, beta)[..., 0], full[..., d], rtol=0, atol=1e-14)


def test_encode_matches_scalar_definition():
    rng = np.random.default_rng(3)
    K, W, D = 6, 10, 3
    alpha, beta = orc.chebyshev_nodes(K, W)
    X = rng.standard_normal((2, K, D)).astype(np.float32)
    coded = orc.encode(X, alpha, beta)
    signs = [(-1) ** j for j in range(K)]
    for g, i, d in itertools.product(range(2), range(W), range(D)):
        want = _berrut_eval_scalar(float(beta[i]), [float(a) for a in alpha], signs, [float(v) for v in X[g, :, d]])
        assert coded[g, i, d] == pytest.approx(want, rel=1e-12, abs=1e-13)


def test_encode_through_query_when_nodes_coincide():
    # K=2, W=5: beta_1 = alpha_0 and beta_3 = alpha_1, the coded query IS the query
    alpha, beta = orc.chebyshev_nodes(2, 5)
    beta = beta.copy()
    beta[1], beta[3] = alpha[0], alpha[1]           # make the coincidence exact in floating point
    X = np.random.default_rng(4).standard_normal((1, 2, 8))
    coded = orc.encode(X, alpha, beta)
    assert np.array_equal(coded[0, 1], X[0, 0]) and np.array_equal(coded[0, 3], X[0, 1])


def test_k2_w3_coded_queries_closed_form():
    # K=2, S=1 (the paper's example figure): coded queries are the line through X_0, X_1 at z = 1, 0, -1
    alpha, beta = orc.chebyshev_nodes(2, 3)
    X = np.array([[[2.0, -1.0], [4.0, 3.0]]])
    coded = orc.encode(X, alpha, beta)[0]
    r = math.sqrt(2.0)
    mid = (X[0, 0] + X[0, 1]) / 2
    half = (X[0, 0] - X[0, 1]) / 2
    assert np.allclose(coded[0], mid + r * half, atol=1e-14)
    assert np.allclose(coded[1], mid, atol=1e-14)
    assert np.allclose(coded[2], mid - r * half, atol=1e-14)


# ----------------------------------------------------------------------------
# decoder
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("mode", [0, 1])
def test_decode_without_stragglers_is_direct_berrut(mode):
    rng = np.random.default_rng(5)
    K, W, C = 4, 7, 5
    alpha, beta = orc.chebyshev_nodes(K, W)
    Y = rng.standard_normal((2, W, C)).astype(np.float32)
    out, st = orc.decode(Y, np.ones((2, W), np.uint8), alpha, beta, 0, mode)
    assert np.all(st == 0)
    signs = [(-1) ** i for i in range(W)]
    for g, j, c in itertools.product(range(2), range(K), range(C)):
        want = _berrut_eval_scalar(float(alpha[j]), [float(b) for b in beta], signs, [float(v) for v in Y[g, :, c]])
        assert out[g, j, c] == pytest.approx(want, rel=1e-12, abs=1e-13)


def test_decode_sign_modes_definition_with_stragglers():
    # W=6, workers 1 and 4 missing: F = {0,2,3,5}
    K, W = 3, 6
    alpha, beta = orc.chebyshev_nodes(K, W)
    F = [0, 2, 3, 5]
    Y = np.random.default_rng(6).standard_normal((1, W, 2))
    Y[0, [1, 4], :] = np.nan                        # never read
    mask = np.zeros((1, W), np.uint8)
    mask[0, F] = 1
    for mode, signs in ((0, [1, 1, -1, -1]), (1, [1, -1, 1, -1])):
        out, st = orc.decode(Y, mask, alpha, beta, 2, mode)
        assert st[0] == 0 and np.all(np.isfinite(out))
        for j, c in itertools.product(range(K), range(2)):
            want = _berrut_eval_scalar(float(alpha[j]), [float(beta[i]) for i in F], signs, [float(Y[0, i, c]) for i in F])
            assert out[0, j, c] == pytest.approx(want, rel=1e-12)


@pytest.mark.parametrize("mode", [0, 1])
def test_decode_constants_and_interpolation_at_worker_nodes(mode):
    rng = np.random.default_rng(8)
    K, W, S, C = 4, 8, 3, 6
    _, beta = orc.chebyshev_nodes(K, W)
    mask = np.zeros((1, W), np.uint8)
    F = [0, 2, 3, 6, 7]
    mask[0, F] = 1
    # constants reproduce
    alpha = rng.uniform(-0.9, 0.9, K)
    Yc = np.broadcast_to(rng.standard_normal(C), (1, W, C)).copy()
    out, _ = orc.decode(Yc, mask, alpha, beta, S, mode)
    assert np.allclose(out, Yc[:, :K], atol=1e-12)
    # r passes through the returned predictions: evaluate at the surviving worker nodes themselves
    Y = rng.standard_normal((1, W, C))
    out, _ = orc.decode(Y, mask, beta[F][:K], beta, S, mode)
    assert np.array_equal(out[0], Y[0, F[:K]])


def test_k2_w3_affine_model_recovery():
    # K=2, W=3, f affine.  f(u(z)) is then a straight line in z, sampled at z = 1, 0, -1.
    # Rank signs (mode 1) on two surviving nodes is linear interpolation: exact for every mask.
    # Worker-index signs (mode 0) equal rank signs for F={0,1} and F={1,2}; for F={0,2} the two
    # terms carry the same sign and r(z) = [(z+1)Y_0 + (z-1)Y_2]/(2z), which is not the line.
    alpha, beta = orc.chebyshev_nodes(2, 3)
    rng = np.random.default_rng(9)
    X = rng.standard_normal((1, 2, 6))
    M, b = rng.standard_normal((6, 3)), rng.standard_normal(3)
    truth = X @ M + b
    Y = orc.encode(X, alpha, beta) @ M + b
    for F in ([0, 1], [1, 2], [0, 2]):
        mask = np.zeros((1, 3), np.uint8)
        mask[0, F] = 1
        out1, _ = orc.decode(Y, mask, alpha, beta, 1, 1)
        assert np.allclose(out1, truth, atol=1e-12)
        out0, _ = orc.decode(Y, mask, alpha, beta, 1, 0)
        if F == [0, 2]:
            a = math.sqrt(2) / 2
            for j, z in enumerate((a, -a)):
                want = ((z + 1) * Y[0, 0] + (z - 1) * Y[0, 2]) / (2 * z)
                assert np.allclose(out0[0, j], want, atol=1e-12)
            assert not np.allclose(out0, truth, atol=1e-3)
        else:
            assert np.allclose(out0, truth, atol=1e-12)


def test_k2_w3_mode_weights_exact():
    # worked example: nodes (1, 0, -1), F = {0, 2}, z = sqrt(2)/2
    alpha, beta = orc.chebyshev_nodes(2, 3)
    w0 = orc.decode_weights(alpha, beta, [0, 2], 0)[0]
    w1 = orc.decode_weights(alpha, beta, [0, 2], 1)[0]
    a = math.sqrt(2) / 2
    assert np.allclose(w0, [(a + 1) / (2 * a), (a - 1) / (2 * a)], atol=1e-15)    # (1.2071, -0.2071)
    assert np.allclose(w1, [(a + 1) / 2, (1 - a) / 2], atol=1e-15)                # (0.8536, 0.1464)


def test_decode_weights_exact_rational():
    # rational nodes: compare with Fractions, both sign modes, with a gap in F
    beta = [Fraction(1), Fraction(1, 2), Fraction(-1, 4), Fraction(-3, 4), Fraction(-1)]
    alpha = [Fraction(2, 3), Fraction(-1, 3)]
    F = [0, 1, 3, 4]
    for mode in (0, 1):
        got = orc.decode_weights([float(a) for a in alpha], [float(b) for b in beta], F, mode)
        for j, z in enumerate(alpha):
            t = []
            for r, i in enumerate(F):
                sign = (-1) ** (i if mode == 0 else r)
                t.append(Fraction(sign) / (z - beta[i]))
            tot = sum(t)
            assert np.allclose(got[j], [float(v / tot) for v in t], rtol=1e-13, atol=1e-15)


def test_decode_status_on_wrong_popcount():
    K, W, S = 2, 4, 1
    alpha, beta = orc.chebyshev_nodes(K, W)
    Y = np.ones((3, W, 2))
    mask = np.array([[1, 1, 1, 0], [1, 1, 0, 0], [1, 1, 1, 1]], np.uint8)
    out, st = orc.decode(Y, mask, alpha, beta, S)
    assert list(st) == [0, 1, 1]
    assert np.all(out[1:] == 0) and np.allclose(out[0], 1.0)


def test_decode_error_shrinks_with_more_workers():
    # Section 3 (background): convergence O(h) in the node spacing; with a smooth f and no
    # stragglers the decoding error must fall as W grows.
    K = 4
    X = np.random.default_rng(10).uniform(0, 1, (1, K, 16))
    f = lambda x: np.tanh(x @ np.linspace(-1, 1, 16 * 3).reshape(16, 3))
    errs = []
    for W in (8, 32, 128):
        alpha, beta = orc.chebyshev_nodes(K, W)
        Y = f(orc.encode(X, alpha, beta))
        out, _ = orc.decode(Y, np.ones((1, W), np.uint8), alpha, beta, 0)
        errs.append(np.max(np.abs(out - f(X))))
    assert errs[0] > errs[1] > errs[2]


def test_decode_top1_definition_and_ties():
    # Section 4.1, "Performance metric": the class of the largest decoded soft label
    rng = np.random.default_rng(31)
    K, W, S, C = 3, 5, 1, 7
    alpha, beta = orc.chebyshev_nodes(K, W)
    Y = rng.standard_normal((4, W, C))
    mask = np.ones((4, W), np.uint8)
    mask[:, 2] = 0
    mask[3, 1] = 0                                   # bad popcount
    top1, score, st = orc.decode_top1(Y, mask, alpha, beta, S, 1)
    out, _ = orc.decode(Y, mask, alpha, beta, S, 1)
    assert top1.dtype == np.int32 and list(st) == [0, 0, 0, 1] and np.all(top1[3] == -1)
    for g in range(3):
        for j in range(K):
            row = list(out[g, j])
            assert top1[g, j] == row.index(max(row)) and score[g, j] == max(row)
    # identical class columns decode to identical values: the smallest class index wins
    Yt = np.repeat(rng.standard_normal((1, W, 1)), C, axis=2)
    Yt[..., 5] += 1.0
    Yt[..., 6] = Yt[..., 5]
    t, _, _ = orc.decode_top1(Yt, np.ones((1, W), np.uint8), alpha, beta, 0)
    o, _ = orc.decode(Yt, np.ones((1, W), np.uint8), alpha, beta, 0)
    assert np.array_equal(o[..., 5], o[..., 6])
    for j in range(K):
        assert t[0, j] == (5 if o[0, j, 5] > o[0, j, 0] else 0)
    # exact recovery case (K=2, W=3, affine model, survivor-rank signs): top-1 equals the true top-1
    alpha, beta = orc.chebyshev_nodes(2, 3)
    X = rng.standard_normal((5, 2, 6))
    Mf, b = rng.standard_normal((6, 4)), rng.standard_normal(4)
    Yc = orc.encode(X, alpha, beta) @ Mf + b
    m = np.ones((5, 3), np.uint8)
    m[:, 1] = 0
    t, _, _ = orc.decode_top1(Yc, m, alpha, beta, 1, 1)
    assert np.array_equal(t, np.argmax(X @ Mf + b, axis=2))


def test_worker_index_signs_can_have_a_real_pole():
    # K=3, five workers, the middle worker missing: with the printed worker-index signs the survivors
    # carry (+,-,-,+) on the symmetric nodes (1, a, -a, -1), and at the middle query node alpha_1 = 0 the
    # denominator 1/(0-1) - 1/(0-a) - 1/(0+a) + 1/(0+1) cancels exactly: r has a pole there.  Berrut's
    # alternation by rank (+,-,+,-) has none (Section 3, background: no pole on the real line).
    alpha, beta = orc.chebyshev_nodes(3, 5)
    F = [0, 1, 3, 4]
    with np.errstate(divide="ignore", invalid="ignore"):
        w0 = orc.decode_weights(alpha, beta, F, 0)
    w1 = orc.decode_weights(alpha, beta, F, 1)
    assert not np.all(np.isfinite(w0[1]))
    assert np.all(np.isfinite(w1)) and np.allclose(w1.sum(axis=1), 1.0)


def test_decode_with_per_group_straggler_counts():
    # S = None: each group is decoded over however many workers its own mask names; that must equal
    # decoding the group alone with its own count, and a mask without survivors is refused
    K, W, C = 3, 9, 5
    alpha, beta = orc.chebyshev_nodes(K, W)
    rng = np.random.default_rng(21)
    Y = rng.standard_normal((6, W, C))
    mask = np.zeros((6, W), np.uint8)
    counts = [9, 1, 4, 0, 3, 7]
    for g, n in enumerate(counts):
        mask[g, rng.permutation(W)[:n]] = 1
    for mode in (0, 1):
        out, st = orc.decode(Y, mask, alpha, beta, None, mode)
        assert list(st) == [0, 0, 0, 1, 0, 0]
        assert np.all(out[3] == 0)
        for g, n in enumerate(counts):
            if n == 0:
                continue
            one, st1 = orc.decode(Y[g:g + 1], mask[g:g + 1], alpha, beta, W - n, mode)
            assert st1[0] == 0 and np.array_equal(out[g], one[0])
        # a single survivor: every query gets that worker's prediction (replication, weights = 1)
        only = np.nonzero(mask[1])[0][0]
        assert np.allclose(out[1], Y[1, only][None, :], rtol=0, atol=0)
    out_neg, st_neg = orc.decode(Y, mask, alpha, beta, -1, 0)
    ref, _ = orc.decode(Y, mask, alpha, beta, None, 0)
    assert np.array_equal(out_neg, ref)


def test_wait_mask_hand_built_cases():
    # Section 3, "ApproxIFER Decoding", step 1: the fastest wait_for workers are the survivors
    inf, nan = np.inf, np.nan
    arrival = np.array([
        [5.0, 1.0, 3.0, 2.0, 4.0],        # plain: the three fastest are workers 1, 3, 2
        [2.0, 2.0, 1.0, 2.0, 2.0],        # ties at the cut: smaller worker index first (our convention)
        [inf, 1.0, nan, -inf, 7.0],       # only two workers ever answer
        [0.0, -1.0, -2.0, 9.0, 8.0],      # negative times are ordinary times
    ])
    mask, count = orc.wait_mask(arrival, 3)
    assert mask.tolist() == [[0, 1, 1, 1, 0], [1, 1, 1, 0, 0], [0, 1, 0, 0, 1], [1, 1, 1, 0, 0]]
    assert count.tolist() == [3, 3, 2, 3]
    everyone, c5 = orc.wait_mask(arrival, 5)
    assert everyone[0].tolist() == [1] * 5 and c5.tolist() == [5, 5, 2, 5]


def test_wait_mask_then_decode_uses_the_fastest_workers():
    # the mask of the wait rule feeds the decoder: decoding with it equals decoding with the set of the
    # K fastest workers written down by hand, and slower workers' rows are never looked at
    K, W = 3, 7
    alpha, beta = orc.chebyshev_nodes(K, W)
    rng = np.random.default_rng(17)
    arrival = rng.permutation(W).astype(np.float64)[None, :]
    Y = rng.standard_normal((1, W, 4))
    mask, count = orc.wait_mask(arrival, K)
    fastest = np.sort(np.argsort(arrival[0])[:K])
    assert count[0] == K and np.array_equal(np.nonzero(mask[0])[0], fastest)
    Y_dirty = Y.copy()
    Y_dirty[0, mask[0] == 0] = np.nan
    out, st = orc.decode(Y_dirty, mask, alpha, beta, W - K, 1)
    ref = orc.decode_weights(alpha, beta, fastest, 1) @ Y[0, fastest]
    assert st[0] == 0 and np.allclose(out[0], ref, rtol=1e-14, atol=0)


def test_group_queries_is_a_view_of_the_stream_with_the_last_query_repeated():
    rng = np.random.default_rng(2)
    stream = rng.standard_normal((12, 5))
    assert np.array_equal(orc.group_queries(stream, 4), stream.reshape(3, 4, 5))      # K divides Q: the stream itself
    assert np.array_equal(orc.group_queries(stream, 1), stream[:, None, :])
    g = orc.group_queries(stream[:7], 3)                                               # 7 = 2 * 3 + 1
    assert g.shape == (3, 3, 5)
    assert np.array_equal(g.reshape(9, 5)[:7], stream[:7])                             # row q is query q
    assert np.array_equal(g[2], np.broadcast_to(stream[6], (3, 5)))
    g = orc.group_queries(stream[:8], 3)
    assert np.array_equal(g[2, 0], stream[6]) and np.array_equal(g[2, 1], stream[7]) and np.array_equal(g[2, 2], stream[7])
    assert orc.group_queries(stream[:0], 3).shape == (0, 3, 5)
    # a last group of one real query is replication: every worker gets that query (constants reproduce),
    # and any survivor set decodes it back
    K, W = 3, 5
    alpha, beta = orc.chebyshev_nodes(K, W)
    coded = orc.encode(orc.group_queries(stream[:7], K), alpha, beta)
    assert np.allclose(coded[2], np.broadcast_to(stream[6], (W, 5)), rtol=0, atol=1e-14)
    mask = np.array([[1, 0, 1, 1, 0]] * 3, np.uint8)
    out, st = orc.decode(coded, mask, alpha, beta, 2, 1)
    assert np.all(st == 0) and np.allclose(out[2], np.broadcast_to(stream[6], (K, 5)), rtol=0, atol=1e-13)

