"""The allowances of the GPU parity tests, recomputed from the oracle alone (no GPU): how many groups each seeded
case sets aside as ill-conditioned, and that the rule which excuses a located set differing from the oracle's only
excuses rounding ties."""
import numpy as np
import pytest

from oracle import approxifer_oracle as orc
from parity_cases import (ILL_POSED_FUZZ_ALL, ILL_POSED_FUZZ_BYZANTINE, ILL_POSED_RAGGED, LEBESGUE_LIMIT,
                          RAGGED_DECODE_SHAPES, assert_rounding_ties, fuzz_all_cases, fuzz_byzantine_cases, lebesgue,
                          ragged_decode_case, tie_classes, well_posed)


def test_lebesgue_limit_follows_from_the_bar():
    # 2 (n + 3) u L <= 1e-5 with n <= 128 survivors and u = 2^-53
    bound = 1e-5 / (2 * 131 * 2.0 ** -53)
    assert LEBESGUE_LIMIT <= bound < 10 * LEBESGUE_LIMIT


def test_lebesgue_constant_is_the_amplification_of_the_ratio():
    # L = max_j sum|t| / |sum t| with t_i = s_i / (alpha_j - beta_i), written out term by term
    K, N = 5, 12
    alpha, beta = orc.chebyshev_nodes(K, N)
    F = np.array([0, 1, 4, 6, 7, 11])
    for mode in (0, 1):
        worst = 0.0
        for j in range(K):
            t = [((-1.0) ** (F[r] if mode == 0 else r)) / (alpha[j] - beta[F[r]]) for r in range(F.size)]
            worst = max(worst, sum(abs(v) for v in t) / abs(sum(t)))
        assert abs(lebesgue(alpha, beta, F, mode) - worst) <= 1e-12 * worst


@pytest.mark.parametrize("K,N,C,G", RAGGED_DECODE_SHAPES)
@pytest.mark.parametrize("mode", [0, 1])
def test_ragged_cases_set_aside_exactly_the_listed_groups(K, N, C, G, mode):
    alpha, beta, Y, mask = ragged_decode_case(K, N, C, G, mode)
    with np.errstate(all="ignore"):
        ref, st = orc.decode(Y, mask, alpha, beta, None, mode)
    assert st[2] == 1 and st.sum() == 1
    finite = np.all(np.isfinite(ref.reshape(G, -1)), axis=1) & (st == 0) & well_posed(alpha, beta, mask, mode)
    assert G - 1 - finite.sum() == ILL_POSED_RAGGED.get((K, N, C, G, mode), 0)


def test_the_one_ragged_group_set_aside_has_a_pole_on_a_query_node():
    K, N, C, G, mode = 3, 9, 5, 12, 0
    alpha, beta, Y, mask = ragged_decode_case(K, N, C, G, mode)
    bad = [g for g in range(G) if mask[g].any() and not well_posed(alpha, beta, mask[g:g + 1], mode)[0]]
    assert len(bad) == 1
    F = np.nonzero(mask[bad[0]])[0]
    # the denominator sum_i (-1)^i / (alpha_j - beta_i) cancels to rounding noise (or exactly) at a query node
    worst = min(abs(sum((-1.0) ** i / (alpha[j] - beta[i]) for i in F)) /
                sum(abs(1.0 / (alpha[j] - beta[i])) for i in F) for j in range(K))
    assert worst < 1e-8
    assert well_posed(alpha, beta, mask[bad[0]:bad[0] + 1], 1)[0]          # Berrut's own signs have no pole


def test_fuzz_cases_set_aside_exactly_the_listed_groups():
    set_aside = 0
    for t in fuzz_all_cases():
        with np.errstate(all="ignore"):
            ref, _ = orc.decode(t["Y"], t["mask"], t["alpha"], t["beta"], t["S"], t["mode"])
        finite = np.all(np.isfinite(ref.reshape(t["G"], -1)), axis=1) & well_posed(t["alpha"], t["beta"], t["mask"],
                                                                                   t["mode"])
        set_aside += int(t["G"] - finite.sum())
    assert set_aside == ILL_POSED_FUZZ_ALL


def test_byzantine_fuzz_cases_set_aside_exactly_the_listed_groups():
    # Algorithm 2's sets on the oracle's side; the planted adversaries come back, so both locators drop the same workers
    set_aside = 0
    for t in fuzz_byzantine_cases():
        _, adv_ref, st = orc.decode_byzantine(t["Y"], t["mask"], t["alpha"], t["beta"], None if t["ragged"] else t["S"],
                                              t["A"], t["mode"])
        assert np.all(st == 0)
        for g in range(t["G"]):
            m2 = t["mask"][g:g + 1].copy()
            m2[0, adv_ref[g]] = 0
            set_aside += 0 if well_posed(t["alpha"], t["beta"], m2, t["mode"])[0] else 1
    assert set_aside == ILL_POSED_FUZZ_BYZANTINE


def _planted(seed, K=4, A=1, N=12, C=6, G=8):
    rng = np.random.default_rng(seed)
    alpha, beta = orc.chebyshev_nodes(K, N)
    X = rng.uniform(0, 1, (G, K, 32))
    clean = (orc.encode(X, alpha, beta) @ (rng.standard_normal((32, C)) / 6)).astype(np.float32)
    mask = np.ones((G, N), np.uint8)
    adv = np.zeros((G, A), np.int32)
    Y = clean.copy()
    for g in range(G):
        adv[g] = np.sort(rng.permutation(N)[:A])
        Y[g, adv[g]] += (10 * clean.std() * rng.standard_normal((A, C))).astype(np.float32)
    return alpha, beta, Y, mask, adv, K, A


def test_rounding_tie_rule_rejects_a_wrong_set_on_clear_data():
    # exactly rational data with a planted adversary: every class separates by orders of magnitude, no class is a
    # tie, and a located set that differs from the oracle's must be refused
    alpha, beta, Y, mask, adv, K, A = _planted(5)
    ref = np.stack([orc.locate(Y[g], np.arange(mask.shape[1]), beta, K, A)[0] for g in range(Y.shape[0])])
    assert np.array_equal(ref, adv)
    for g in range(Y.shape[0]):
        assert tie_classes(Y[g], np.arange(mask.shape[1]), beta, K, A) == []
    assert assert_rounding_ties(Y, mask, beta, K, A, ref, ref) == 0
    wrong = ref.copy()
    wrong[3, 0] = (wrong[3, 0] + 1) % mask.shape[1]
    with pytest.raises(AssertionError):
        assert_rounding_ties(Y, mask, beta, K, A, wrong, ref)


def test_rounding_tie_rule_accepts_a_genuine_tie_and_bounds_its_reach():
    # no adversary at all and A = 1, a single class: Q is the denominator of an exactly rational function, nothing
    # vanishes, and two workers at mirrored nodes can carry the same |a| to the last bits -- here the tie is made
    # exact by symmetric data (an even function of the node), so either of the two is a fair answer
    K, A, N = 2, 1, 8
    _, beta = orc.chebyshev_nodes(K, N)
    y = (1.0 / (1.0 + 0.3 * beta ** 2)).astype(np.float32)          # even in the node: a_i = a_(N-1-i)
    Y = y[None, :, None].copy()
    mask = np.ones((1, N), np.uint8)
    assert tie_classes(Y[0], np.arange(N), beta, K, A) == [0]
    ref = orc.locate(Y[0], np.arange(N), beta, K, A)[0][None, :]
    mirrored = (N - 1 - ref).astype(np.int32)
    assert assert_rounding_ties(Y, mask, beta, K, A, mirrored, ref) == (0 if np.array_equal(mirrored, ref) else 1)
    # but a worker that is not available is never excused
    m2 = mask.copy()
    m2[0, mirrored[0, 0]] = 0
    if not np.array_equal(mirrored, ref):
        with pytest.raises(AssertionError):
            assert_rounding_ties(Y, m2, beta, K, A, mirrored, orc.locate(Y[0], np.nonzero(m2[0])[0], beta, K, A)[0][None, :])
