"""Float64 CPU oracle for the ApproxIFER coding layer (arXiv 2109.09868).

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain statement of what the
coding layer computes, written from the paper.  It is used by the tests, by the
smoke check and by the benchmark's CPU-baseline leg; the GPU library never
imports it and shares no code, table or helper with it.

Notation (paper, Section 2 and Section 3):
  K        queries per group, X_0..X_{K-1}
  W        number of workers.  The paper has N+1 workers indexed 0..N; here
           W = N_paper + 1 so that every array is simply W long.
  S        stragglers (erasures); the decoder sees W-S available workers
  A        Byzantine workers (the paper's E)
  alpha_j  query nodes, Chebyshev points of the first kind
  beta_i   worker nodes, Chebyshev points of the second kind
  F        indices of the workers whose predictions enter the decoder

Every function takes float64 node arrays as arguments; inputs given in float32
are widened exactly and all arithmetic is float64.

Pins: the weights, the encoder, the decoder and the locator are pinned in
tests/test_oracle_*.py by exact-rational evaluation, closed forms, invariants
and brute force.  The tie-break conventions of `pick_smallest` and `vote`
(equal magnitudes / equal counts -> smaller worker index first) are a reading
of our own, the paper is silent on them: parity unpinned for those two
conventions.  On data that is not exactly rational (a non-linear hosted model)
Algorithm 2's system has no solution; "solve" is read as ordinary least squares,
and under that reading the fit is pinned to the exact minimiser (normal equations
over rationals on small systems); the reading itself is ours: parity unpinned.  Algorithm 1's homogeneous system is read as "the
unit coefficient vector of least residual" (smallest right singular vector); on
exactly rational data every reading gives the same null vector and the pins
hold it there, on other data: parity unpinned beyond that reading.  Algorithm 3
(`rational_reconstruction`, `decode_rational`) is pinned by Theorem 2: on exactly
rational float64 data with at most A errors it returns the hosted function itself.
"""
from __future__ import annotations

import numpy as np

SIGN_WORKER_INDEX = 0   # (-1)^i with i the worker index, as the decoder formula is printed
SIGN_SURVIVOR_RANK = 1  # (-1)^r with r the position of the node among the surviving nodes

LOCATOR_ALGORITHM_2 = 2  # Q_0 = 1, least squares: the locator of Section 4.1
LOCATOR_ALGORITHM_1 = 1  # Q_0 free, null vector of the homogeneous system (Section 2)


# --------------------------------------------------------------------------
# nodes
# --------------------------------------------------------------------------
def chebyshev_nodes(K: int, W: int):
    """Query nodes alpha_j = cos((2j+1)pi/(2K)), j=0..K-1 (first kind) and worker
    nodes beta_i = cos(i pi/(W-1)), i=0..W-1 (second kind).

    Section 3, "ApproxIFER Encoding": the definitions of alpha_j and beta_i, with
    the paper's N equal to W-1.
    """
    if K < 1 or W < 2:
        raise ValueError("need K >= 1 and W >= 2")
    j = np.arange(K, dtype=np.float64)
    i = np.arange(W, dtype=np.float64)
    alpha = np.cos((2.0 * j + 1.0) * np.pi / (2.0 * K))
    beta = np.cos(i * np.pi / (W - 1.0))
    return alpha, beta


# --------------------------------------------------------------------------
# Berrut basis functions
# --------------------------------------------------------------------------
def berrut_weights(z, x, s):
    """Matrix L[m, i] = l_i(z_m) of Berrut's basis functions on the nodes x with
    signs s_i in {+1,-1}:

        l_i(z) = (s_i / (z - x_i)) / sum_k (s_k / (z - x_k)).

    Section 3, "Rational Interpolation Background", eqs. (1)-(2), where s_i is
    (-1)^i.  At z equal to a node the interpolant passes through the data
    (Section 3, "ApproxIFER Encoding": u passes through the queries), so the row
    is the unit vector of that node; equality is tested exactly on the doubles.
    """
    z = np.asarray(z, dtype=np.float64)
    x = np.asarray(x, dtype=np.float64)
    s = np.asarray(s, dtype=np.float64)
    L = np.zeros((z.size, x.size), dtype=np.float64)
    for m in range(z.size):
        hit = np.nonzero(z[m] == x)[0]
        if hit.size:
            L[m, hit[0]] = 1.0
            continue
        t = s / (z[m] - x)
        L[m, :] = t / np.sum(t)
    return L


def alternating_signs(n: int):
    return np.where(np.arange(n) % 2 == 0, 1.0, -1.0)


# --------------------------------------------------------------------------
# encoder
# --------------------------------------------------------------------------
def encode_weights(alpha, beta):
    """W x K matrix l_j(beta_i): basis on the query nodes, evaluated at the worker
    nodes.  Section 3, "ApproxIFER Encoding": definition of l_j(z) and of the
    coded query as u(beta_i)."""
    alpha = np.asarray(alpha, dtype=np.float64)
    return berrut_weights(beta, alpha, alternating_signs(alpha.size))


def encode(X, alpha, beta):
    """Coded queries.  X is [G, K, D]; the result is [G, W, D] float64 with
    coded[g, i, :] = u_g(beta_i) = sum_j X[g, j, :] l_j(beta_i).
    Section 3, "ApproxIFER Encoding"."""
    X = np.asarray(X)
    if X.ndim != 3 or X.shape[1] != np.asarray(alpha).size:
        raise ValueError("X must be [G, K, D] with K = len(alpha)")
    L = encode_weights(alpha, beta)                       # [W, K]
    return np.einsum("ij,gjd->gid", L, X.astype(np.float64))


def group_queries(stream, K):
    """Groups of K consecutive queries out of a stream [Q, D] (Section 2, "System Architecture": the K queries of
    a group are encoded together).  Returns [G, K, D] with G = ceil(Q / K).  The paper has no rule for a stream whose
    length K does not divide; here the last group is completed by repeating the stream's last query (a reading of
    our own), and the answers of the repeats are not read back: answers [G, K, ...] flattened to [G K, ...] hold
    query q's answer in row q."""
    stream = np.asarray(stream)
    Q, D = stream.shape
    G = -(-Q // K)
    out = np.empty((G * K, D), dtype=stream.dtype)
    out[:Q] = stream
    out[Q:] = stream[Q - 1] if Q > 0 else 0
    return out.reshape(G, K, D)


# --------------------------------------------------------------------------
# decoder
# --------------------------------------------------------------------------
def decode_weights(alpha, beta, F, sign_mode=SIGN_WORKER_INDEX):
    """K x |F| matrix of the decoder's basis functions evaluated at the query nodes:

        Wdec[j, r] = (s_r / (alpha_j - beta_{F_r})) / sum_r' (s_r' / (alpha_j - beta_{F_r'})).

    Section 3, "ApproxIFER Decoding", step 2: the rational function r(z) built on
    the workers in F, read at z = alpha_j.  F is in ascending worker order.
    sign_mode 0 takes s = (-1)^(worker index) exactly as that formula is printed;
    sign_mode 1 takes s = (-1)^(rank in F), which is Berrut's interpolant (eq. (2))
    on the surviving nodes.  The two agree when no worker is missing.
    """
    F = np.asarray(F, dtype=np.int64)
    beta = np.asarray(beta, dtype=np.float64)
    if sign_mode == SIGN_WORKER_INDEX:
        s = np.where(F % 2 == 0, 1.0, -1.0)
    elif sign_mode == SIGN_SURVIVOR_RANK:
        s = alternating_signs(F.size)
    else:
        raise ValueError("sign_mode must be 0 or 1")
    return berrut_weights(alpha, beta[F], s)


def decode(Y, mask, alpha, beta, S, sign_mode=SIGN_WORKER_INDEX):
    """Approximate predictions from the workers that returned.

    Y is [G, W, C] coded predictions (rows of missing workers are never read),
    mask is [G, W] with 1 = returned.  Returns (out [G, K, C] float64, status [G]).
    status 0: decoded; status 1: the group's mask does not hold exactly W-S ones,
    its output row is left at zero.  S = None (or negative): every group brings its own
    straggler count; only a group without any survivor is refused.
    Section 3, "ApproxIFER Decoding", step 2: Y_hat_j = r(alpha_j).
    """
    Y = np.asarray(Y)
    mask = np.asarray(mask)
    G, W, C = Y.shape
    K = np.asarray(alpha).size
    out = np.zeros((G, K, C), dtype=np.float64)
    status = np.zeros(G, dtype=np.int32)
    for g in range(G):
        F = np.nonzero(mask[g] != 0)[0]
        if (F.size != W - S) if (S is not None and S >= 0) else (F.size < 1):
            status[g] = 1
            continue
        Wd = decode_weights(alpha, beta, F, sign_mode)    # [K, |F|]
        out[g] = Wd @ Y[g, F, :].astype(np.float64)
    return out, status


def decode_top1(Y, mask, alpha, beta, S, sign_mode=SIGN_WORKER_INDEX):
    """Class of the largest decoded soft label of every query, the quantity the paper scores
    (Section 4.1, "Performance metric").  Equal values: the smallest class index.
    Returns (top1 [G, K] int32 with -1 for groups whose mask is bad, score [G, K] float64, status)."""
    out, status = decode(Y, mask, alpha, beta, S, sign_mode)
    top1 = np.argmax(out, axis=2).astype(np.int32)      # first occurrence of the maximum
    score = np.max(out, axis=2)
    top1[status != 0] = -1
    return top1, score, status


# --------------------------------------------------------------------------
# wait rule
# --------------------------------------------------------------------------
def wait_mask(arrival, wait_for):
    """Survivor mask from arrival times: per group the wait_for workers that answer first get 1.
    Section 3, "ApproxIFER Decoding", step 1 (the decoder waits for the fastest K workers, or
    2(K+E) of them when E may be adversarial).  A non-finite time means the worker never answers.
    Equal times: smaller worker index first (a reading of our own; the paper is silent).
    Returns (mask [G, W] uint8, count [G] int32)."""
    arrival = np.asarray(arrival, dtype=np.float64)
    G, W = arrival.shape
    mask = np.zeros((G, W), dtype=np.uint8)
    count = np.zeros(G, dtype=np.int32)
    for g in range(G):
        answered = [i for i in range(W) if np.isfinite(arrival[g, i])]
        answered.sort(key=lambda i: (arrival[g, i], i))
        first = answered[:wait_for]
        mask[g, first] = 1
        count[g] = len(first)
    return mask, count


# --------------------------------------------------------------------------
# adversary location (Algorithm 2)
# --------------------------------------------------------------------------
def locator_system(x, y, K, A):
    """Matrix and right-hand side of Algorithm 2, steps 1-2, for one class.

    Unknowns P_0..P_{M-1}, Q_1..Q_{M-1} with M = K + A and Q_0 fixed to 1.  Row of
    node x_i:  sum_k P_k x_i^k - y_i sum_{k>=1} Q_k x_i^k = y_i.
    Returns (Amat [n, 2M-1], rhs [n]).
    """
    x = np.asarray(x, dtype=np.float64)
    y = np.asarray(y, dtype=np.float64)
    M = K + A
    V = np.vander(x, M, increasing=True)                  # x^0 .. x^{M-1}
    Amat = np.concatenate([V, -y[:, None] * V[:, 1:]], axis=1)
    return Amat, y.copy()


def locator_values(x, y, K, A):
    """a_i = Q(x_i) of Algorithm 2, step 3, with (P, Q) the ordinary least-squares
    solution of the system of step 2 (the system has one more equation than
    unknowns at the paper's minimum worker count and is inconsistent whenever the
    data are not exactly rational)."""
    M = K + A
    Amat, rhs = locator_system(x, y, K, A)
    sol = np.linalg.lstsq(Amat, rhs, rcond=None)[0]
    Qc = np.concatenate([[1.0], sol[M:]])                 # Q_0 = 1, Q_1..Q_{M-1}
    x = np.asarray(x, dtype=np.float64)
    a = np.zeros_like(x)
    for k in range(M - 1, -1, -1):                        # Horner
        a = a * x + Qc[k]
    return a


def pick_smallest(a, avail, A):
    """Algorithm 2, steps 4-5: worker indices of the A smallest |a_i|.  Equal
    magnitudes keep ascending worker order (stable sort)."""
    order = np.argsort(np.abs(a), kind="stable")
    return np.asarray(avail, dtype=np.int64)[order[:A]]


def vote(I, W, A):
    """Return step of Algorithm 2: the A most frequent worker indices in I, ties
    broken toward the smaller index, returned in ascending order."""
    counts = np.bincount(np.asarray(I, dtype=np.int64).ravel(), minlength=W)
    order = np.lexsort((np.arange(W), -counts))           # count desc, index asc
    return np.sort(order[:A]).astype(np.int32), counts


def locate(Yg, avail, beta, K, A, locator=LOCATOR_ALGORITHM_2):
    """Adversary location for one group: Algorithm 2 (or, with locator = LOCATOR_ALGORITHM_1,
    the homogeneous fit of Algorithm 1 applied class by class, with the same picks and vote).
    Yg is [W, C]; avail lists the available workers in ascending order.
    Returns (adv [A] int32 ascending, I [C, A], counts [W])."""
    Yg = np.asarray(Yg)
    avail = np.asarray(avail, dtype=np.int64)
    beta = np.asarray(beta, dtype=np.float64)
    W, C = Yg.shape
    x = beta[avail]
    I = np.zeros((C, A), dtype=np.int64)
    for c in range(C):
        y = Yg[avail, c].astype(np.float64)
        if locator == LOCATOR_ALGORITHM_1:
            a = locator_values_homogeneous(x, y, K, A)
        else:
            a = locator_values(x, y, K, A)
        I[c, :] = pick_smallest(a, avail, A)
    adv, counts = vote(I, W, A)
    return adv, I, counts


def decode_byzantine(Y, mask, alpha, beta, S, A, sign_mode=SIGN_WORKER_INDEX, locator=LOCATOR_ALGORITHM_2):
    """Locate the adversaries among the available workers (Algorithm 2; Algorithm 1's fit
    per class with locator = LOCATOR_ALGORITHM_1), drop them, decode over the rest
    (Section 4.1, "Encoding and Decoding").
    Returns (out [G, K, C] float64, adv [G, A] int32, status [G])."""
    Y = np.asarray(Y)
    mask = np.asarray(mask)
    G, W, C = Y.shape
    K = np.asarray(alpha).size
    out = np.zeros((G, K, C), dtype=np.float64)
    adv = np.full((G, A), -1, dtype=np.int32)
    status = np.zeros(G, dtype=np.int32)
    for g in range(G):
        avail = np.nonzero(mask[g] != 0)[0]
        if (avail.size != W - S) if (S is not None and S >= 0) else (avail.size < 2 * (K + A)):
            status[g] = 1                                 # S None/negative: per-group count, Section 3 eq. (3) must hold
            continue
        adv[g], _, _ = locate(Y[g], avail, beta, K, A, locator)
        F = np.setdiff1d(avail, adv[g])
        Wd = decode_weights(alpha, beta, F, sign_mode)
        out[g] = Wd @ Y[g, F, :].astype(np.float64)
    return out, adv, status


# --------------------------------------------------------------------------
# Algorithm 1 (homogeneous form) -- cross-checks Algorithm 2; the alternate locator
# --------------------------------------------------------------------------
def locator_values_homogeneous(x, y, K, A):
    """Algorithm 1: P and Q both of degree K+A-1 with Q_0 free; the coefficient
    vector is a null vector of the homogeneous system P(x_i) - y_i Q(x_i) = 0,
    taken as the right singular vector of the smallest singular value.  Returns
    a_i = Q(x_i), defined up to one common factor."""
    x = np.asarray(x, dtype=np.float64)
    y = np.asarray(y, dtype=np.float64)
    M = K + A
    V = np.vander(x, M, increasing=True)
    H = np.concatenate([V, -y[:, None] * V], axis=1)      # [n, 2M]
    _, _, Vt = np.linalg.svd(H, full_matrices=True)
    coef = Vt[-1]
    return V @ coef[M:]


# --------------------------------------------------------------------------
# Algorithm 3 (P / Q reconstruction) -- not on the serving path, kept to show why
# --------------------------------------------------------------------------
def rational_reconstruction(x, y, K, A, z):
    """Appendix A, Algorithm 3: with (P, Q) the least-squares solution of P(x_i) = y_i Q(x_i)
    (degrees K+A-1, Q_0 = 1, the system of Algorithm 2), return r(z) = P(z) / Q(z).
    Theorem 2 makes this exact for exactly rational data with at most A errors; the paper
    sets it aside because the division is fragile under round-off (P and Q share the
    error-locator factor, which nearly vanishes close to a corrupted node)."""
    M = K + A
    Amat, rhs = locator_system(x, y, K, A)
    sol = np.linalg.lstsq(Amat, rhs, rcond=None)[0]
    P = sol[:M]
    Q = np.concatenate([[1.0], sol[M:]])
    z = np.asarray(z, dtype=np.float64)
    num = np.zeros_like(z)
    den = np.zeros_like(z)
    for k in range(M - 1, -1, -1):
        num = num * z + P[k]
        den = den * z + Q[k]
    return num / den


def decode_rational(Y, mask, alpha, beta, S, A):
    """Appendix A, Algorithm 3 as a decoder for whole groups: out[g, j, c] = r_c(alpha_j) with r_c = P / Q the
    reconstruction of class c from the group's available workers (rational_reconstruction above).  No worker is
    located or dropped.  Group acceptance as in decode_byzantine.  Returns (out [G, K, C] float64, status [G])."""
    Y = np.asarray(Y)
    mask = np.asarray(mask)
    alpha = np.asarray(alpha, dtype=np.float64)
    beta = np.asarray(beta, dtype=np.float64)
    G, W, C = Y.shape
    K = alpha.size
    out = np.zeros((G, K, C), dtype=np.float64)
    status = np.zeros(G, dtype=np.int32)
    for g in range(G):
        avail = np.nonzero(mask[g] != 0)[0]
        if (avail.size != W - S) if (S is not None and S >= 0) else (avail.size < 2 * (K + A)):
            status[g] = 1
            continue
        for c in range(C):
            out[g, :, c] = rational_reconstruction(beta[avail], Y[g, avail, c], K, A, alpha)
    return out, status

