"""How sharp are the oracle's pins?  (no GPU)

Every case below plants ONE plausible mistake in the oracle -- a dropped term, a wrong sign or index,
a swapped operand, an off-by-one in the node formula -- and re-runs the pin tests of
tests/test_oracle_*.py against the mistaken oracle.  At least one pin has to fail for every mistake;
with no mistake planted, every pin passes.  The mistakes live in the CPU oracle only.
"""
import itertools

import numpy as np
import pytest

from oracle import approxifer_oracle as orc

import test_oracle_codec
import test_oracle_locator
import test_oracle_weights

PIN_MODULES = (test_oracle_weights, test_oracle_codec, test_oracle_locator)


def _cases(fn):
    """Keyword-argument sets of a test function: the product of its parametrize marks."""
    axes = []
    for mark in getattr(fn, "pytestmark", []):
        if mark.name != "parametrize":
            continue
        names = [n.strip() for n in mark.args[0].split(",")] if isinstance(mark.args[0], str) else list(mark.args[0])
        rows = []
        for value in mark.args[1]:
            value = value if len(names) > 1 else (value,)
            rows.append(dict(zip(names, value)))
        axes.append(rows)
    for combo in itertools.product(*axes):
        kw = {}
        for part in combo:
            kw.update(part)
        yield kw


def run_pins():
    """Runs every pin; returns the names of those that fail (assertion or any other error)."""
    failed = []
    for mod in PIN_MODULES:
        for name in sorted(dir(mod)):
            fn = getattr(mod, name)
            if not name.startswith("test_") or not callable(fn):
                continue
            for kw in _cases(fn):
                try:
                    with np.errstate(all="ignore"):
                        fn(**kw)
                except Exception:                      # noqa: BLE001 - any failure is a detection
                    failed.append("%s.%s%s" % (mod.__name__.split(".")[-1], name, kw or ""))
    return failed


def test_unmutated_oracle_passes_every_pin():
    assert run_pins() == []


# ---- the planted mistakes -------------------------------------------------------------------------
def _nodes_paper_n_confused(K, W):
    # the paper has N+1 workers with beta_i = cos(i pi / N): dividing by the worker count instead
    alpha, _ = _ORIG["chebyshev_nodes"](K, W)
    return alpha, np.cos(np.arange(W) * np.pi / W)


def _nodes_kinds_swapped(K, W):
    alpha = np.cos(np.arange(K) * np.pi / max(K - 1, 1))
    beta = np.cos((2.0 * np.arange(W) + 1.0) * np.pi / (2.0 * W))
    return alpha, beta


def _nodes_alpha_denominator(K, W):
    _, beta = _ORIG["chebyshev_nodes"](K, W)
    return np.cos((2.0 * np.arange(K) + 1.0) * np.pi / (2.0 * K + 1.0)), beta


def _weights_not_normalised(z, x, s):
    L = _ORIG["berrut_weights"](z, x, s)
    z = np.asarray(z, dtype=np.float64)
    x = np.asarray(x, dtype=np.float64)
    for m in range(z.size):
        if not np.any(z[m] == x):
            L[m] = np.asarray(s, dtype=np.float64) / (z[m] - x)
    return L


def _weights_no_unit_row(z, x, s):
    z = np.asarray(z, dtype=np.float64)
    x = np.asarray(x, dtype=np.float64)
    with np.errstate(all="ignore"):
        t = np.asarray(s, dtype=np.float64)[None, :] / (z[:, None] - x[None, :])
        return t / t.sum(axis=1, keepdims=True)


def _weights_squared_distance(z, x, s):
    z = np.asarray(z, dtype=np.float64)
    x = np.asarray(x, dtype=np.float64)
    L = _ORIG["berrut_weights"](z, x, s)
    for m in range(z.size):
        if not np.any(z[m] == x):
            t = np.asarray(s, dtype=np.float64) / (z[m] - x) ** 2
            L[m] = t / t.sum()
    return L


def _signs_all_plus(n):
    return np.ones(n)


def _signs_start_negative_then_pairs(n):
    return np.where((np.arange(n) // 2) % 2 == 0, 1.0, -1.0)      # + + - - instead of + - + -


def _decode_weights_modes_swapped(alpha, beta, F, sign_mode=0):
    return _ORIG["decode_weights"](alpha, beta, F, 1 - sign_mode)


def _decode_ignores_mask(Y, mask, alpha, beta, S, sign_mode=0):
    Y = np.asarray(Y)
    everyone = np.ones_like(np.asarray(mask))
    out, _ = _ORIG["decode"](Y, everyone, alpha, beta, 0, sign_mode)
    _, status = _ORIG["decode"](np.zeros_like(Y), mask, alpha, beta, S, sign_mode)
    out[status != 0] = 0
    return out, status


def _encode_weights_transposed_roles(alpha, beta):
    # basis built on the worker nodes and read at the query nodes, then transposed into shape
    alpha = np.asarray(alpha, dtype=np.float64)
    beta = np.asarray(beta, dtype=np.float64)
    return _ORIG["berrut_weights"](alpha, beta, orc.alternating_signs(beta.size)).T


def _system_plus_y(x, y, K, A):
    Amat, rhs = _ORIG["locator_system"](x, y, K, A)
    M = K + A
    Amat[:, M:] = -Amat[:, M:]
    return Amat, rhs


def _system_q_starts_at_x0(x, y, K, A):
    x = np.asarray(x, dtype=np.float64)
    y = np.asarray(y, dtype=np.float64)
    M = K + A
    V = np.vander(x, M, increasing=True)
    return np.concatenate([V, -y[:, None] * V[:, : M - 1]], axis=1), y.copy()


def _system_p_one_degree_short(x, y, K, A):
    Amat, rhs = _ORIG["locator_system"](x, y, K, A)
    Amat[:, K + A - 1] = 0.0                       # P loses its highest power
    return Amat, rhs


def _values_without_q0(x, y, K, A):
    return _ORIG["locator_values"](x, y, K, A) - 1.0


def _homogeneous_largest_singular_vector(x, y, K, A):
    x = np.asarray(x, dtype=np.float64)
    y = np.asarray(y, dtype=np.float64)
    M = K + A
    V = np.vander(x, M, increasing=True)
    H = np.concatenate([V, -y[:, None] * V], axis=1)
    return V @ np.linalg.svd(H)[2][0][M:]


def _homogeneous_reads_p_half(x, y, K, A):
    x = np.asarray(x, dtype=np.float64)
    y = np.asarray(y, dtype=np.float64)
    M = K + A
    V = np.vander(x, M, increasing=True)
    H = np.concatenate([V, -y[:, None] * V], axis=1)
    return V @ np.linalg.svd(H)[2][-1][:M]


def _homogeneous_q_one_degree_short(x, y, K, A):
    x = np.asarray(x, dtype=np.float64)
    y = np.asarray(y, dtype=np.float64)
    M = K + A
    V = np.vander(x, M, increasing=True)
    H = np.concatenate([V, -y[:, None] * V[:, : M - 1]], axis=1)
    return V[:, : M - 1] @ np.linalg.svd(H)[2][-1][M:]


def _pick_largest(a, avail, A):
    order = np.argsort(-np.abs(a), kind="stable")
    return np.asarray(avail, dtype=np.int64)[order[:A]]


def _pick_positions_not_workers(a, avail, A):
    return np.argsort(np.abs(a), kind="stable")[:A].astype(np.int64)


def _vote_least_frequent(I, W, A):
    counts = np.bincount(np.asarray(I, dtype=np.int64).ravel(), minlength=W)
    order = np.lexsort((np.arange(W), counts))
    return np.sort(order[:A]).astype(np.int32), counts


def _byzantine_keeps_adversaries(Y, mask, alpha, beta, S, A, sign_mode=0):
    Y = np.asarray(Y)
    out, adv, status = _ORIG["decode_byzantine"](Y, mask, alpha, beta, S, A, sign_mode)
    plain, _ = _ORIG["decode"](Y, mask, alpha, beta, S, sign_mode)
    return plain, adv, status


def _wait_for_the_slowest(arrival, wait_for):
    arrival = np.asarray(arrival, dtype=np.float64)
    flipped = np.where(np.isfinite(arrival), -arrival, arrival)
    return _ORIG["wait_mask"](flipped, wait_for)


def _wait_counts_absentees(arrival, wait_for):
    arrival = np.asarray(arrival, dtype=np.float64)
    return _ORIG["wait_mask"](np.nan_to_num(arrival, nan=1e300, posinf=1e300, neginf=-1e300), wait_for)


def _top1_last_on_ties(Y, mask, alpha, beta, S, sign_mode=0):
    out, status = orc.decode(Y, mask, alpha, beta, S, sign_mode)
    C = out.shape[2]
    top1 = (C - 1 - np.argmax(out[:, :, ::-1], axis=2)).astype(np.int32)
    top1[status != 0] = -1
    return top1, np.max(out, axis=2), status


def _reconstruction_inverted(x, y, K, A, z):
    return 1.0 / _ORIG["rational_reconstruction"](x, y, K, A, z)


def _reconstruction_without_q0(x, y, K, A, z):
    # Q read without its constant term
    M = K + A
    Amat, rhs = orc.locator_system(x, y, K, A)
    sol = np.linalg.lstsq(Amat, rhs, rcond=None)[0]
    z = np.asarray(z, dtype=np.float64)
    num = sum(sol[k] * z ** k for k in range(M))
    den = sum(sol[M - 1 + k] * z ** k for k in range(1, M))
    return num / den


def _decode_rational_at_worker_nodes(Y, mask, alpha, beta, S, A):
    # P / Q read at the first K worker nodes instead of the query nodes
    return _ORIG["decode_rational"](Y, mask, np.asarray(beta)[: np.asarray(alpha).size] * 0.999, beta, S, A)


MUTATIONS = {
    "worker nodes divided by the worker count (the paper's N is W-1)": ("chebyshev_nodes", _nodes_paper_n_confused),
    "first and second kind nodes swapped": ("chebyshev_nodes", _nodes_kinds_swapped),
    "query nodes with 2K+1 in the denominator": ("chebyshev_nodes", _nodes_alpha_denominator),
    "basis functions not divided by their sum": ("berrut_weights", _weights_not_normalised),
    "no unit row at a node": ("berrut_weights", _weights_no_unit_row),
    "squared distances in the basis functions": ("berrut_weights", _weights_squared_distance),
    "signs not alternating": ("alternating_signs", _signs_all_plus),
    "signs alternating in pairs": ("alternating_signs", _signs_start_negative_then_pairs),
    "decoder sign modes swapped": ("decode_weights", _decode_weights_modes_swapped),
    "decoder ignores the mask": ("decode", _decode_ignores_mask),
    "encoder basis built on the worker nodes": ("encode_weights", _encode_weights_transposed_roles),
    "locator system with +y": ("locator_system", _system_plus_y),
    "locator Q starting at x^0": ("locator_system", _system_q_starts_at_x0),
    "locator P one degree short": ("locator_system", _system_p_one_degree_short),
    "locator values without Q_0 = 1": ("locator_values", _values_without_q0),
    "Algorithm 1 with the largest singular vector": ("locator_values_homogeneous", _homogeneous_largest_singular_vector),
    "Algorithm 1 reading Q from the P half": ("locator_values_homogeneous", _homogeneous_reads_p_half),
    "Algorithm 1 with Q one degree short": ("locator_values_homogeneous", _homogeneous_q_one_degree_short),
    "picks the largest |a|": ("pick_smallest", _pick_largest),
    "picks returned as positions, not worker indices": ("pick_smallest", _pick_positions_not_workers),
    "vote keeps the least frequent": ("vote", _vote_least_frequent),
    "Byzantine decoder keeps the located workers": ("decode_byzantine", _byzantine_keeps_adversaries),
    "wait rule keeps the slowest": ("wait_mask", _wait_for_the_slowest),
    "wait rule counts workers that never answer": ("wait_mask", _wait_counts_absentees),
    "top-1 takes the last class on ties": ("decode_top1", _top1_last_on_ties),
    "Algorithm 3 returns Q / P": ("rational_reconstruction", _reconstruction_inverted),
    "Algorithm 3 drops Q_0": ("rational_reconstruction", _reconstruction_without_q0),
    "Algorithm 3 read at the worker nodes": ("decode_rational", _decode_rational_at_worker_nodes),
}
_ORIG = {name: getattr(orc, name) for name, _ in MUTATIONS.values()}


@pytest.mark.parametrize("what", sorted(MUTATIONS))
def test_planted_mistake_is_caught_by_a_pin(what, monkeypatch):
    name, wrong = MUTATIONS[what]
    monkeypatch.setattr(orc, name, wrong)
    failed = run_pins()
    assert failed, "no pin notices: " + what
