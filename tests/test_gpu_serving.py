"""The closed serving loop (Section 2, "System Architecture"; Section 4.1, "Performance metric") on the GPU against
the same chain run by the oracle on the CPU:

    stream of Q queries (K does not divide Q) -> groups -> encode -> stand-in model f -> drawn response times
      -> wait rule -> (locate and drop the Byzantine workers) -> decode -> top-1

The hosted model is a stand-in (a seeded linear map, with a softmax in the straggler runs): the paper's datasets and
trained networks are not available, so the accuracies printed here are NOT the paper's figures -- parity unpinned
against them.  What is asserted is that the GPU chain and the oracle's chain agree, stage by stage and group by group.
"""
import numpy as np
import pytest

from oracle import approxifer_oracle as orc
from parity_cases import TOL, group_err, lebesgue

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    from paper_2109_09868_amd import binding, serving
    assert torch.cuda.is_available(), "these tests need the MI355X"
    binding.load()
    return torch, binding, serving, torch.device("cuda:0")


def _chain(gpu, K, S, E, Q, softmax, seed, sigma=10.0):
    torch, binding, serving, dev = gpu
    D, C = 784, 10
    N = K + S if E == 0 else 2 * (K + E) + S
    rng = np.random.default_rng(seed)
    stream = rng.uniform(0, 1, (Q, D)).astype(np.float32)
    Mf = (rng.standard_normal((D, C)) * (3.0 / np.sqrt(D))).astype(np.float64)

    def f_host(x):                                          # the stand-in hosted model, float64, answers in float32
        z = np.asarray(x, dtype=np.float64) @ Mf
        if softmax:
            z = np.exp(z - z.max(-1, keepdims=True))
            z /= z.sum(-1, keepdims=True)
        return z.astype(np.float32)

    Md = torch.from_numpy(Mf).to(dev)

    def f_dev(x):
        z = x.double() @ Md
        return (torch.softmax(z, dim=-1) if softmax else z).float()

    G = -(-Q // K)
    arrival_h, arrival_d = serving.exponential_arrivals(G, N, seed + 1, dev, slow_fraction=0.0)
    mask, count = orc.wait_mask(arrival_h, N - S)
    # Byzantine workers: E per group among the workers that answer in time (a liar that straggles never reaches the
    # decoder, and with fewer than E liars the innocent picks are not unique); they add zero-mean Gaussian noise
    # to their answers (Section 4.2, "Byzantine-Robustness")
    bad = (np.stack([np.sort(rng.permutation(np.nonzero(mask[g])[0])[:E]) for g in range(G)]) if E
           else np.zeros((G, 0), np.int64))
    noise = (sigma * rng.standard_normal((G, E, C))).astype(np.float32)
    bad_d, noise_d = torch.from_numpy(bad).to(dev), torch.from_numpy(noise).to(dev)

    def tamper(preds):
        if E:
            preds.scatter_add_(1, bad_d[:, :, None].expand(-1, -1, C), noise_d)

    loop = serving.ServingLoop(K, N, S, E, D, C, Q + 5, dev, sign_mode=1)
    assert loop.load(torch.from_numpy(stream)) == Q
    res = loop.step(Q, f_dev, arrival_d, tamper)
    torch.cuda.synchronize()

    # ---- the same chain on the CPU -------------------------------------------------------------------
    alpha, beta = orc.chebyshev_nodes(K, N)
    groups = orc.group_queries(stream, K)
    coded = orc.encode(groups, alpha, beta)
    preds = f_host(coded)
    for g in range(G):
        preds[g, bad[g]] += noise[g]
    if E:
        out, adv, status = orc.decode_byzantine(preds, mask, alpha, beta, S, E, 1)
    else:
        out, status = orc.decode(preds, mask, alpha, beta, S, 1)
        adv = np.zeros((G, 0), np.int32)
    top1 = out.argmax(-1).reshape(G * K)[:Q]
    truth = f_host(stream).argmax(-1)                       # the model on the uncoded queries

    # ---- stage by stage --------------------------------------------------------------------------------
    assert res["groups"] == G and Q % K != 0
    assert np.array_equal(loop.queries[:G * K].cpu().numpy().reshape(G, K, D), groups)     # grouping, bit for bit
    assert group_err(res["coded"].cpu().numpy(), coded).max() <= TOL
    assert np.array_equal(res["mask"].cpu().numpy(), mask) and np.all(count == N - S)
    assert np.all(res["status"].cpu().numpy() == 0) and np.all(status == 0)
    assert group_err(res["preds"].cpu().numpy(), preds).max() <= 4 * TOL       # f of coded queries that differ by 1e-6
    if E:
        got_adv = res["adv"].cpu().numpy()
        assert np.array_equal(got_adv, adv)                                    # located sets, bit for bit
        assert np.array_equal(got_adv, bad)                                    # and they are the liars
    # decoded values: the two decoders saw predictions that differ by float32 rounding of f's outputs and by the
    # 1e-6 of the coded queries; the group's Lebesgue constant bounds how much of that reaches the output
    got = res["values"].cpu().numpy().astype(np.float64)
    want = out.reshape(G * K, C)[:Q]
    leb = np.empty(G)
    for g in range(G):
        F = np.setdiff1d(np.nonzero(mask[g])[0], adv[g])
        leb[g] = lebesgue(alpha, beta, F, 1)
    assert leb.max() < 30.0                                                    # Berrut's signs: no pole
    err = np.abs(got - want).max(axis=1) / np.abs(want).max()
    assert np.all(err <= 4 * TOL * (1.0 + np.repeat(leb, K)[:Q]))
    # top-1: identical wherever the oracle's two best classes are further apart than that
    srt = np.sort(want, axis=1)
    clear = (srt[:, -1] - srt[:, -2]) > 8 * TOL * (1.0 + np.repeat(leb, K)[:Q]) * np.abs(want).max()
    got_top1 = res["top1"].cpu().numpy()
    assert clear.mean() > 0.98 and np.array_equal(got_top1[clear], top1[clear])
    acc_gpu, acc_cpu = float((got_top1 == truth).mean()), float((top1 == truth).mean())
    print("K=%d S=%d E=%d N=%d Q=%d %s: top-1 agreement with f on the uncoded queries: gpu %.4f, oracle %.4f"
          % (K, S, E, N, Q, "softmax" if softmax else "linear", acc_gpu, acc_cpu), flush=True)
    assert abs(acc_gpu - acc_cpu) <= 0.01
    return acc_gpu


@pytest.mark.parametrize("S", [1, 2, 3])
@pytest.mark.parametrize("K", [8, 12])
def test_serving_loop_with_stragglers(gpu, K, S):
    # Section 4.2, "Straggler-Resilience": K = 8, 12 queries per group, S = 1, 2, 3 stragglers, N = K + S workers
    _chain(gpu, K, S, 0, 1003, True, 100 * K + S)


@pytest.mark.parametrize("E", [1, 2, 3])
def test_serving_loop_with_byzantine_workers(gpu, E):
    # Section 4.2, "Byzantine-Robustness": K = 12, S = 0, E = 1, 2, 3 workers adding Gaussian noise, N = 2 (K + E)
    _chain(gpu, 12, 0, E, 1003, False, 500 + E)


def test_serving_loop_with_stragglers_and_byzantine_workers(gpu):
    _chain(gpu, 8, 2, 2, 517, False, 77)


def test_pad_last_group_and_top1_on_their_own(gpu):
    torch, binding, serving, dev = gpu
    rng = np.random.default_rng(9)
    for Q, K, D in [(1, 4, 7), (7, 3, 5), (8, 4, 3), (1000, 12, 784), (5, 1, 9), (64, 64, 2), (65, 64, 130)]:
        G = binding.approxifer_group_count(Q, K)
        stream = rng.standard_normal((Q, D)).astype(np.float32)
        buf = torch.full((G * K + 3, D), 7.5, dtype=torch.float32, device=dev)
        buf[:Q] = torch.from_numpy(stream).to(dev)
        groups = binding.approxifer_pad_last_group(buf, Q, K)
        assert np.array_equal(groups.cpu().numpy(), orc.group_queries(stream, K))
        assert torch.all(buf[G * K:] == 7.5)                                     # nothing past the last group
    for rows, C in [(1, 1), (5, 3), (1000, 10), (33, 1000), (7, 64), (3, 65), (2, 4099)]:
        v = rng.standard_normal((rows, C)).astype(np.float32)
        v[0, :] = v[0, 0]                                                        # a row of ties: class 0
        if C > 2:
            v[rows - 1, C - 1] = v[rows - 1].max() + 1.0                         # the last class wins
            v[rows - 1, 1] = np.nan
        top1, score = binding.approxifer_top1(torch.from_numpy(v).to(dev))
        ref = np.nanargmax(v, axis=1)
        assert np.array_equal(top1.cpu().numpy(), ref)
        assert np.array_equal(score.cpu().numpy(), np.nanmax(v, axis=1))
    nan_row = torch.full((2, 5), float("nan"), dtype=torch.float32, device=dev)
    top1, _ = binding.approxifer_top1(nan_row)
    assert np.all(top1.cpu().numpy() == 0)
