"""Seeded synthetic workloads shaped like the image and text serving workloads.

This module only draws inputs: query tensors, survivor masks, the parameters of
the stand-in hosted model f, adversary positions and adversarial noise.  It holds
none of the coding layer's arithmetic (no nodes, no interpolation weights, no
encoding or decoding), so both the GPU library's callers and the CPU oracle's
callers may use it.

Every draw is a pure function of (workload name, stream, group index): any group
can be regenerated alone, which is what lets full-size runs be checked on sampled
groups.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass

import numpy as np

BASE_SEED = 210909868

_STREAM_QUERIES, _STREAM_MASKS, _STREAM_MODEL, _STREAM_ADV, _STREAM_NOISE, _STREAM_PREDS = range(6)


@dataclass(frozen=True)
class Workload:
    name: str
    index: int            # seed offset
    G: int                # groups
    K: int                # queries per group
    W: int                # workers
    S: int                # stragglers
    A: int                # adversarial workers
    query_shape: tuple    # shape of one query; D = prod
    C: int                # prediction length
    query_dist: str       # "uniform01" | "clipped_normal" | "normal"
    model: str            # "linear_softmax" | "mlp" | "iid_logits" | "linear" | "meanpool_linear"

    @property
    def D(self) -> int:
        return int(np.prod(self.query_shape))

    @property
    def n_avail(self) -> int:
        return self.W - self.S


WORKLOADS = {
    "tiny": Workload("tiny", 0, 64, 4, 6, 2, 0, (3, 32, 32), 10, "uniform01", "linear_softmax"),
    "cifar": Workload("cifar", 1, 4096, 8, 12, 4, 0, (3, 32, 32), 100, "uniform01", "mlp"),
    "imagenet": Workload("imagenet", 2, 512, 12, 20, 8, 0, (3, 224, 224), 1000, "clipped_normal", "iid_logits"),
    "byzantine": Workload("byzantine", 3, 2048, 8, 24, 4, 2, (3, 32, 32), 10, "uniform01", "linear"),
    "text": Workload("text", 4, 1024, 16, 24, 6, 0, (128, 768), 2, "normal", "meanpool_linear"),
    # the paper's own operating point (Section 4.2): MNIST-sized queries, K = 8, one straggler, 10 classes
    "mnist_k8": Workload("mnist_k8", 6, 16384, 8, 9, 1, 0, (1, 28, 28), 10, "uniform01", "linear_softmax"),
    "text_k32": Workload("text_k32", 5, 1024, 32, 48, 12, 0, (128, 768), 2, "normal", "meanpool_linear"),
    # the paper's Byzantine operating point (Section 4.2, "Byzantine-Robustness"): K = 12, no stragglers,
    # E = 2 adversaries, N = 2 (K + E) = 28 workers, MNIST-sized queries, 10 classes
    "mnist_byz_k12": Workload("mnist_byz_k12", 7, 8192, 12, 28, 0, 2, (1, 28, 28), 10, "uniform01", "linear"),
}


def scaled(w: Workload, **changes) -> Workload:
    """Same recipe with some sizes replaced (smaller G for CPU-sized tests)."""
    d = dict(w.__dict__)
    d.update(changes)
    return Workload(**d)


def _rng(w: Workload, stream: int, *key) -> np.random.Generator:
    ss = np.random.SeedSequence(entropy=BASE_SEED + w.index, spawn_key=(stream,) + tuple(int(k) for k in key))
    return np.random.Generator(np.random.PCG64(ss))


# ----------------------------------------------------------------------------
# queries
# ----------------------------------------------------------------------------
def query_group(w: Workload, g: int) -> np.ndarray:
    """Queries of group g, float32 [K, D]."""
    rng = _rng(w, _STREAM_QUERIES, g)
    shape = (w.K, w.D)
    if w.query_dist == "uniform01":
        return rng.random(shape, dtype=np.float32)
    if w.query_dist == "normal":
        return rng.standard_normal(shape, dtype=np.float32)
    if w.query_dist == "clipped_normal":
        x = rng.standard_normal(shape, dtype=np.float32)
        x *= np.float32(0.25)
        x += np.float32(0.45)
        np.clip(x, 0.0, 1.0, out=x)
        return x
    raise ValueError(w.query_dist)


def queries(w: Workload, g0: int = 0, g1: int | None = None, out: np.ndarray | None = None, threads: int = 8) -> np.ndarray:
    """Queries of groups g0..g1-1, float32 [g1-g0, K, D]."""
    g1 = w.G if g1 is None else g1
    if out is None:
        out = np.empty((g1 - g0, w.K, w.D), dtype=np.float32)

    def fill(g):
        out[g - g0] = query_group(w, g)

    if g1 - g0 <= 1 or threads <= 1:
        for g in range(g0, g1):
            fill(g)
    else:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(fill, range(g0, g1)))
    return out


# ----------------------------------------------------------------------------
# survivor masks and adversary positions
# ----------------------------------------------------------------------------
def masks(w: Workload, g0: int = 0, g1: int | None = None) -> np.ndarray:
    """uint8 [g1-g0, W]; each row has exactly W-S ones at uniformly drawn positions."""
    g1 = w.G if g1 is None else g1
    m = np.zeros((g1 - g0, w.W), dtype=np.uint8)
    for g in range(g0, g1):
        keep = _rng(w, _STREAM_MASKS, g).permutation(w.W)[: w.W - w.S]
        m[g - g0, keep] = 1
    return m


def adversaries(w: Workload, mask: np.ndarray, g0: int = 0) -> np.ndarray:
    """int32 [G', A] ascending worker indices drawn uniformly among each row's available workers."""
    adv = np.zeros((mask.shape[0], w.A), dtype=np.int32)
    for r in range(mask.shape[0]):
        avail = np.nonzero(mask[r])[0]
        pick = _rng(w, _STREAM_ADV, g0 + r).permutation(avail.size)[: w.A]
        adv[r] = np.sort(avail[pick])
    return adv


# ----------------------------------------------------------------------------
# the stand-in hosted model f
# ----------------------------------------------------------------------------
def model_params(w: Workload) -> dict:
    rng = _rng(w, _STREAM_MODEL)
    D = w.D
    if w.model in ("linear_softmax", "linear"):
        if D == WORKLOADS["tiny"].D:
            # the "byzantine" workload reuses the linear map of the "tiny" workload
            rng = _rng(WORKLOADS["tiny"], _STREAM_MODEL)
        return {"M": rng.standard_normal((D, w.C)) / np.sqrt(D), "b": np.zeros(w.C)}
    if w.model == "mlp":
        H = 512
        return {
            "M1": (rng.standard_normal((D, H)) / np.sqrt(D)).astype(np.float32),
            "b1": (0.1 * rng.standard_normal(H)).astype(np.float32),
            "M2": (rng.standard_normal((H, w.C)) / np.sqrt(H)).astype(np.float32),
            "b2": (0.1 * rng.standard_normal(w.C)).astype(np.float32),
        }
    if w.model == "meanpool_linear":
        E = w.query_shape[1]
        return {"M": rng.standard_normal((E, w.C)) / np.sqrt(E), "b": 0.1 * rng.standard_normal(w.C)}
    if w.model == "iid_logits":
        return {}
    raise ValueError(w.model)


def model_apply(w: Workload, params: dict, x: np.ndarray) -> np.ndarray:
    """f applied to a batch of (coded) queries [..., D]; float32 [..., C]."""
    lead = x.shape[:-1]
    x2 = x.reshape(-1, x.shape[-1])
    if w.model == "linear":
        y = x2.astype(np.float64) @ params["M"] + params["b"]
    elif w.model == "linear_softmax":
        z = x2.astype(np.float64) @ params["M"] + params["b"]
        z -= z.max(axis=1, keepdims=True)
        e = np.exp(z)
        y = e / e.sum(axis=1, keepdims=True)
    elif w.model == "mlp":
        h = np.maximum(x2.astype(np.float32) @ params["M1"] + params["b1"], 0.0)
        y = h @ params["M2"] + params["b2"]
    elif w.model == "meanpool_linear":
        T, E = w.query_shape
        pooled = x2.astype(np.float64).reshape(-1, T, E).mean(axis=1)
        y = pooled @ params["M"] + params["b"]
    else:
        raise ValueError("model %r has no forward pass (its predictions are drawn directly)" % w.model)
    return y.astype(np.float32).reshape(lead + (w.C,))


def iid_logits(w: Workload, g0: int = 0, g1: int | None = None) -> np.ndarray:
    """Coded predictions drawn directly: float32 [g1-g0, W, C], N(0, 3^2)."""
    g1 = w.G if g1 is None else g1
    out = np.empty((g1 - g0, w.W, w.C), dtype=np.float32)
    for g in range(g0, g1):
        out[g - g0] = np.float32(3.0) * _rng(w, _STREAM_PREDS, g).standard_normal((w.W, w.C), dtype=np.float32)
    return out


def corrupt(w: Workload, preds: np.ndarray, adv: np.ndarray, g0: int = 0, sigma_scale: float = 10.0) -> np.ndarray:
    """Adversarial rows = clean row + N(0, (sigma_scale * std)^2), std being the
    population standard deviation of the whole clean tensor (float64); float32 result."""
    std = float(np.std(preds.astype(np.float64)))
    out = preds.copy()
    for r in range(preds.shape[0]):
        noise = _rng(w, _STREAM_NOISE, g0 + r).standard_normal((w.A, w.C))
        for k, i in enumerate(adv[r]):
            out[r, i, :] = (preds[r, i, :].astype(np.float64) + sigma_scale * std * noise[k]).astype(np.float32)
    return out
