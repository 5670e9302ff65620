"""The seeded input generators: shapes, value ranges, reproducibility (no GPU)."""
import numpy as np

from paper_2109_09868_amd import synthetic as syn


def test_workload_table_matches_counting_rules():
    # Section 3, "ApproxIFER Encoding": W = K + S without adversaries, W = 2(K + A) + S with them
    for name in ("tiny", "cifar", "imagenet"):
        w = syn.WORKLOADS[name]
        assert w.A == 0 and w.W == w.K + w.S
    b = syn.WORKLOADS["byzantine"]
    assert b.W == 2 * (b.K + b.A) + b.S
    assert syn.WORKLOADS["imagenet"].D == 150528 and syn.WORKLOADS["text"].D == 98304


def test_queries_reproducible_per_group_and_in_range():
    w = syn.scaled(syn.WORKLOADS["tiny"], G=5)
    X = syn.queries(w)
    assert X.shape == (5, 4, 3072) and X.dtype == np.float32
    assert X.min() >= 0 and X.max() < 1
    assert np.array_equal(X[3], syn.query_group(w, 3))
    assert np.array_equal(syn.queries(w, 2, 4), X[2:4])
    wi = syn.scaled(syn.WORKLOADS["imagenet"], G=1, query_shape=(3, 16, 16))
    Xi = syn.queries(wi)
    assert Xi.min() >= 0 and Xi.max() <= 1 and abs(Xi.mean() - 0.45) < 0.02


def test_masks_and_adversaries():
    w = syn.scaled(syn.WORKLOADS["byzantine"], G=50)
    m = syn.masks(w)
    assert m.shape == (50, 24) and m.dtype == np.uint8
    assert np.all(m.sum(axis=1) == 20)
    assert len({tuple(r) for r in m}) > 40           # masks differ between groups
    adv = syn.adversaries(w, m)
    assert adv.shape == (50, 2) and np.all(adv[:, 0] < adv[:, 1])
    assert all(m[g, adv[g]].all() for g in range(50))
    assert np.array_equal(syn.masks(w, 10, 12), m[10:12])


def test_models_and_corruption():
    w = syn.scaled(syn.WORKLOADS["tiny"], G=2)
    p = syn.model_params(w)
    y = syn.model_apply(w, p, syn.queries(w))
    assert y.shape == (2, 4, 10) and y.dtype == np.float32 and np.allclose(y.sum(-1), 1, atol=1e-6)
    wb = syn.scaled(syn.WORKLOADS["byzantine"], G=2)
    assert np.array_equal(syn.model_params(wb)["M"], p["M"])          # same linear map
    clean = syn.model_apply(wb, syn.model_params(wb), np.ones((2, wb.W, wb.D), np.float32))
    m = syn.masks(wb)
    adv = syn.adversaries(wb, m)
    bad = syn.corrupt(wb, clean + np.arange(wb.W, dtype=np.float32)[None, :, None], adv)
    diff = bad - (clean + np.arange(wb.W, dtype=np.float32)[None, :, None])
    for g in range(2):
        rows = np.nonzero(np.abs(diff[g]).sum(-1))[0]
        assert list(rows) == list(adv[g])
    wt = syn.scaled(syn.WORKLOADS["text"], G=1, query_shape=(4, 8))
    yt = syn.model_apply(wt, syn.model_params(wt), syn.queries(wt))
    assert yt.shape == (1, 16, 2)
    z = syn.iid_logits(syn.scaled(syn.WORKLOADS["imagenet"], G=3))
    assert z.shape == (3, 20, 1000) and abs(z.std() - 3) < 0.1
