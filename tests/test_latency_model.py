"""Latency model f_DA = a c_DA + h g + b (paper, latency-model section): the oracle fit against things
that are not the oracle, then the product's fit against the oracle; on the GPU, a small profile-and-fit."""
import numpy as np
import pytest

from oracle import latency_fit as oracle_fit
from paper_2603_12831_amd import latency_model as lm


def _samples(seed, n=40):
    rng = np.random.default_rng(seed)
    c = rng.integers(1_000, 900_000, size=n).astype(np.float64)
    g = rng.integers(1, 513, size=n).astype(np.float64)
    return c, g, rng


def test_oracle_recovers_planted_coefficients_exactly():
    c, g, _ = _samples(1)
    a, h, b = 2.0 ** -11, 2.0 ** -6, 0.015625                      # exactly representable: the fit is exact
    t = a * c + h * g + b
    assert oracle_fit.fit(c, g, t) == (a, h, b)


def test_oracle_agrees_with_library_polyfit_on_the_one_variable_reductions():
    """At the optimum, a straight-line fit (library routine) of t - h g against c must return (a, b), and
    of t - a c against g must return (h, b)."""
    c, g, rng = _samples(2)
    t = 6e-7 * c + 0.004 + 1e-3 * rng.standard_normal(c.size)
    a, h, b = oracle_fit.fit(c, g, t)
    pa, pb = np.polyfit(c, t - h * g, 1)
    assert abs(pa - a) < 1e-12 * abs(a) + 1e-18 and abs(pb - b) < 1e-9
    ph, pb2 = np.polyfit(g, t - a * c, 1)
    assert abs(ph - h) < 1e-9 and abs(pb2 - b) < 1e-9


def test_oracle_residual_is_orthogonal_to_the_regressors():
    c, g, rng = _samples(3)
    t = 5e-7 * c + 2e-4 * g + 0.01 + 2e-3 * rng.standard_normal(c.size)
    a, h, b = oracle_fit.fit(c, g, t)
    r = t - (a * c + h * g + b)
    scale = np.abs(t).sum()
    assert abs(r.sum()) < 1e-9 * scale and abs((r * g).sum()) < 1e-9 * scale * g.max()
    assert abs((r * c).sum()) < 1e-9 * scale * c.max()
    with pytest.raises(ValueError):
        oracle_fit.fit(c, 2 * c, t)                                 # collinear regressors


@pytest.mark.parametrize("seed", [4, 5, 6])
def test_product_fit_matches_oracle(seed):
    c, g, rng = _samples(seed, n=60)
    t = 5.5e-7 * c + 1.5e-4 * g + 0.012 + 3e-3 * rng.standard_normal(c.size)
    m = lm.fit(c, g, t)
    a, h, b = oracle_fit.fit(c, g, t)
    assert abs(m["a"] - a) <= 1e-9 * abs(a) and abs(m["h"] - h) <= 1e-7 * abs(h) + 1e-12
    assert abs(m["b"] - b) <= 1e-7 * abs(b) + 1e-10
    pred = lm.predict(m, c, g)
    acc = lm.accuracy(pred, t)
    assert 0.9 < acc["p90"] <= acc["avg"] <= 1.0 and acc["min"] <= acc["p90"]
    with pytest.raises(ValueError):
        lm.fit(c[:2], g[:2], t[:2])
    with pytest.raises(ValueError):
        lm.fit(c, 3 * c, t)


def test_accuracy_definition_and_sampler():
    acc = lm.accuracy([1.0, 2.2, 2.7], [1.0, 2.0, 3.0])
    assert abs(acc["avg"] - (1 + 0.9 + 0.9) / 3) < 1e-12 and abs(acc["min"] - 0.9) < 1e-12
    s1, s2 = lm.sample_batches(0, 5), lm.sample_batches(0, 5)
    assert all(np.array_equal(x, y) for x, y in zip(s1, s2))
    assert all(4 <= len(x) <= 512 and x.min() >= 1 and x.max() <= 8192 and x.sum() <= 600_000 for x in s1)


@pytest.mark.gpu
def test_profile_and_fit_on_gpu():
    """Latencies measured on the GPU: the product's fit of them must be the oracle's fit of the same
    samples, and the model must predict the held-out samples as well as the paper's accuracy table says
    such models do (its averages are 93 % and more)."""
    res = lm.profile_and_fit(n_samples=40, seed=1, reps=5, keep_samples=True)
    print({k: v for k, v in res.items() if k != "samples"})
    c, g, t = (np.array(res["samples"][k]) for k in ("c_da", "g", "ms"))
    n_train = res["train_samples"]
    a, h, b = oracle_fit.fit(c[:n_train], g[:n_train], t[:n_train])
    m = res["model_ms"]
    assert abs(m["a"] - a) <= 1e-9 * abs(a)
    assert abs(m["h"] - h) <= 1e-9 * abs(h) + 1e-15
    assert abs(m["b"] - b) <= 1e-9 * abs(b) + 1e-15
    # accuracy recomputed from the oracle's coefficients, by the table's definition
    held = 1.0 - np.abs(a * c[n_train:] + h * g[n_train:] + b - t[n_train:]) / t[n_train:]
    assert abs(held.mean() - res["accuracy_test"]["avg"]) < 1e-9
    assert held.mean() >= 0.93
    assert a > 0                                                    # more context costs more
    # the per-token slope must correspond to a plausible HBM rate (between 1 and 8 TB/s)
    assert 1000.0 < res["implied_kv_GBps"] < 8000.0
