"""Pins of the oracle's tensor-moments function (population moments about the mean; Results section, first
paragraph): a library routine (scipy.stats), closed forms, and the two distribution families the paper reports."""
import numpy as np
import scipy.stats as st

from oracle import oracle as O


def summary(out):
    d = dict(zip(O.MOMENT_FIELDS, out))
    d["var"] = d["m2"]; d["skew"] = d["m3"] / d["m2"] ** 1.5; d["kurt"] = d["m4"] / d["m2"] ** 2
    return d


def test_against_scipy_on_random_data():
    rng = np.random.default_rng(7)
    for x in (rng.normal(0.3, 2.0, 100001), rng.lognormal(-8, 2, 50000) * rng.choice([-1, 1], 50000), rng.standard_t(4, 77777)):
        x = x.astype(np.float32)
        d = summary(O.moments(x))
        x64 = x.astype(np.float64)
        assert d["n"] == x.size and d["nan_cnt"] == 0
        assert np.isclose(d["mean"], x64.mean(), rtol=1e-12, atol=1e-300)
        assert np.isclose(d["var"], st.moment(x64, 2), rtol=1e-12)
        assert np.isclose(d["m3"], st.moment(x64, 3), rtol=1e-10, atol=1e-14 * d["m2"] ** 1.5)
        assert np.isclose(d["m4"], st.moment(x64, 4), rtol=1e-12)
        assert np.isclose(d["skew"], st.skew(x64), rtol=1e-9, atol=1e-12)
        assert np.isclose(d["kurt"], st.kurtosis(x64, fisher=False), rtol=1e-12)
        assert d["absmax"] == np.abs(x64).max()


def test_closed_forms():
    # 0, 1, ..., n-1: mean (n-1)/2, variance (n^2-1)/12, skew 0, kurtosis 3 (3 n^2 - 7) / (5 (n^2 - 1))
    n = 1000
    d = summary(O.moments(np.arange(n, dtype=np.float32)))
    assert np.isclose(d["mean"], (n - 1) / 2, rtol=1e-15) and np.isclose(d["var"], (n * n - 1) / 12, rtol=1e-14)
    assert abs(d["skew"]) < 1e-12 and np.isclose(d["kurt"], 3 * (3 * n * n - 7) / (5 * (n * n - 1)), rtol=1e-13)
    # two-point distribution: p of value 1, 1-p of value 0: skew (1-2p)/sqrt(p(1-p)), kurtosis 1/(p(1-p)) - 3
    x = np.zeros(1000, np.float32); x[:200] = 1.0
    p = 0.2
    d = summary(O.moments(x))
    assert np.isclose(d["mean"], p) and np.isclose(d["var"], p * (1 - p))
    assert np.isclose(d["skew"], (1 - 2 * p) / np.sqrt(p * (1 - p))) and np.isclose(d["kurt"], 1 / (p * (1 - p)) - 3)
    # a constant offset changes the mean only; a scale s multiplies m_k by s^k
    rng = np.random.default_rng(3)
    y = (np.round(rng.normal(size=4096) * 256) / 256).astype(np.float32)             # few bits: 4 y + 16 is exact
    a, b = O.moments(y), O.moments((y.astype(np.float64) * 4.0 + 16.0).astype(np.float32))    # exact in binary32
    assert np.isclose(b[1], 4 * a[1] + 16, rtol=1e-12) and np.allclose(b[2:5], a[2:5] * [16.0, 64.0, 256.0], rtol=1e-10)


def test_distribution_families_of_the_paper():
    """Weights close to normal (skew 0, kurtosis 3); log-normal magnitudes with a random sign: symmetric, heavy
    tails (kurtosis far above 3)."""
    rng = np.random.default_rng(11)
    d = summary(O.moments(rng.normal(0, 0.02, 1 << 20).astype(np.float32)))
    assert abs(d["skew"]) < 0.01 and abs(d["kurt"] - 3) < 0.02 and np.isclose(d["var"], 4e-4, rtol=5e-3)
    g = (np.exp(rng.normal(-8, 0.8, 1 << 20)) * rng.choice([-1.0, 1.0], 1 << 20)).astype(np.float32)
    d = summary(O.moments(g))
    # E x^2 = exp(2 mu + 2 s^2), E x^4 = exp(4 mu + 8 s^2): kurtosis exp(4 s^2) = 12.9 for s = 0.8
    assert abs(d["skew"]) < 0.2 and 10 < d["kurt"] < 16 and np.isclose(d["var"], np.exp(-16 + 2 * 0.64), rtol=0.02)


def test_nan_and_empty_and_degenerate():
    x = np.array([1.0, np.nan, 3.0, np.nan, -5.0], np.float32)
    out = O.moments(x)
    assert out[0] == 3 and out[6] == 2 and np.isclose(out[1], -1.0 / 3) and out[5] == 5.0
    assert np.all(O.moments(np.zeros(0, np.float32)) == 0)
    c = O.moments(np.full(100, 2.5, np.float32))
    assert c[1] == 2.5 and c[2] == 0 and c[3] == 0 and c[4] == 0
