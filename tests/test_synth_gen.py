"""The shared input generator (host side): Philox known answers and Gaussian quality."""
import os

import numpy as np
from scipy import stats

from synth import gen

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_philox_known_answers():
    for line in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")):
        if line.startswith("#") or not line.strip():
            continue
        w = [int(v, 16) for v in line.split()]
        out = gen.philox4x32_10(w[0], w[1], w[2], w[3], w[4], w[5])
        assert [int(v) for v in out] == w[6:10]


def test_normal_moments_and_ks():
    z = gen.normal(42, gen.DOMAIN_INIT, 5, np.arange(400000)).astype(np.float64)
    assert z.dtype == np.float64 and np.all(np.isfinite(z))
    assert abs(z.mean()) < 5 / np.sqrt(len(z))
    assert abs(z.var() - 1) < 0.01 and abs((z ** 4).mean() - 3) < 0.06
    assert stats.kstest(z, "norm").pvalue > 1e-3
    pairs = np.corrcoef(z[0::2], z[1::2])[0, 1]
    assert abs(pairs) < 0.01


def test_normal_is_a_pure_function_of_its_coordinates():
    cols = np.array([0, 1, 2, 3, 4, 1023, 25_599_999, 7, 7])
    a = gen.normal(9, gen.DOMAIN_XI, 123456789012, cols, sigma=1e-3)
    full = gen.normal(9, gen.DOMAIN_XI, 123456789012, np.arange(1024), sigma=1e-3)
    assert np.array_equal(a[:6], full[[0, 1, 2, 3, 4, 1023]]) and a[7] == a[8]
    assert not np.array_equal(full, gen.normal(9, gen.DOMAIN_C, 123456789012, np.arange(1024), sigma=1e-3))
    assert not np.array_equal(full, gen.normal(9, gen.DOMAIN_XI, 123456789013, np.arange(1024), sigma=1e-3))
    assert not np.array_equal(full, gen.normal(10, gen.DOMAIN_XI, 123456789012, np.arange(1024), sigma=1e-3))
    assert abs(full.std() / 1e-3 - 1) < 0.1
    shifted = gen.normal(9, gen.DOMAIN_XI, 1, np.arange(64), sigma=2.0, mean=3.0)
    base = gen.normal(9, gen.DOMAIN_XI, 1, np.arange(64))
    assert np.array_equal(shifted, np.float32(3.0) + np.float32(2.0) * base)
