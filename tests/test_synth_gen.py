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


def test_c_implementation_is_bit_identical_to_numpy():
    rng = np.random.default_rng(0)
    cols = np.unique(np.concatenate([np.arange(40), rng.integers(0, 25_600_000, 3000)]))
    rows = [0, 1, 63, 999_999, (1 << 33) + 5]
    for domain, sigma, mean in [(gen.DOMAIN_INIT, 1.0, 0.0), (gen.DOMAIN_XI, 1e-3, 0.0), (gen.DOMAIN_C, 2.0, -0.5)]:
        a = gen.normal_rows(0xA2C1D2 + (3 << 32), domain, rows, cols, sigma, mean)
        b = gen.normal_rows_fast(0xA2C1D2 + (3 << 32), domain, rows, cols, sigma, mean)
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
    big = gen.normal_rows_fast(1, gen.DOMAIN_INIT, [0], np.arange(2_000_000))[0]
    assert np.array_equal(big[:5000], gen.normal(1, gen.DOMAIN_INIT, 0, np.arange(5000)))
    assert abs(big.astype(np.float64).std() - 1) < 0.005
