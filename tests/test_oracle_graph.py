"""Pins for Definition 3.1, chi_1, chi_2 and the hyper-parameter rule of Proposition 3.2."""
import os

import numpy as np
import pytest

from oracle import graph

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
BUILDERS = {"complete": graph.complete, "exponential": graph.exponential, "ring": graph.ring}


def test_paper_printed_values_n16():
    for line in open(os.path.join(GOLDEN, "fig6_chi.txt")):
        if line.startswith("#") or not line.strip():
            continue
        name, c1, c2 = line.split()
        edges = BUILDERS[name](16)
        lam = graph.laplacian(16, edges, graph.per_worker_to_edge_rate(16, edges, 1.0))
        assert round(graph.chi1(lam)) == int(c1), name
        assert round(graph.chi2(lam, edges)) == int(c2), name


def test_edge_counts():
    assert len(graph.complete(64)) == 2016
    assert len(graph.ring(64)) == 64
    assert len(graph.exponential(64)) == 352      # degree 11: offsets 1..16 twice, offset 32 once
    assert len(graph.exponential(16)) == 56       # degree 7


@pytest.mark.parametrize("n,rate", [(4, 1.0), (16, 0.3), (64, 2.0)])
def test_complete_graph_closed_form(n, rate):
    # Lambda = rate (n I - 1 1^T): non-zero eigenvalues rate*n; resistance between any two nodes 2/(rate n)
    edges = graph.complete(n)
    lam = graph.laplacian(n, edges, rate)
    assert np.allclose(lam, rate * (n * np.eye(n) - np.ones((n, n))))
    assert np.isclose(graph.chi1(lam), 1 / (rate * n))
    assert np.isclose(graph.chi2(lam, edges), 1 / (rate * n))


@pytest.mark.parametrize("n,rate", [(5, 1.0), (16, 1.0), (64, 2.0)])
def test_ring_closed_forms(n, rate):
    # circulant spectrum rate*(2 - 2cos(2 pi k/n)); adjacent nodes of a ring of n resistors of 1/rate ohm:
    # one resistor in parallel with n-1 in series = (n-1)/(n rate)
    edges = graph.ring(n)
    lam = graph.laplacian(n, edges, rate)
    assert np.isclose(graph.chi1(lam), 1 / (rate * (2 - 2 * np.cos(2 * np.pi / n))))
    assert np.isclose(graph.chi2(lam, edges), 0.5 * (n - 1) / (n * rate))


def test_exponential_graph_circulant_closed_form():
    n, rate = 64, 1.0
    edges = graph.exponential(n)
    lam = graph.laplacian(n, edges, rate)
    offs = [1, 2, 4, 8, 16, 32]
    k = np.arange(1, n)
    # a node has two neighbours at offset o (i+o and i-o) except at o = n/2, where they coincide:
    # eigenvalue contribution rate*(2 - 2cos(2 pi k o/n)), halved for o = n/2
    eig = sum(rate * (2 - 2 * np.cos(2 * np.pi * k * o / n)) * (0.5 if 2 * o == n else 1.0) for o in offs)
    assert np.isclose(graph.chi1(lam), 1 / eig.min())
    # effective resistance between nodes o apart: (1/n) sum_{k != 0} (2 - 2cos(2 pi k o/n)) / eig_k
    res = max(np.sum((2 - 2 * np.cos(2 * np.pi * k * o / n)) / eig) / n for o in offs)
    assert np.isclose(graph.chi2(lam, edges), 0.5 * res)


def test_chi2_le_chi1_random_connected_graphs():
    rng = np.random.default_rng(0)
    for _ in range(30):
        n = int(rng.integers(3, 12))
        edges = set(graph.ring(n))          # connected backbone
        for _ in range(int(rng.integers(0, n * 2))):
            i, j = rng.integers(0, n, 2)
            if i != j:
                edges.add((min(i, j), max(i, j)))
        edges = sorted(edges)
        rates = rng.uniform(0.1, 3.0, len(edges))
        lam = graph.laplacian(n, edges, rates)
        assert graph.chi2(lam, edges) <= graph.chi1(lam) * (1 + 1e-12)


def test_hyper_parameter_rule():
    p = graph.acid_params(4, graph.complete(4), 1.0)
    assert np.isclose(p["chi1"], 0.25) and np.isclose(p["chi2"], 0.25)
    assert np.isclose(p["eta"], 2.0) and np.isclose(p["alpha_tilde"], 0.5) and p["alpha"] == 0.5
    p = graph.acid_params(16, graph.ring(16), 1.0)
    assert np.isclose(p["eta"], 1 / (2 * np.sqrt(p["chi1"] * p["chi2"])))
    assert np.isclose(p["alpha_tilde"], 0.5 * np.sqrt(p["chi1"] / p["chi2"]))
    assert np.isclose(p["chi1"], 6.568536, atol=1e-6) and np.isclose(p["chi2"], 0.46875)
    b = graph.baseline_params()
    assert b == {"eta": 0.0, "alpha": 0.5, "alpha_tilde": 0.5}
