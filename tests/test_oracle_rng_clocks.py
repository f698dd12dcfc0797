"""Pins for the oracle's random streams and Poisson-clock event source (Assumption 3.1)."""
import os

import numpy as np
from scipy import stats

from oracle import core, graph

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_philox_known_answers():
    for line in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")):
        if line.startswith("#") or not line.strip():
            continue
        w = [int(v, 16) for v in line.split()]
        assert list(core.philox4x32_10(w[0:4], w[4:6])) == w[6:10]


def _stream(n, edges, node_rate, edge_rate, seed, m):
    eu = [e[0] for e in edges]; ev = [e[1] for e in edges]
    return core.generate_events(n, eu, ev, node_rate, edge_rate, seed, m)


def test_stream_is_time_ordered_and_well_formed():
    n = 8
    edges = graph.ring(n)
    ev = _stream(n, edges, np.ones(n), np.full(len(edges), 2.0), 11, 5000)
    assert len(ev) == 5000
    assert np.all(np.diff(ev.t) >= 0) and ev.t[0] > 0
    g = ev.kind == 0
    assert np.all(ev.j[g] == -1) and np.all(ev.clock[g] == ev.i[g])
    eidx = ev.clock[~g] - n
    assert np.all(np.array(edges)[eidx, 0] == ev.i[~g]) and np.all(np.array(edges)[eidx, 1] == ev.j[~g])


def test_event_counts_match_rates():
    # Proposition 3.2: n T gradient events and Tr(Lambda)/2 * T communications in expectation.
    n = 16
    edges = graph.exponential(n)
    lam = 0.7
    ev = _stream(n, edges, np.ones(n), np.full(len(edges), lam), 5, 200000)
    T = ev.t[-1]
    n_grad = int((ev.kind == 0).sum()); n_comm = len(ev) - n_grad
    tr_half = np.trace(graph.laplacian(n, edges, lam)) / 2
    assert abs(n_grad - n * T) < 5 * np.sqrt(n * T)
    assert abs(n_comm - tr_half * T) < 5 * np.sqrt(tr_half * T)


def test_interarrivals_are_exponential_with_the_clock_rate():
    n = 3
    edges = graph.complete(n)
    node_rate = np.array([0.5, 1.0, 3.0]); edge_rate = np.array([2.0, 0.25, 1.0])
    ev = _stream(n, edges, node_rate, edge_rate, 1234, 120000)
    rates = np.concatenate([node_rate, edge_rate])
    for c, r in enumerate(rates):
        tc = ev.t[ev.clock == c]
        gaps = np.diff(np.concatenate([[0.0], tc]))
        assert len(gaps) > 1000
        p = stats.kstest(gaps, "expon", args=(0, 1.0 / r)).pvalue
        assert p > 1e-3, (c, p)
        assert abs(gaps.mean() * r - 1) < 5 / np.sqrt(len(gaps))


def test_clocks_are_independent_streams():
    # removing one clock must not change the arrival times of the others
    n = 4
    edges = graph.ring(n)
    a = _stream(n, edges, np.ones(n), np.ones(len(edges)), 9, 4000)
    rate2 = np.ones(len(edges)); rate2[2] = 0.0
    b = _stream(n, edges, np.ones(n), rate2, 9, 4000)
    assert not np.any(b.clock == n + 2)
    for c in range(n + len(edges)):
        if c == n + 2:
            continue
        ta, tb = a.t[a.clock == c], b.t[b.clock == c]
        m = min(len(ta), len(tb))
        assert m > 50 and np.array_equal(ta[:m], tb[:m])


def test_uniform_pairing_histogram_is_flat():
    # appendix "Uniform neighbor selection check": equal edge rates -> flat communication heat-map
    n = 16
    edges = graph.ring(n)
    ev = _stream(n, edges, np.zeros(n), np.ones(len(edges)), 3, 160000)
    assert np.all(ev.kind == 1)
    counts = np.bincount(ev.clock - n, minlength=len(edges))
    assert stats.chisquare(counts).pvalue > 1e-3


def test_seed_changes_stream_and_same_seed_repeats():
    n = 4
    edges = graph.complete(n)
    a = _stream(n, edges, np.ones(n), np.ones(len(edges)), 1, 500)
    b = _stream(n, edges, np.ones(n), np.ones(len(edges)), 1, 500)
    c = _stream(n, edges, np.ones(n), np.ones(len(edges)), 2, 500)
    d = _stream(n, edges, np.ones(n), np.ones(len(edges)), 1 + (1 << 32), 500)
    assert np.array_equal(a.t, b.t) and np.array_equal(a.clock, b.clock)
    assert not np.array_equal(a.t, c.t) and not np.array_equal(a.t, d.t)
    # a prefix of a longer stream is the shorter stream
    e = _stream(n, edges, np.ones(n), np.ones(len(edges)), 1, 200)
    assert np.array_equal(a.t[:200], e.t) and np.array_equal(a.clock[:200], e.clock)
