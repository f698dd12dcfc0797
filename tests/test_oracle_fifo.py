"""Pins for the oracle's practical event source (Poisson count per gradient step + FIFO pairing)."""
import numpy as np
from scipy import stats

from oracle import fifo, graph


def _run(n, topo, rate, rho, comm_time, jitter, seed, m):
    edges = getattr(graph, topo)(n)
    ev = fifo.generate(n, edges, np.broadcast_to(rate, (n,)).astype(float), rho, comm_time, jitter, seed, m)
    return edges, ev


def test_stream_is_ordered_pairs_are_edges_and_no_worker_is_in_two_averagings_at_once():
    n = 16
    edges, ev = _run(n, "exponential", 1.0, 1.0, 0.07, 0.2, 5, 6000)
    assert len(ev) == 6000 and np.all(np.diff(ev.t) >= 0)
    eset = set(edges)
    last_comm = np.full(n, -np.inf)
    for t, k, i, j in zip(ev.t, ev.kind, ev.i, ev.j):
        if k == 1:
            assert (i, j) in eset and i < j
            for w in (i, j):
                assert t >= last_comm[w] + 0.07 - 1e-12      # busy for comm_time after each pairing
                last_comm[w] = t
        else:
            assert j == -1


def test_gradient_steps_follow_the_duration_model():
    n = 4
    rate = np.array([0.5, 1.0, 2.0, 1.0])
    edges, ev = _run(n, "complete", rate, 1.0, 0.0, 0.3, 9, 8000)
    for i in range(n):
        ti = ev.t[(ev.kind == 0) & (ev.i == i)]
        gaps = np.diff(np.concatenate([[0.0], ti])) * rate[i]
        assert gaps.min() >= 0.7 - 1e-12 and gaps.max() <= 1.3 + 1e-12
        assert abs(gaps.mean() - 1.0) < 0.02
        assert stats.kstest((gaps - 0.7) / 0.6, "uniform").pvalue > 1e-3
    # slower workers take fewer steps (the statistic behind the paper's slowest / fastest worker table)
    counts = np.array([((ev.kind == 0) & (ev.i == i)).sum() for i in range(n)])
    assert counts[0] < counts[1] < counts[2]


def test_communication_count_tracks_the_poisson_mean():
    # each gradient step adds Poisson(rho) pending averagings to its worker; an averaging uses up one of each partner
    n, rho = 16, 1.5
    edges, ev = _run(n, "complete", 1.0, rho, 0.0, 0.1, 11, 40000)
    n_grad = int((ev.kind == 0).sum()); n_comm = len(ev) - n_grad
    expect = rho * n_grad / 2
    assert abs(n_comm - expect) < 5 * np.sqrt(rho * n_grad) / 2 + n          # Poisson noise + pending leftovers
    # rho = 0: no communication at all
    _, ev0 = _run(n, "complete", 1.0, 0.0, 0.0, 0.1, 11, 500)
    assert np.all(ev0.kind == 0)


def test_pairing_is_uniform_over_the_edges():
    # appendix "Uniform neighbor selection check": the communication heat-map is flat on all three topologies
    for topo, tol in (("complete", 0.25), ("ring", 0.15), ("exponential", 0.25)):
        n = 16
        edges, ev = _run(n, topo, 1.0, 1.0, 0.02, 0.3, 3, 60000)
        counts = np.bincount(ev.clock[ev.kind == 1] - n, minlength=len(edges)).astype(float)
        assert counts.min() > 0
        assert counts.std() / counts.mean() < tol, (topo, counts.std() / counts.mean())


def test_first_in_first_out():
    # three workers in a line 0 - 1 - 2, worker 1 slow to become available: 0 and 2 queue up, 0 first; when 1 arrives
    # it must be paired with 0 (the older entry), never with 2 first
    edges = [(0, 1), (1, 2)]
    ev = fifo.generate(3, edges, np.array([4.0, 1.0, 3.9]), 50.0, 1e-9, 0.0, 1, 40)
    first = np.nonzero(ev.kind == 1)[0][0]
    assert (ev.i[first], ev.j[first]) == (0, 1)
    assert ev.t[first] == ev.t[(ev.kind == 0) & (ev.i == 1)][0]       # paired the moment worker 1 became available


def test_prefix_and_seed():
    e, a = _run(8, "ring", 1.0, 1.0, 0.05, 0.2, 7, 3000)
    _, b = _run(8, "ring", 1.0, 1.0, 0.05, 0.2, 7, 1000)
    _, c = _run(8, "ring", 1.0, 1.0, 0.05, 0.2, 8, 1000)
    assert np.array_equal(a.t[:1000], b.t) and np.array_equal(a.clock[:1000], b.clock)
    assert not np.array_equal(b.t, c.t)


# ---- normalised clock (a running average of the gradient-step durations normalises time) -----------

def test_normalised_clock_is_a_reparametrisation_with_one_gradient_step_per_unit_time():
    n, edges = 8, graph.ring(8)
    # identical workers, no jitter: every step lasts 1 / r, so normalised time is exactly r x real time and the
    # k-th gradient step of every worker ends at k, whatever r is (the unit-time gradient process of the analysis)
    for r in (0.25, 2.0, 7.0):
        real = fifo.generate(n, edges, np.full(n, r), 1.5, 0.01 / r, 0.0, 3, 3000)
        norm = fifo.generate(n, edges, np.full(n, r), 1.5, 0.01 / r, 0.0, 3, 3000, normalize=True)
        assert np.array_equal(real.kind, norm.kind) and np.array_equal(real.i, norm.i) and np.array_equal(real.j, norm.j)
        assert np.allclose(norm.t, r * real.t, rtol=1e-12, atol=0)
        for w in range(n):
            ends = norm.t[(norm.kind == 0) & (norm.i == w)]
            assert np.allclose(ends, np.arange(1, len(ends) + 1), rtol=1e-9)
    # the stream does not depend on the time unit at all: scaling every rate and comm_time scales real time only
    a = fifo.generate(n, edges, np.full(n, 0.25), 1.5, 0.04, 0.0, 3, 3000, normalize=True)
    b = fifo.generate(n, edges, np.full(n, 2.0), 1.5, 0.005, 0.0, 3, 3000, normalize=True)
    assert np.array_equal(a.kind, b.kind) and np.array_equal(a.i, b.i) and np.allclose(a.t, b.t, rtol=1e-12)


def test_normalised_clock_with_unequal_workers():
    n, edges = 12, graph.exponential(12)
    rate = np.array([0.4, 0.7, 1.0, 1.0, 1.3, 2.0, 2.5, 3.0, 0.9, 1.1, 1.6, 0.5])
    real = fifo.generate(n, edges, rate, 1.0, 0.02, 0.3, 9, 30000)
    norm = fifo.generate(n, edges, rate, 1.0, 0.02, 0.3, 9, 30000, normalize=True)
    # only the stamps change: same events in the same order, stamps non-decreasing, equal real times stay equal
    assert np.array_equal(real.kind, norm.kind) and np.array_equal(real.i, norm.i) and np.array_equal(real.j, norm.j)
    assert np.all(np.diff(norm.t) >= 0)
    assert np.array_equal(np.diff(real.t) == 0, np.diff(norm.t) == 0)
    # in normalised time the workers together complete one gradient step per worker and unit time
    grads = (norm.kind == 0).sum()
    assert abs(grads / (n * norm.t[-1]) - 1.0) < 0.01
    # before the first completion the unit is the mean nominal duration; afterwards the running average: recompute
    # the first few stamps by hand from the real stream
    unit = np.mean(1.0 / rate)
    done, t_norm, last = [], 0.0, 0.0
    step_start = np.zeros(n)
    for k in range(200):
        t_norm += (real.t[k] - last) / unit
        last = real.t[k]
        assert np.isclose(norm.t[k], t_norm, rtol=1e-12)
        if real.kind[k] == 0:
            done.append(real.t[k] - step_start[real.i[k]])
            step_start[real.i[k]] = real.t[k]
            # averaging ends between events move the clock too but never change the unit, so applying the new unit
            # from this event on is the same thing
            unit = np.mean(done)
