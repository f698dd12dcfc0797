"""Pins for the oracle's practical event source (Poisson count per gradient step + FIFO pairing)."""
import numpy as np
from scipy import stats

from oracle import core, fifo, graph


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


# ---- the same normalisation read per worker: every worker's clock runs on its own gradient steps --------------

def test_per_worker_clock_speeds_are_the_running_averages_of_the_workers_own_steps():
    n, edges = 6, graph.ring(6)
    rate = np.array([0.4, 1.0, 2.5, 1.0, 0.7, 1.6])
    real = fifo.generate(n, edges, rate, 1.2, 0.02, 0.3, 4, 4000)
    per = fifo.generate(n, edges, rate, 1.2, 0.02, 0.3, 4, 4000, normalize="worker")
    # the events and their real-time stamps do not change; only gradient events carry a speed
    assert np.array_equal(real.t, per.t) and np.array_equal(real.kind, per.kind) and np.array_equal(real.i, per.i)
    assert np.all(per.speed[per.kind == 1] == 0) and np.all(per.speed[per.kind == 0] > 0)
    for w in range(n):
        ends = per.t[(per.kind == 0) & (per.i == w)]
        durations = np.diff(np.concatenate([[0.0], ends]))                 # steps run back to back from time 0
        want = 1.0 / (np.cumsum(durations) / np.arange(1, len(durations) + 1))
        got = per.speed[(per.kind == 0) & (per.i == w)]
        assert np.allclose(got, want, rtol=2e-7)                           # rounded to fp32
        assert np.array_equal(got, got.astype(np.float32).astype(np.float64))
        # on its own clock a worker completes one gradient step per unit of time in the long run: the time that
        # elapses for it during step k is duration_k x (speed before the step's completion)
        before = np.concatenate([[rate[w]], got[:-1]])
        assert abs((durations * before).sum() / len(durations) - 1.0) < 0.02


def test_per_worker_clocks_of_identical_workers_are_the_common_normalised_clock():
    """Identical workers, no jitter: every step of every worker lasts 1 / r, so every worker's own average is the
    global one and the dynamic driven by the per-worker speeds equals the one driven by the normalised stamps."""
    n, edges, r = 8, graph.ring(8), 2.0
    glob = fifo.generate(n, edges, np.full(n, r), 1.5, 0.005, 0.0, 3, 2500, normalize=True)
    per = fifo.generate(n, edges, np.full(n, r), 1.5, 0.005, 0.0, 3, 2500, normalize="worker")
    assert np.array_equal(glob.kind, per.kind) and np.array_equal(glob.i, per.i) and np.array_equal(glob.j, per.j)
    assert np.allclose(per.speed[per.kind == 0], r, rtol=1e-7)
    rng = np.random.default_rng(2)
    x0 = rng.normal(size=(n, 5))
    a = core.State(x0, None, 0.8, 0.5, 1.1).apply(glob, 0.05, 1.0)
    b = core.State(x0, None, 0.8, 0.5, 1.1)
    b.rate[:] = r
    b.apply(per, 0.05, 1.0)
    assert np.allclose(a.x, b.x, rtol=1e-9, atol=1e-12) and np.allclose(a.xt, b.xt, rtol=1e-9, atol=1e-12)


def test_per_worker_clocks_do_not_depend_on_the_unit_of_time():
    n, edges = 10, graph.exponential(10)
    rate = np.array([0.5, 0.8, 1.0, 1.0, 1.2, 2.0, 2.2, 3.0, 0.9, 1.4])
    rng = np.random.default_rng(6)
    x0 = rng.normal(size=(n, 4))
    out = []
    for k in (1.0, 8.0):                                   # k times faster machines, k times shorter exchanges
        ev = fifo.generate(n, edges, k * rate, 1.0, 0.02 / k, 0.3, 9, 3000, normalize="worker")
        st = core.State(x0, None, 0.5, 0.5, 0.9)
        st.rate[:] = k * rate
        st.apply(ev, 0.05, 1.0)
        out.append((ev, st))
    (ea, sa), (eb, sb) = out
    assert np.array_equal(ea.kind, eb.kind) and np.array_equal(ea.i, eb.i) and np.allclose(ea.t, 8.0 * eb.t, rtol=1e-12)
    assert np.allclose(sa.x, sb.x, rtol=1e-5, atol=1e-7)   # the speeds are rounded to fp32 on both sides
