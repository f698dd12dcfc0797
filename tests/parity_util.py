"""CPU side of the GPU parity tests: runs the oracle on a column subset of a workload and holds the comparisons.

Every step of the method is element-wise in the coordinate index (Eq. (1) couples workers, never
coordinates), so following a subset of columns through the whole event stream is exact.
Inputs come from the shared generator (synth.gen); events from the oracle's own clock code.
"""
import math
from concurrent.futures import ThreadPoolExecutor

import numpy as np

from oracle import core, graph
from synth import gen
from synth import configs as wl          # configurations and clock rates: shared inputs, no product code

TOL = 1e-5     # spec tolerance: max relative error, fp32, norm-wise per worker and buffer


def sample_columns(d, count, seed=0):
    """First and last 1024 columns (tile edges, ragged tail) plus seeded random ones."""
    head = np.arange(min(d, 1024))
    tail = np.arange(max(0, d - 1024), d)
    rng = np.random.default_rng(seed)
    mid = rng.integers(0, d, size=max(0, count - len(head) - len(tail)))
    return np.unique(np.concatenate([head, tail, mid]))


def oracle_params(cfg, fifo=None):
    edges = getattr(graph, cfg.topology)(cfg.n)
    node_rate, edge_rate = wl.clock_rates(cfg)
    if fifo is not None:
        steps_per_unit_time = 1.0 if fifo.get("normalize") else float(node_rate.mean())
        edge_rate = graph.per_worker_to_edge_rate(cfg.n, edges, fifo["comm_per_grad"] * steps_per_unit_time)
    if cfg.accelerated:
        p = graph.acid_params(cfg.n, edges, edge_rate)
        eta, alpha_t = p["eta"], p["alpha_tilde"]
    else:
        eta, alpha_t = 0.0, 0.5
    if cfg.eta is not None:
        eta = cfg.eta
    if cfg.alpha_tilde is not None:
        alpha_t = cfg.alpha_tilde
    return edges, node_rate, edge_rate, eta, 0.5, alpha_t


class OracleStream:
    """The oracle following columns `cols` of a workload, fed with the serial stream chunk by chunk."""

    def __init__(self, cfg, cols, order=0, fifo=None):
        self.cfg, self.cols, self.fifo = cfg, np.asarray(cols, np.int64), fifo
        edges, node_rate, edge_rate, eta, alpha, alpha_t = oracle_params(cfg, fifo)
        self.edges, self.node_rate, self.edge_rate = edges, node_rate, edge_rate
        x0 = gen.normal_rows_fast(cfg.seed, gen.DOMAIN_INIT, np.arange(cfg.n), self.cols, cfg.init_sigma)
        self.state = core.State(x0, None, eta, alpha, alpha_t, order=order)
        self.c = gen.normal_rows_fast(cfg.seed, gen.DOMAIN_C, np.arange(cfg.n), self.cols, 1.0) if cfg.use_c else None
        self.h = gen.curvature(gen.normal_rows_fast(cfg.seed, gen.DOMAIN_H, np.arange(cfg.n), self.cols, 1.0)) \
            if cfg.curvature else None
        self.events = None
        self.done = 0
        if fifo is not None and fifo.get("normalize") == "worker":
            self.state.rate[:] = node_rate                  # the workers' own clocks start at their nominal step rates

    def generate(self, n_events):
        """The first n_events events of the stream (the oracle's own clock code, from time 0)."""
        if self.fifo is not None:
            from oracle import fifo as fifo_source
            self.events = fifo_source.generate(self.cfg.n, self.edges, self.node_rate, self.fifo["comm_per_grad"],
                                               self.fifo["comm_time"], self.fifo["jitter"], self.cfg.seed, n_events,
                                               normalize=self.fifo.get("normalize", False))
            return self.events
        self.events = core.generate_events(self.cfg.n, [e[0] for e in self.edges], [e[1] for e in self.edges],
                                           self.node_rate, np.full(len(self.edges), self.edge_rate), self.cfg.seed,
                                           n_events)
        return self.events

    def advance(self, upto):
        """Applies events [done, upto) of the generated stream."""
        cfg, ev = self.cfg, self.events[self.done:upto]
        is_grad = ev.kind == 0
        m = len(ev)
        c_row = xi = xi_row = h_row = None
        if self.c is not None:
            c_row = np.where(is_grad, ev.i, -1)
        if self.h is not None:
            h_row = np.where(is_grad, ev.i, -1)
        if cfg.xi_sigma > 0:
            ids = np.nonzero(is_grad)[0]
            xi = gen.normal_rows_fast(cfg.seed, gen.DOMAIN_XI, ids + self.done, self.cols, cfg.xi_sigma)
            xi_row = np.full(m, -1, np.int64)
            xi_row[ids] = np.arange(len(ids))
        # the engine receives gamma and gscale as fp32 values
        self.state.apply(ev, float(np.float32(cfg.gamma)), float(np.float32(cfg.gscale)), xi, xi_row, self.c, c_row,
                         self.h, h_row)
        self.done = upto
        return self.state


class SlicedOracle:
    """OracleStream over several slices of the sampled columns, advanced by one thread per slice.  Coordinates never
    interact, so the slices are independent runs of the same serial event loop on the same events; the threads only
    shorten the wait (the C loop and numpy release the interpreter lock)."""

    def __init__(self, cfg, cols, threads=4, order=0, fifo=None):
        self.cols = np.asarray(cols, np.int64)
        self.parts = [OracleStream(cfg, p, order, fifo) for p in np.array_split(self.cols, threads)]
        self.pool = ThreadPoolExecutor(len(self.parts))
        self.events = None
        self.pending = None

    def generate(self, n_events):
        self.events = self.parts[0].generate(n_events)
        for o in self.parts[1:]:
            o.events = self.events
        return self.events

    def start(self, upto):
        """Begins applying events [done, upto) in the background; wait() returns when they are applied."""
        assert self.pending is None
        self.pending = [self.pool.submit(o.advance, upto) for o in self.parts]

    def wait(self):
        for f in self.pending:
            f.result()
        self.pending = None
        return self

    @property
    def t(self):
        return self.parts[0].state.t

    @property
    def rate(self):
        return self.parts[0].state.rate

    def rows(self):
        """(x, xt) on all sampled columns, as stored (each worker at its own time stamp)."""
        return (np.concatenate([o.state.x for o in self.parts], axis=1),
                np.concatenate([o.state.xt for o in self.parts], axis=1))

    def flushed(self, t_now):
        both = [o.state.flushed(t_now) for o in self.parts]
        return np.concatenate([b[0] for b in both], axis=1), np.concatenate([b[1] for b in both], axis=1)

    def close(self):
        self.pool.shutdown()


def oracle_run(cfg, cols, n_events, chunk=20000, order=0, fifo=None):
    """Oracle state after the first n_events events of cfg, restricted to columns cols."""
    o = OracleStream(cfg, cols, order, fifo)
    ev = o.generate(n_events)
    for lo in range(0, len(ev), chunk):
        o.advance(min(len(ev), lo + chunk))
    return o.state, ev


def rel_err(got, want):
    """Norm-wise relative error per row: max_k |got - want| / max_k |want|; returns the max over rows."""
    got = np.asarray(got, np.float64); want = np.asarray(want, np.float64)
    num = np.abs(got - want).max(axis=1)
    den = np.maximum(np.abs(want).max(axis=1), 1e-30)
    return float((num / den).max())


def consensus_of_rows(rows):
    """||pi v||_F^2 = sum_i ||v_i - vbar||^2 of an (n, k) array, in fp64 (appendix "Notations")."""
    rows = np.asarray(rows, np.float64)
    return float(((rows - rows.mean(axis=0, keepdims=True)) ** 2).sum())


def consensus_slack(consensus_ref, delta):
    """How far a state error delta can move the consensus distance: pi is an orthogonal projection, hence
    | ||pi (v + delta)||^2 - ||pi v||^2 | <= 2 ||pi v|| ||delta||_F + ||delta||_F^2."""
    nd = float(np.linalg.norm(np.asarray(delta, np.float64)))
    return 2.0 * math.sqrt(max(consensus_ref, 0.0)) * nd + nd * nd


def assert_consensus(got, ref, rows_got, rows_ref, what=""):
    """got: a consensus distance that belongs to the state rows_got; ref: the oracle's, of rows_ref (same shape).
    Always: the two differ by no more than the measured state error allows (consensus_slack; 1e-9 relative on top
    for the reductions themselves).  And where the workers are not close to consensus (||pi v||^2 >= 1 % of ||v||^2,
    so that the observable is as well conditioned as the state) also the benchmark spec's tolerance TOL, relative."""
    rows_ref = np.asarray(rows_ref, np.float64)
    slack = consensus_slack(ref, np.asarray(rows_got, np.float64) - rows_ref) + 1e-9 * abs(ref)
    assert abs(got - ref) <= slack, (what, got, ref, slack)
    if ref >= 1e-2 * float((rows_ref ** 2).sum()):
        assert abs(got - ref) <= TOL * ref, (what, got, ref)


def check_observables(w, st, t_now, cols):
    """a2cid_stats at t_now, then a2cid_flush to t_now, against the oracle.  Leaves the state flushed.

    The flush and the observables kernel apply the same fp32 mixing to the same stored values, so the library's own
    flushed rows are exactly the state the observables describe: plain numpy reductions of those rows check the
    kernel's reductions alone (fp64 accumulation: 1e-9; per-worker sums go through fp32 partial sums of 512
    values, at most 9 roundings of 2^-24 each: 1e-6 of the row's L1 norm).  Against the oracle the observables may
    differ by what the measured state error allows (parity_util.assert_consensus), and by no more than TOL where
    the observable is as well conditioned as the state."""
    cfg = w.cfg
    gs = w.engine.stats(t_now)
    w.engine.flush(t_now)
    fx, fxt = w.columns(cols)
    ox, oxt = st.flushed(t_now)
    assert rel_err(fx, ox) <= TOL and rel_err(fxt, oxt) <= TOL
    assert np.all(w.engine.times() == t_now)
    if len(cols) != cfg.d:
        # a column sample: the same comparison in the observable's metric, both sides reduced by numpy
        assert_consensus(consensus_of_rows(fx), consensus_of_rows(ox), fx, ox, "x, sampled columns")
        assert_consensus(consensus_of_rows(fxt), consensus_of_rows(oxt), fxt, oxt, "xt, sampled columns")
        return gs
    os_ = st.stats(t_now)
    for name, g_rows, o_rows in (("x", fx, ox), ("xt", fxt, oxt)):
        own = consensus_of_rows(g_rows)
        assert math.isclose(gs["consensus_" + name], own, rel_tol=1e-9, abs_tol=1e-300), (name, gs["consensus_" + name], own)
        l1 = np.abs(g_rows.astype(np.float64)).sum(1)
        assert np.all(np.abs(gs["sum_" + name] - g_rows.astype(np.float64).sum(1)) <= 1e-6 * l1)
        assert_consensus(gs["consensus_" + name], os_["consensus_" + name], g_rows, o_rows, name)
        assert np.all(np.abs(gs["sum_" + name] - os_["sum_" + name]) <= TOL * np.abs(o_rows).sum(1))
    return gs
