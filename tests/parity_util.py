"""CPU side of the GPU parity tests: runs the oracle on a column subset of a workload.

Every step of the method is element-wise in the coordinate index (Eq. (1) couples workers, never
coordinates), so following a subset of columns through the whole event stream is exact.
Inputs come from the shared generator (synth.gen); events from the oracle's own clock code.
"""
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
        self.events = None
        self.done = 0

    def generate(self, n_events):
        """The first n_events events of the stream (the oracle's own clock code, from time 0)."""
        if self.fifo is not None:
            from oracle import fifo as fifo_source
            self.events = fifo_source.generate(self.cfg.n, self.edges, self.node_rate, self.fifo["comm_per_grad"],
                                               self.fifo["comm_time"], self.fifo["jitter"], self.cfg.seed, n_events,
                                               normalize=bool(self.fifo.get("normalize", False)))
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
        c_row = xi = xi_row = None
        if self.c is not None:
            c_row = np.where(is_grad, ev.i, -1)
        if cfg.xi_sigma > 0:
            ids = np.nonzero(is_grad)[0]
            xi = gen.normal_rows_fast(cfg.seed, gen.DOMAIN_XI, ids + self.done, self.cols, cfg.xi_sigma)
            xi_row = np.full(m, -1, np.int64)
            xi_row[ids] = np.arange(len(ids))
        # the engine receives gamma and gscale as fp32 values
        self.state.apply(ev, float(np.float32(cfg.gamma)), float(np.float32(cfg.gscale)), xi, xi_row, self.c, c_row)
        self.done = upto
        return self.state


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
