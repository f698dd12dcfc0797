"""The five synthetic workloads and the device-side harness that feeds them to the engine.

Harness only: it allocates device memory through torch, fills it with the shared seeded
generator (synth), asks the library's scheduler for batches, attaches gradient inputs to the
gradient operations and calls a2cid_apply_events.  All arithmetic of the method happens inside
the library.

The workloads stand in for the paper's ResNet-18 / ResNet-50 runs on CIFAR-10 / ImageNet with
up to 64 workers on ring, exponential and complete graphs (section "Numerical Experiments"):
same flat-vector sizes, worker counts, topologies and communication rates, with Gaussian
initial parameters and an affine-plus-noise gradient model in place of datasets and networks.
"""
import numpy as np

from synth import gen

from synth.configs import CONFIGS, DOMAIN_RATE, GAMMA, Config, clock_rates, scaled  # noqa: F401  (re-exported)


def edge_list(topology, n):
    """Sorted undirected edge list (u < v)."""
    if topology == "complete":
        return [(i, j) for i in range(n) for j in range(i + 1, n)]
    if topology == "ring":
        return sorted({(min(i, (i + 1) % n), max(i, (i + 1) % n)) for i in range(n) if n > 1})
    if topology == "exponential":
        edges, k = set(), 1
        while k < n:
            for i in range(n):
                j = (i + k) % n
                if i != j:
                    edges.add((min(i, j), max(i, j)))
            k *= 2
        return sorted(edges)
    raise ValueError(topology)


def fifo_edge_rate(cfg, fifo):
    """Per-edge rate equivalent to every worker doing comm_per_grad averagings per gradient step with peers chosen
    uniformly among its neighbours: n * comm_per_grad * (gradient steps per worker and unit time) / 2 communications
    per unit time.  With the normalised clock a worker makes one gradient step per unit time."""
    node, _ = clock_rates(cfg)
    steps_per_unit_time = 1.0 if fifo.get("normalize") else float(node.mean())
    return cfg.n * fifo["comm_per_grad"] * steps_per_unit_time / 2.0 / len(edge_list(cfg.topology, cfg.n))


def grad_fraction(cfg):
    node, er = clock_rates(cfg)
    ne = len(edge_list(cfg.topology, cfg.n))
    return node.sum() / (node.sum() + er * ne)


class Workload:
    """Device-side instance of a config: state, gradient inputs, scheduler and engine."""

    def __init__(self, cfg, device="cuda:0", batch_events=1024, xi_slots=None, reuse_xi=False, fifo=None, ld_pad=0):
        """fifo = dict(comm_per_grad, comm_time, jitter[, normalize]) replaces the Poisson clocks by the first-in-first-out
        pairing source; the edge rate that enters chi_1, chi_2 is then comm_per_grad spread evenly over the edges
        (uniform pairing among neighbours, as the paper assumes when it computes them)."""
        import torch
        from . import binding
        from synth import fill
        self.torch, self.fill = torch, fill
        self.cfg, self.device = cfg, torch.device(device)
        self.batch_events = int(batch_events)
        self.reuse_xi = bool(reuse_xi)
        n, d = cfg.n, cfg.d
        self.ld = (d + 3) // 4 * 4 + 4 * int(ld_pad)      # row pitch in floats (a multiple of 4)
        edges = edge_list(cfg.topology, n)
        self.u = [e[0] for e in edges]
        self.v = [e[1] for e in edges]
        self.node_rate, self.edge_rate = clock_rates(cfg)
        if fifo is not None:
            self.edge_rate = fifo_edge_rate(cfg, fifo)
        if cfg.accelerated:
            p = binding.a2cid_graph_params(n, self.u, self.v, self.edge_rate)
            eta, alpha_t = p["eta"], p["alpha_tilde"]
            self.chi1, self.chi2 = p["chi1"], p["chi2"]
        else:
            eta, alpha_t = 0.0, 0.5
        self.eta = cfg.eta if cfg.eta is not None else eta
        self.alpha = 0.5
        self.alpha_tilde = cfg.alpha_tilde if cfg.alpha_tilde is not None else alpha_t

        with torch.cuda.device(self.device):
            self.x = torch.empty((n, self.ld), dtype=torch.float32, device=self.device)
            self.xt = torch.empty((n, self.ld), dtype=torch.float32, device=self.device)
            if self.ld != d:
                self.x[:, d:].fill_(float("nan"))      # padding must never be touched or used
                self.xt[:, d:].fill_(float("nan"))
            for i in range(n):
                fill.fill_normal(self.x[i, :d], cfg.seed, gen.DOMAIN_INIT, i, cfg.init_sigma)
            self.xt[:, :d].copy_(self.x[:, :d])       # Algorithm 1: xt_i <- x_i
            self.c = None
            if cfg.use_c:
                self.c = torch.empty((n, self.ld), dtype=torch.float32, device=self.device)
                for i in range(n):
                    fill.fill_normal(self.c[i, :d], cfg.seed, gen.DOMAIN_C, i, 1.0)
            self.h = None
            if cfg.curvature:
                self.h = torch.empty((n, self.ld), dtype=torch.float32, device=self.device)
                for i in range(n):
                    row = self.h[i, :d]
                    fill.fill_normal(row, cfg.seed, gen.DOMAIN_H, i, 1.0)
                    row.mul_(row).clamp_(max=4.0).mul_(0.75).add_(0.25)      # synth.gen.curvature, step by step
            self.xi = None
            if cfg.xi_sigma > 0:
                if xi_slots is None:
                    frac = grad_fraction(cfg) if fifo is None else 1.0 / (1.0 + 0.5 * fifo["comm_per_grad"])
                    xi_slots = min(self.batch_events, int(self.batch_events * frac * 1.5) + 16)
                self.xi = torch.empty((int(xi_slots), self.ld), dtype=torch.float32, device=self.device)
                if self.reuse_xi:
                    for s in range(self.xi.shape[0]):
                        fill.fill_normal(self.xi[s, :d], cfg.seed, gen.DOMAIN_XI, s, cfg.xi_sigma)
            self.engine = binding.Engine(self.x, self.xt, d, self.u, self.v, self.edge_rate, self.eta,
                                         self.alpha, self.alpha_tilde)
        self.sched = binding.Scheduler(n, self.u, self.v, self.edge_rate, self.node_rate, cfg.seed, fifo=fifo)
        if fifo is not None and fifo.get("normalize") == "worker":
            # every worker's clock starts at its nominal step rate and then follows its own measured steps
            self.engine.set_clock_rates(self.node_rate)
        self.events_done = 0
        self.t_last = 0.0

    def next_batch(self, max_events=None, t_sync=None):
        """Draws the next batch and attaches gamma, gscale, xi, c to its gradient operations.
        Per-event noise is regenerated into the slot pool unless reuse_xi is set."""
        cfg = self.cfg
        b = self.sched.next(self.batch_events if max_events is None else max_events)
        ops = b.ops
        grad = np.nonzero(ops["kind"] == 0)[0]
        ops["gamma"][grad] = cfg.gamma
        ops["gscale"][grad] = cfg.gscale
        row_bytes = self.ld * 4
        if self.c is not None:
            ops["c"][grad] = self.c.data_ptr() + ops["i"][grad].astype(np.uint64) * np.uint64(row_bytes)
        if self.h is not None:
            ops["h"][grad] = self.h.data_ptr() + ops["i"][grad].astype(np.uint64) * np.uint64(row_bytes)
        if self.xi is not None:
            slots = self.xi.shape[0]
            if not self.reuse_xi and len(grad) > slots:
                raise RuntimeError(f"batch has {len(grad)} gradient events but only {slots} noise slots")
            for s, k in enumerate(grad):
                slot = s % slots
                if not self.reuse_xi:
                    self.fill.fill_normal(self.xi[slot, :cfg.d], cfg.seed, gen.DOMAIN_XI, int(ops["id"][k]),
                                          cfg.xi_sigma)
                ops["xi"][k] = self.xi.data_ptr() + slot * row_bytes
        if t_sync is not None:
            b.t_sync = float(t_sync)
        if len(ops):
            self.t_last = float(ops["t"].max())
        return b

    def step(self, max_events=None):
        b = self.next_batch(max_events)
        self.engine.apply_events(b)
        self.events_done += len(b.ops)
        return b

    def run(self, events):
        left = int(events)
        while left > 0:
            b = self.step(min(left, self.batch_events))
            if len(b.ops) == 0:
                break
            left -= len(b.ops)
        return self

    def columns(self, cols):
        """(x[:, cols], xt[:, cols]) as numpy arrays after synchronising."""
        idx = self.torch.as_tensor(np.asarray(cols, np.int64), device=self.device)
        self.engine.synchronize()
        return self.x[:, idx].cpu().numpy(), self.xt[:, idx].cpu().numpy()

    def close(self):
        self.engine.close()
        self.sched.close()
