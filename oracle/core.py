"""ctypes view of the C oracle (test infrastructure; see a2cid_oracle.c for the readings used).

All state is fp64.  Inputs that the GPU side holds in fp32 (initial state, c_i, xi)
are widened exactly before they get here.
"""
import ctypes as C

import numpy as np

from . import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(_build.build())
        d_p = np.ctypeslib.ndpointer(np.float64, flags="C_CONTIGUOUS")
        i32_p = np.ctypeslib.ndpointer(np.int32, flags="C_CONTIGUOUS")
        i64_p = np.ctypeslib.ndpointer(np.int64, flags="C_CONTIGUOUS")
        u32_p = np.ctypeslib.ndpointer(np.uint32, flags="C_CONTIGUOUS")
        _lib.a2o_mix_row.argtypes = [d_p, d_p, C.c_int64, C.c_double, C.c_double]
        _lib.a2o_mix_row.restype = None
        _lib.a2o_apply_events.argtypes = [
            C.c_int32, C.c_int64, d_p, d_p, d_p, C.c_double, C.c_double, C.c_double,
            C.c_int64, d_p, i32_p, i32_p, i32_p, d_p, d_p,
            i64_p, C.c_void_p, i64_p, C.c_void_p, i64_p, C.c_void_p, C.c_int32, d_p, C.c_void_p]
        _lib.a2o_apply_events.restype = C.c_int64
        _lib.a2o_stats.argtypes = [C.c_int32, C.c_int64, d_p, d_p, d_p, C.c_double, C.c_double,
                                   C.POINTER(C.c_double), C.POINTER(C.c_double), d_p, d_p, d_p]
        _lib.a2o_stats.restype = C.c_int
        _lib.a2o_philox4x32_10.argtypes = [u32_p, u32_p, u32_p]
        _lib.a2o_philox4x32_10.restype = None
        _lib.a2o_generate_events.argtypes = [
            C.c_int32, C.c_int32, i32_p, i32_p, d_p, d_p, C.c_uint64, C.c_int64,
            d_p, i32_p, i32_p, i32_p, i32_p]
        _lib.a2o_generate_events.restype = C.c_int64
    return _lib


def philox4x32_10(counter, key):
    out = np.zeros(4, np.uint32)
    lib().a2o_philox4x32_10(np.asarray(counter, np.uint32), np.asarray(key, np.uint32), out)
    return out


class Events:
    """A serial event stream: parallel arrays, one entry per event, in time order."""

    def __init__(self, t, kind, i, j, clock=None, speed=None):
        """clock: which clock fired (worker, or n + edge index).  speed: per event, > 0 on a gradient event sets the
        speed of that worker's own clock from the event on (0 / None: unchanged)."""
        self.t = np.ascontiguousarray(t, np.float64)
        self.kind = np.ascontiguousarray(kind, np.int32)
        self.i = np.ascontiguousarray(i, np.int32)
        self.j = np.ascontiguousarray(j, np.int32)
        self.clock = None if clock is None else np.ascontiguousarray(clock, np.int32)
        self.speed = None if speed is None else np.ascontiguousarray(speed, np.float64)

    def __len__(self):
        return len(self.t)

    def __getitem__(self, s):
        return Events(self.t[s], self.kind[s], self.i[s], self.j[s],
                      None if self.clock is None else self.clock[s], None if self.speed is None else self.speed[s])


def generate_events(n, edges_u, edges_v, node_rate, edge_rate, seed, n_events):
    """Merged stream of the n node clocks and the per-edge clocks (Assumption 3.1)."""
    eu = np.ascontiguousarray(edges_u, np.int32)
    ev = np.ascontiguousarray(edges_v, np.int32)
    nr = np.ascontiguousarray(node_rate, np.float64)
    er = np.ascontiguousarray(edge_rate, np.float64)
    assert len(nr) == n and len(er) == len(eu) == len(ev)
    if len(eu) == 0:  # ndpointer rejects size-0 views of None; give it real arrays
        eu = np.zeros(1, np.int32); ev = np.zeros(1, np.int32); er = np.zeros(1, np.float64)
        ne = 0
    else:
        ne = len(edges_u)
    te = np.zeros(n_events, np.float64)
    kind = np.zeros(n_events, np.int32)
    wi = np.zeros(n_events, np.int32)
    wj = np.zeros(n_events, np.int32)
    clock = np.zeros(n_events, np.int32)
    got = lib().a2o_generate_events(n, ne, eu, ev, nr, er, int(seed), n_events, te, kind, wi, wj, clock)
    assert got >= 0
    return Events(te[:got], kind[:got], wi[:got], wj[:got], clock[:got])


class State:
    """x, xt (n x d, fp64) and the per-worker last-update times t (Algorithm 1, initialisation)."""

    def __init__(self, x0, xt0=None, eta=0.0, alpha=0.5, alpha_t=0.5, order=0):
        self.x = np.array(x0, dtype=np.float64, order="C")
        self.xt = self.x.copy() if xt0 is None else np.array(xt0, dtype=np.float64, order="C")
        assert self.x.ndim == 2 and self.x.shape == self.xt.shape
        self.n, self.d = self.x.shape
        self.t = np.zeros(self.n, np.float64)
        self.eta, self.alpha, self.alpha_t = float(eta), float(alpha), float(alpha_t)
        self.order = int(order)      # 0: jumps after the mixing (Eq. (1)); 1: Algorithm 1's listing order
        self.rate = np.ones(self.n, np.float64)   # speed of every worker's own clock against the event times

    def apply(self, ev, gamma=None, gscale=None, xi=None, xi_row=None, c=None, c_row=None, h=None, h_row=None):
        """Run the serial event loop over ev.

        gamma, gscale: per-event arrays (scalars broadcast).  xi: (m, d) matrix of additive
        gradient terms, xi_row[e] the row used by event e (-1: none); same for c, c_row (centres) and
        h, h_row (per-coordinate curvatures: g = gscale * h .* (x - c) + xi; none: h = 1).
        """
        m = len(ev)
        gamma = np.ascontiguousarray(np.broadcast_to(0.0 if gamma is None else gamma, (m,)), np.float64)
        gscale = np.ascontiguousarray(np.broadcast_to(0.0 if gscale is None else gscale, (m,)), np.float64)
        none = np.full(m, -1, np.int64)

        def prep(mat, rows):
            if mat is None:
                return None, none, None
            mat = np.ascontiguousarray(mat, np.float64)
            assert mat.ndim == 2 and mat.shape[1] == self.d
            rows = np.ascontiguousarray(rows, np.int64)
            assert rows.shape == (m,) and rows.max(initial=-1) < mat.shape[0]
            return mat, rows, mat.ctypes.data_as(C.c_void_p)

        xi_m, xi_r, xi_p = prep(xi, xi_row)
        c_m, c_r, c_p = prep(c, c_row)
        h_m, h_r, h_p = prep(h, h_row)
        rc = lib().a2o_apply_events(self.n, self.d, self.x, self.xt, self.t,
                                    self.eta, self.alpha, self.alpha_t, m,
                                    ev.t, ev.kind, ev.i, ev.j, gamma, gscale,
                                    xi_r, xi_p, c_r, c_p, h_r, h_p, self.order, self.rate,
                                    None if ev.speed is None else ev.speed.ctypes.data_as(C.c_void_p))
        if rc != 0:
            raise ValueError(f"malformed event at position {-rc - 1}")
        return self

    def stats(self, t_now):
        cx, cxt = C.c_double(), C.c_double()
        sx = np.zeros(self.n); sxt = np.zeros(self.n)
        rc = lib().a2o_stats(self.n, self.d, self.x, self.xt, self.t, self.eta, float(t_now),
                             C.byref(cx), C.byref(cxt), sx, sxt, self.rate)
        assert rc == 0
        return {"consensus_x": cx.value, "consensus_xt": cxt.value, "sum_x": sx, "sum_xt": sxt}

    def mix_workers(self, workers, t_now):
        """Applies the mixing flow up to t_now to the listed workers in place (and moves their time stamps)."""
        for i in workers:
            lib().a2o_mix_row(self.x[i], self.xt[i], self.d, self.eta, self.rate[i] * (float(t_now) - self.t[i]))
            self.t[i] = float(t_now)
        return self

    def average(self, t_now):
        """Every worker mixed to t_now, then every row replaced by the mean over workers (x and xt): the
        All-Reduce averaging the experimental protocol performs before and after training."""
        self.mix_workers(range(self.n), t_now)
        self.x[:] = self.x.mean(axis=0, keepdims=True)
        self.xt[:] = self.xt.mean(axis=0, keepdims=True)
        return self

    def flushed(self, t_now):
        """Copy of (x, xt) with every worker mixed up to t_now (what Algorithm 1 returns at T)."""
        x = self.x.copy(); xt = self.xt.copy()
        for i in range(self.n):
            lib().a2o_mix_row(x[i], xt[i], self.d, self.eta, self.rate[i] * (float(t_now) - self.t[i]))
        return x, xt


def mix(x, xt, eta, tau):
    """exp(tau * [[-eta, eta], [eta, -eta]]) applied element-wise to copies of (x, xt)."""
    x = np.array(x, np.float64).ravel().copy()
    xt = np.array(xt, np.float64).ravel().copy()
    lib().a2o_mix_row(x, xt, len(x), float(eta), float(tau))
    return x, xt
