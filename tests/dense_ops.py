"""Dense jump / flow operators of the appendix's Ito decomposition, for brute-force pins.

State of one coordinate: v = (x_1..x_n, xt_1..xt_n, 1) in R^(2n+1).  Every event of the
dynamic is an affine map of v, written as a (2n+1) x (2n+1) matrix:

  flow over tau for worker w : identity except the 2x2 block on (w, n+w) = expm(tau * A),
                               A = [[-eta, eta], [eta, -eta]]  (scipy's matrix exponential)
  gossip on (i, j)           : x  <- (I - alpha E_ij) x,  xt <- xt - alpha_t E_ij x,
                               E_ij = (e_i - e_j)(e_i - e_j)^T
  gradient on i, g = s h (x_i - c) + xi : x_i <- x_i - gamma g, xt_i <- xt_i - gamma g
                               (h: the coordinate's curvature, 1 when none is given)
"""
import numpy as np
from scipy.linalg import expm


def flow(n, w, eta, tau):
    m = np.eye(2 * n + 1)
    blk = expm(tau * np.array([[-eta, eta], [eta, -eta]]))
    m[w, w], m[w, n + w], m[n + w, w], m[n + w, n + w] = blk[0, 0], blk[0, 1], blk[1, 0], blk[1, 1]
    return m


def gossip(n, i, j, alpha, alpha_t):
    v = np.zeros(n); v[i] = 1.0; v[j] = -1.0
    e = np.outer(v, v)
    m = np.eye(2 * n + 1)
    m[:n, :n] -= alpha * e
    m[n:2 * n, :n] -= alpha_t * e
    return m


def gradient(n, i, gamma, s, c_k, xi_k):
    m = np.eye(2 * n + 1)
    for row in (i, n + i):
        m[row, i] -= gamma * s
        m[row, 2 * n] += gamma * s * c_k - gamma * xi_k
    return m


def run(x0, xt0, eta, alpha, alpha_t, events, gamma, s, c, xi, t_final=None, order=0, h=None, flow_time=None):
    """events: list of (t, kind, i, j).  c: (n, d) or None.  xi: list (per event) of d-vectors or None.
    h: (n, d) per-worker, per-coordinate curvatures or None.
    flow_time: None, or a function (event index or None for the final flush, worker, t_from, t_to) -> duration of the
    flow of that worker between the two times (worker clocks that do not run at the speed of the event times).
    order 0: v <- J F v (flow, then the jump evaluated at the flowed state, Eq. (1));
    order 1: v <- F v + (J - I) v (the jump evaluated at the stored state, Algorithm 1's listing order).
    Returns (x, xt) after the events, every worker flowed to t_final if given."""
    n, d = x0.shape
    x = np.zeros((n, d)); xt = np.zeros((n, d))
    for k in range(d):
        v = np.concatenate([x0[:, k], xt0[:, k], [1.0]])
        t = np.zeros(n)
        total = np.eye(2 * n + 1)
        for e, (te, kind, i, j) in enumerate(events):
            ws = [i] if kind == 0 else [i, j]
            f = np.eye(2 * n + 1)
            for w in ws:
                f = flow(n, w, eta, te - t[w] if flow_time is None else flow_time(e, w, t[w], te)) @ f
                t[w] = te
            if kind == 0:
                ck = 0.0 if c is None else c[i, k]
                xk = 0.0 if xi is None or xi[e] is None else xi[e][k]
                hk = 1.0 if h is None else h[i, k]
                jump = gradient(n, i, gamma[e], s[e] * hk, ck, xk)
            else:
                jump = gossip(n, i, j, alpha, alpha_t)
            step = jump @ f if order == 0 else f + jump - np.eye(2 * n + 1)
            total = step @ total
        if t_final is not None:
            for w in range(n):
                total = flow(n, w, eta, t_final - t[w] if flow_time is None else flow_time(None, w, t[w], t_final)) @ total
        v = total @ v
        x[:, k], xt[:, k] = v[:n], v[n:2 * n]
    return x, xt
