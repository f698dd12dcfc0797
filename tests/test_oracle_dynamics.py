"""Pins for the oracle's state update: mixing flow, gradient and gossip jumps (Eq. (1), Algorithm 1),
the mean tracker (Eq. (2)), the consensus contraction of the appendix, and the observables."""
import numpy as np
import pytest
from scipy.linalg import expm

import dense_ops
from oracle import core, graph


def _events(n, edges, node_rate, edge_rate, seed, m):
    return core.generate_events(n, [e[0] for e in edges], [e[1] for e in edges],
                                np.broadcast_to(node_rate, (n,)).astype(float),
                                np.broadcast_to(edge_rate, (len(edges),)).astype(float), seed, m)


# ---------------------------------------------------------------- mixing flow
@pytest.mark.parametrize("eta,tau", [(0.5, 0.3), (3.3, 1.7), (0.14, 12.0), (18.0, 0.01), (1.0, 0.0)])
def test_mix_equals_matrix_exponential(eta, tau):
    rng = np.random.default_rng(1)
    x, xt = rng.normal(size=7), rng.normal(size=7)
    mx, mxt = core.mix(x, xt, eta, tau)
    big = expm(tau * np.array([[-eta, eta], [eta, -eta]]))
    ref = big @ np.stack([x, xt])
    assert np.allclose(mx, ref[0], rtol=1e-13, atol=1e-15)
    assert np.allclose(mxt, ref[1], rtol=1e-13, atol=1e-15)


def test_mix_semigroup_identity_limit_and_conservation():
    rng = np.random.default_rng(2)
    x, xt = rng.normal(size=50), rng.normal(size=50)
    a1 = core.mix(*core.mix(x, xt, 0.8, 0.4), 0.8, 1.1)
    a2 = core.mix(x, xt, 0.8, 1.5)
    assert np.allclose(a1[0], a2[0], rtol=1e-14) and np.allclose(a1[1], a2[1], rtol=1e-14)
    i0 = core.mix(x, xt, 0.0, 5.0)
    assert np.array_equal(i0[0], x) and np.array_equal(i0[1], xt)
    inf = core.mix(x, xt, 1.0, 1e3)
    assert np.allclose(inf[0], (x + xt) / 2) and np.allclose(inf[1], (x + xt) / 2)
    m = core.mix(x, xt, 2.0, 0.37)
    assert np.allclose(m[0] + m[1], x + xt, rtol=1e-15)
    assert np.allclose(m[0] - m[1], (x - xt) * np.exp(-2 * 2.0 * 0.37), rtol=1e-13)


# ---------------------------------------------------------------- whole path against dense operator products
@pytest.mark.parametrize("n,d,topo,seed", [(2, 3, "complete", 0), (3, 8, "ring", 1), (4, 8, "complete", 2),
                                           (4, 5, "ring", 3)])
def test_event_loop_equals_product_of_dense_operators(n, d, topo, seed):
    rng = np.random.default_rng(seed)
    edges = getattr(graph, topo)(n)
    ev = _events(n, edges, 1.0, 1.3, 100 + seed, 150)
    eta, alpha, alpha_t = 0.7, 0.45, 1.3
    x0 = rng.normal(size=(n, d)); xt0 = rng.normal(size=(n, d))
    c = rng.normal(size=(n, d))
    m = len(ev)
    gamma = rng.uniform(0.01, 0.2, m); s = rng.uniform(0.0, 1.5, m)
    is_grad = ev.kind == 0
    xi = rng.normal(size=(int(is_grad.sum()), d))
    xi_row = np.full(m, -1, np.int64); xi_row[is_grad] = np.arange(is_grad.sum())
    c_row = np.where(is_grad, ev.i, -1).astype(np.int64)

    st = core.State(x0, xt0, eta, alpha, alpha_t).apply(ev, gamma, s, xi, xi_row, c, c_row)
    T = ev.t[-1] + 0.25
    ox, oxt = st.flushed(T)

    evl = list(zip(ev.t, ev.kind, ev.i, ev.j))
    xi_l = [xi[xi_row[e]] if xi_row[e] >= 0 else None for e in range(m)]
    bx, bxt = dense_ops.run(x0, xt0, eta, alpha, alpha_t, evl, gamma, s, c, xi_l, t_final=T)
    assert np.allclose(ox, bx, rtol=1e-10, atol=1e-12)
    assert np.allclose(oxt, bxt, rtol=1e-10, atol=1e-12)


# ---------------------------------------------------------------- gossip jump
def test_gossip_half_is_exact_pairwise_average_and_conserves_sums():
    rng = np.random.default_rng(3)
    n, d = 5, 16
    x0 = rng.normal(size=(n, d)); xt0 = rng.normal(size=(n, d))
    ev = core.Events([0.0], [1], [1], [3])     # at t=0 no flow has happened yet
    st = core.State(x0, xt0, eta=0.9, alpha=0.5, alpha_t=2.0).apply(ev)
    avg = (x0[1] + x0[3]) / 2
    assert np.allclose(st.x[1], avg, rtol=1e-15) and np.allclose(st.x[3], avg, rtol=1e-15)
    # the momentum buffer moves by alpha_tilde times the x difference (not the xt difference)
    assert np.allclose(st.xt[1], xt0[1] - 2.0 * (x0[1] - x0[3]), rtol=1e-14)
    assert np.allclose(st.xt[3], xt0[3] + 2.0 * (x0[1] - x0[3]), rtol=1e-14)
    untouched = [0, 2, 4]
    assert np.array_equal(st.x[untouched], x0[untouched]) and np.array_equal(st.xt[untouched], xt0[untouched])
    assert np.allclose(st.x.sum(0), x0.sum(0), rtol=1e-14) and np.allclose(st.xt.sum(0), xt0.sum(0), rtol=1e-14)


def test_gossip_stream_conserves_column_sums_after_flush():
    # communication updates are orthogonal to 1; the flow conserves x_i + xt_i
    rng = np.random.default_rng(4)
    n, d = 8, 12
    edges = graph.ring(n)
    ev = _events(n, edges, 0.0, 1.0, 77, 400)
    x0 = rng.normal(size=(n, d))
    st = core.State(x0, None, eta=0.4, alpha=0.5, alpha_t=1.9).apply(ev)
    x, xt = st.flushed(ev.t[-1])
    assert np.allclose((x + xt).sum(0), 2 * x0.sum(0), rtol=1e-12)
    # with xbar(0) = xtbar(0) the two means stay equal (sentence before Eq. (2))
    assert np.allclose(x.sum(0), xt.sum(0), rtol=1e-10, atol=1e-12)


# ---------------------------------------------------------------- gradient jump and the mean tracker
def test_gradient_event_moves_both_buffers_by_the_same_amount():
    rng = np.random.default_rng(5)
    n, d = 3, 10
    x0 = rng.normal(size=(n, d)); xt0 = rng.normal(size=(n, d)); c = rng.normal(size=(n, d))
    xi = rng.normal(size=(1, d))
    ev = core.Events([0.0], [0], [2], [-1])
    st = core.State(x0, xt0, eta=0.6).apply(ev, gamma=0.1, gscale=0.8, xi=xi, xi_row=[0], c=c, c_row=[2])
    g = 0.8 * (x0[2] - c[2]) + xi[0]
    assert np.allclose(st.x[2], x0[2] - 0.1 * g, rtol=1e-15)
    assert np.allclose(st.xt[2], xt0[2] - 0.1 * g, rtol=1e-15)
    assert np.array_equal(st.x[:2], x0[:2])
    # after a flow of length tau the gradient is taken at the mixed point
    ev = core.Events([0.9], [0], [2], [-1])
    st = core.State(x0, xt0, eta=0.6).apply(ev, gamma=0.1, gscale=1.0, c=c, c_row=[2])
    mx, mxt = core.mix(x0[2], xt0[2], 0.6, 0.9)
    assert np.allclose(st.x[2], mx - 0.1 * (mx - c[2]), rtol=1e-14)
    assert np.allclose(st.xt[2], mxt - 0.1 * (mx - c[2]), rtol=1e-14)
    assert st.t[2] == 0.9 and st.t[0] == 0.0


def test_mean_tracker_eq2():
    # xbar(T) = xbar(0) - (1/n) sum_e gamma_e g_e  with g_e = xi_e here (gscale = 0), and xbar = xtbar
    rng = np.random.default_rng(6)
    n, d = 6, 9
    edges = graph.exponential(n)
    ev = _events(n, edges, 1.0, 1.0, 5, 600)
    is_grad = ev.kind == 0
    xi = rng.normal(size=(int(is_grad.sum()), d))
    xi_row = np.full(len(ev), -1, np.int64); xi_row[is_grad] = np.arange(is_grad.sum())
    gamma = rng.uniform(0.01, 0.1, len(ev))
    x0 = rng.normal(size=(n, d))
    p = graph.acid_params(n, edges, 1.0)
    st = core.State(x0, None, p["eta"], p["alpha"], p["alpha_tilde"]).apply(ev, gamma, 0.0, xi, xi_row)
    x, xt = st.flushed(ev.t[-1] + 1.0)
    drift = (gamma[is_grad, None] * xi).sum(0)
    assert np.allclose(x.sum(0), x0.sum(0) - drift, rtol=1e-10, atol=1e-10)
    assert np.allclose(xt.sum(0), x0.sum(0) - drift, rtol=1e-10, atol=1e-10)


# ---------------------------------------------------------------- baseline special case and contraction
def test_eta_zero_is_textbook_pairwise_gossip_plus_sgd():
    # eta = 0, alpha = 1/2 (Eq. (3)): randomized pairwise averaging (Boyd et al.) interleaved with SGD steps
    rng = np.random.default_rng(7)
    n, d = 7, 5
    edges = graph.ring(n)
    ev = _events(n, edges, 1.0, 2.0, 21, 500)
    x0 = rng.normal(size=(n, d)); c = rng.normal(size=(n, d))
    st = core.State(x0, None, 0.0, 0.5, 0.5).apply(ev, 0.1, 1.0, c=c, c_row=np.where(ev.kind == 0, ev.i, -1))
    x = x0.copy()
    for k, i, j in zip(ev.kind, ev.i, ev.j):
        if k == 0:
            x[i] = x[i] - 0.1 * (x[i] - c[i])
        else:
            x[i] = x[j] = (x[i] + x[j]) / 2
    assert np.allclose(st.x, x, rtol=1e-12, atol=1e-14)


def test_consensus_never_increases_under_plain_averaging():
    # eta = 0, alpha = 1/2, communications only: every event is an orthogonal projection
    rng = np.random.default_rng(8)
    n, d = 16, 20
    edges = graph.ring(n)
    ev = _events(n, edges, 0.0, 1.0, 3, 300)
    st = core.State(rng.normal(size=(n, d)), None, 0.0, 0.5, 0.5)
    prev = st.stats(0.0)["consensus_x"]
    for e in range(len(ev)):
        st.apply(ev[e:e + 1])
        cur = st.stats(ev.t[e])["consensus_x"]
        assert cur <= prev * (1 + 1e-14)
        prev = cur


def test_expected_consensus_decay_rate():
    # appendix, "Study of the ||pi x||_F^2 terms", alpha = 1/2, no gradients, eta = 0:
    #   d/dt E||pi x||^2 = 2 alpha (alpha - 1) E||x||_Lambda^2 = -1/2 E||x||_Lambda^2 <= -(1/(2 chi_1)) E||pi x||^2.
    # The second moment C = E[x x^T] of one coordinate obeys the linear ODE
    #   dC/dt = sum_ij lambda_ij (W_ij C W_ij - C),  W_ij = I - E_ij / 2,
    # solved here exactly with a Kronecker-product generator and scipy's expm; the oracle, averaged over
    # clock seeds and coordinates, must reproduce tr(pi C_T) and respect the chi_1 bound.
    rng = np.random.default_rng(9)
    n, d, T = 8, 500, 6.0
    edges = graph.ring(n)
    lam = graph.laplacian(n, edges, 1.0)
    c1 = graph.chi1(lam)
    gen = np.zeros((n * n, n * n))
    for i, j in edges:
        v = np.zeros(n); v[i] = 1.0; v[j] = -1.0
        w = np.eye(n) - 0.5 * np.outer(v, v)
        gen += np.kron(w, w) - np.eye(n * n)
    c_T = (expm(T * gen) @ np.eye(n).ravel()).reshape(n, n)      # C_0 = I: unit normal start
    pi = np.eye(n) - np.ones((n, n)) / n
    expect = d * np.trace(pi @ c_T)
    start = d * np.trace(pi)
    assert expect <= np.exp(-T / (2 * c1)) * start

    x0 = rng.normal(size=(n, d))
    vals = []
    for seed in range(60):
        ev = _events(n, edges, 0.0, 1.0, 1000 + seed, 400)
        k = int(np.searchsorted(ev.t, T))
        assert k < len(ev)
        vals.append(core.State(x0, None, 0.0, 0.5, 0.5).apply(ev[:k]).stats(T)["consensus_x"])
    # x0 is one draw: rescale the prediction by its actual starting consensus (expectation is linear in C_0,
    # and pi x0 x0^T pi / d concentrates on pi for d = 500)
    c0 = core.State(x0).stats(0.0)["consensus_x"]
    predicted = expect * c0 / start
    assert abs(np.mean(vals) - predicted) < 4 * np.std(vals) / np.sqrt(len(vals)) + 0.03 * predicted
    assert np.mean(vals) <= np.exp(-T / (2 * c1)) * c0


def test_acid_beats_baseline_on_the_ring():
    # the paper's claim in miniature (ring, communications only): the accelerated parameters shrink the
    # consensus distance faster than plain averaging at the same communication rate
    rng = np.random.default_rng(10)
    n, d = 16, 400
    edges = graph.ring(n)
    ev = _events(n, edges, 0.0, 1.0, 4, 16 * 60)
    x0 = rng.normal(size=(n, d))
    p = graph.acid_params(n, edges, 1.0)
    T = ev.t[-1]
    acc = core.State(x0, None, p["eta"], p["alpha"], p["alpha_tilde"]).apply(ev).stats(T)["consensus_x"]
    base = core.State(x0, None, 0.0, 0.5, 0.5).apply(ev).stats(T)["consensus_x"]
    assert acc < 0.2 * base


def test_quadratic_objective_converges_near_mean_of_minimisers():
    # config-1 style: f_i = 1/2 ||x - c_i||^2, no noise; the network average obeys Eq. (2) and settles around cbar
    rng = np.random.default_rng(11)
    n, d = 4, 50
    edges = graph.complete(n)
    ev = _events(n, edges, 1.0, 1.0, 12, 6000)
    c = rng.normal(size=(n, d)); x0 = rng.normal(size=(n, d))
    st = core.State(x0, None, 0.5, 0.5, 0.5).apply(ev, 0.05, 1.0, c=c, c_row=np.where(ev.kind == 0, ev.i, -1))
    x, _ = st.flushed(ev.t[-1])
    err0 = np.linalg.norm(x0.mean(0) - c.mean(0))
    err = np.linalg.norm(x.mean(0) - c.mean(0))
    assert err < 0.15 * err0


# ---------------------------------------------------------------- observables
def test_stats_against_library_variance_and_identities():
    rng = np.random.default_rng(12)
    n, d = 9, 33
    x0 = rng.normal(size=(n, d)); xt0 = rng.normal(size=(n, d))
    st = core.State(x0, xt0, eta=0.0)
    s = st.stats(0.0)
    assert np.isclose(s["consensus_x"], n * np.var(x0, axis=0).sum(), rtol=1e-13)
    assert np.isclose(s["consensus_xt"], (xt0 ** 2).sum() - n * (xt0.mean(0) ** 2).sum(), rtol=1e-12)
    assert np.allclose(s["sum_x"], x0.sum(1)) and np.allclose(s["sum_xt"], xt0.sum(1))
    same = core.State(np.tile(x0[:1], (n, 1))).stats(0.0)
    assert same["consensus_x"] < 1e-25 and same["consensus_xt"] < 1e-25    # mean of n equal values rounds


def test_stats_use_the_virtually_mixed_state_and_do_not_mutate():
    rng = np.random.default_rng(13)
    n, d = 4, 6
    x0 = rng.normal(size=(n, d)); xt0 = rng.normal(size=(n, d))
    st = core.State(x0, xt0, eta=0.7)
    st.t[:] = [0.0, 0.5, 1.0, 1.5]
    s = st.stats(2.0)
    fx, fxt = st.flushed(2.0)
    assert np.isclose(s["consensus_x"], n * np.var(fx, axis=0).sum(), rtol=1e-13)
    assert np.allclose(s["sum_xt"], fxt.sum(1), rtol=1e-13)
    assert np.allclose(s["sum_x"] + s["sum_xt"], (x0 + xt0).sum(1), rtol=1e-13)   # flow conserves x_i + xt_i
    assert np.array_equal(st.x, x0) and np.array_equal(st.xt, xt0)


def test_malformed_events_are_rejected():
    st = core.State(np.zeros((3, 2)))
    with pytest.raises(ValueError):
        st.apply(core.Events([1.0], [1], [0], [0]))          # self loop
    with pytest.raises(ValueError):
        st.apply(core.Events([1.0], [0], [5], [-1]))         # worker out of range
    st.apply(core.Events([1.0], [0], [1], [-1]), 0.1, 0.0)
    with pytest.raises(ValueError):
        st.apply(core.Events([0.5], [1], [1], [2]))          # time runs backwards for worker 1


@pytest.mark.parametrize("n,d,topo,seed", [(3, 4, "ring", 5), (4, 6, "complete", 6)])
def test_listing_order_variant_equals_its_dense_operator_product(n, d, topo, seed):
    # Algorithm 1 as listed: g and m_ij from the stored values, then the mixing, then the jump
    rng = np.random.default_rng(seed)
    edges = getattr(graph, topo)(n)
    ev = _events(n, edges, 1.0, 1.3, 200 + seed, 120)
    eta, alpha, alpha_t = 0.9, 0.5, 1.4
    x0 = rng.normal(size=(n, d)); xt0 = rng.normal(size=(n, d)); c = rng.normal(size=(n, d))
    m = len(ev)
    gamma = rng.uniform(0.01, 0.2, m); s = rng.uniform(0.0, 1.5, m)
    is_grad = ev.kind == 0
    xi = rng.normal(size=(int(is_grad.sum()), d))
    xi_row = np.full(m, -1, np.int64); xi_row[is_grad] = np.arange(is_grad.sum())
    c_row = np.where(is_grad, ev.i, -1).astype(np.int64)
    st = core.State(x0, xt0, eta, alpha, alpha_t, order=1).apply(ev, gamma, s, xi, xi_row, c, c_row)
    T = ev.t[-1] + 0.5
    ox, oxt = st.flushed(T)
    evl = list(zip(ev.t, ev.kind, ev.i, ev.j))
    xi_l = [xi[xi_row[e]] if xi_row[e] >= 0 else None for e in range(m)]
    bx, bxt = dense_ops.run(x0, xt0, eta, alpha, alpha_t, evl, gamma, s, c, xi_l, t_final=T, order=1)
    assert np.allclose(ox, bx, rtol=1e-10, atol=1e-12) and np.allclose(oxt, bxt, rtol=1e-10, atol=1e-12)
    # the two orders differ (unless eta = 0, where there is no flow to be stale against) ...
    st0 = core.State(x0, xt0, eta, alpha, alpha_t, order=0).apply(ev, gamma, s, xi, xi_row, c, c_row)
    assert not np.allclose(st0.x, st.x, rtol=1e-6)
    a = core.State(x0, xt0, 0.0, alpha, alpha_t, order=0).apply(ev, gamma, s, xi, xi_row, c, c_row)
    b = core.State(x0, xt0, 0.0, alpha, alpha_t, order=1).apply(ev, gamma, s, xi, xi_row, c, c_row)
    assert np.allclose(a.x, b.x, rtol=1e-13) and np.allclose(a.xt, b.xt, rtol=1e-13)
    # ... and both keep the invariants: column sums of x + xt move only by the gradient steps
    comm_only = _events(n, edges, 0.0, 1.0, 9, 80)
    s1 = core.State(x0, None, eta, alpha, alpha_t, order=1).apply(comm_only)
    fx, fxt = s1.flushed(comm_only.t[-1])
    assert np.allclose((fx + fxt).sum(0), 2 * x0.sum(0), rtol=1e-12)


def test_average_reaches_consensus_and_keeps_the_means():
    rng = np.random.default_rng(14)
    n, d = 6, 11
    edges = graph.ring(n)
    ev = _events(n, edges, 1.0, 1.0, 31, 200)
    x0 = rng.normal(size=(n, d))
    st = core.State(x0, None, 0.6, 0.5, 1.2).apply(ev, 0.05, 0.0, rng.normal(size=(int((ev.kind == 0).sum()), d)),
                                                   np.where(ev.kind == 0, np.cumsum(ev.kind == 0) - 1, -1))
    T = ev.t[-1] + 0.3
    fx, fxt = st.flushed(T)
    st.average(T)
    assert np.allclose(st.x, fx.mean(0, keepdims=True), rtol=1e-14) and np.allclose(st.xt, fxt.mean(0), rtol=1e-14)
    s = st.stats(T)
    assert s["consensus_x"] < 1e-25 and s["consensus_xt"] < 1e-25 and np.all(st.t == T)
    assert np.allclose(st.x.sum(0), fx.sum(0), rtol=1e-13)


# ---------------------------------------------------------------- strongly convex local objectives (curvature h)
def _diag_quadratics(rng, n, d, h_lo=0.5, h_hi=2.0):
    """f_i(x) = 1/2 sum_k h_ik (x_k - c_ik)^2: centres, curvatures and the minimiser of sum_i f_i."""
    c = rng.normal(size=(n, d))
    h = rng.uniform(h_lo, h_hi, size=(n, d))
    return c, h, (h * c).sum(0) / h.sum(0)


@pytest.mark.parametrize("order", [0, 1])
def test_event_loop_with_per_coordinate_curvature_equals_dense_operator_product(order):
    rng = np.random.default_rng(20 + order)
    n, d = 4, 7
    edges = graph.ring(n)
    ev = _events(n, edges, 1.0, 1.1, 300 + order, 140)
    eta, alpha, alpha_t = 0.8, 0.5, 1.2
    x0 = rng.normal(size=(n, d)); xt0 = rng.normal(size=(n, d))
    c, h, _ = _diag_quadratics(rng, n, d, 0.1, 3.0)
    m = len(ev)
    gamma = rng.uniform(0.01, 0.2, m); s = rng.uniform(0.2, 1.5, m)
    is_grad = ev.kind == 0
    xi = rng.normal(size=(int(is_grad.sum()), d))
    xi_row = np.full(m, -1, np.int64); xi_row[is_grad] = np.arange(is_grad.sum())
    row = np.where(is_grad, ev.i, -1).astype(np.int64)
    st = core.State(x0, xt0, eta, alpha, alpha_t, order=order).apply(ev, gamma, s, xi, xi_row, c, row, h, row)
    T = ev.t[-1] + 0.3
    ox, oxt = st.flushed(T)
    evl = list(zip(ev.t, ev.kind, ev.i, ev.j))
    xi_l = [xi[xi_row[e]] if xi_row[e] >= 0 else None for e in range(m)]
    bx, bxt = dense_ops.run(x0, xt0, eta, alpha, alpha_t, evl, gamma, s, c, xi_l, t_final=T, order=order, h=h)
    assert np.allclose(ox, bx, rtol=1e-10, atol=1e-12) and np.allclose(oxt, bxt, rtol=1e-10, atol=1e-12)
    # the curvature matters: the same run with h = 1 ends elsewhere
    flat = core.State(x0, xt0, eta, alpha, alpha_t, order=order).apply(ev, gamma, s, xi, xi_row, c, row)
    assert not np.allclose(flat.x, st.x, rtol=1e-3)


def test_repeated_gradient_steps_on_a_diagonal_quadratic_follow_the_textbook_closed_form():
    # one worker, eta = 0 (no flow), N gradient events with constant step: gradient descent on
    # f(x) = s/2 sum_k h_k (x_k - c_k)^2 gives x_k(N) = c_k + (1 - gamma s h_k)^N (x_k(0) - c_k), coordinate by
    # coordinate; xt receives the same increments
    rng = np.random.default_rng(22)
    n, d, N, gamma, s = 3, 12, 40, 0.15, 0.7
    x0 = rng.normal(size=(n, d)); xt0 = rng.normal(size=(n, d))
    c, h, _ = _diag_quadratics(rng, n, d, 0.1, 4.0)
    ev = core.Events(np.arange(1, N + 1, dtype=float), np.zeros(N, np.int32), np.full(N, 1, np.int32),
                     np.full(N, -1, np.int32))
    row = np.full(N, 1, np.int64)
    st = core.State(x0, xt0, eta=0.0).apply(ev, gamma, s, c=c, c_row=row, h=h, h_row=row)
    want = c[1] + (1.0 - gamma * s * h[1]) ** N * (x0[1] - c[1])
    assert np.allclose(st.x[1], want, rtol=1e-12, atol=1e-14)
    assert np.allclose(st.xt[1] - xt0[1], want - x0[1], rtol=1e-11, atol=1e-13)
    assert np.array_equal(st.x[[0, 2]], x0[[0, 2]])
    # a curvature row of another worker may be attached to the event: the row index is what counts
    other = core.State(x0, xt0, eta=0.0).apply(ev, gamma, s, c=c, c_row=row, h=h, h_row=np.full(N, 2, np.int64))
    assert np.allclose(other.x[1], c[1] + (1.0 - gamma * s * h[2]) ** N * (x0[1] - c[1]), rtol=1e-12, atol=1e-14)


def test_network_mean_is_stationary_exactly_at_the_minimiser_of_the_sum_of_local_objectives():
    # all workers at x* = argmin sum_i f_i = (sum_i h_i c_i) / (sum_i h_i), x = xt (so the flow moves nothing): one
    # gradient event per worker, at any times, leaves the network mean where it is because sum_i grad f_i(x*) = 0
    # (Eq. (2) with a vanishing right-hand side); from the mean of the centres instead, the mean moves
    rng = np.random.default_rng(23)
    n, d, gamma = 6, 9, 0.1
    c, h, x_star = _diag_quadratics(rng, n, d)
    order = rng.permutation(n).astype(np.int32)
    ev = core.Events(np.sort(rng.uniform(0.1, 2.0, n)), np.zeros(n, np.int32), order, np.full(n, -1, np.int32))
    row = order.astype(np.int64)
    at_opt = core.State(np.tile(x_star, (n, 1)), None, 0.4, 0.5, 1.3).apply(ev, gamma, 1.0, c=c, c_row=row, h=h, h_row=row)
    x, xt = at_opt.flushed(3.0)
    assert np.allclose(x.mean(0), x_star, rtol=1e-13, atol=1e-14) and np.allclose(xt.mean(0), x_star, rtol=1e-13, atol=1e-14)
    off = core.State(np.tile(c.mean(0), (n, 1)), None, 0.4, 0.5, 1.3).apply(ev, gamma, 1.0, c=c, c_row=row, h=h, h_row=row)
    assert np.abs(off.flushed(3.0)[0].mean(0) - c.mean(0)).max() > 1e-3


def test_workers_settle_around_the_minimiser_of_the_sum_not_around_the_mean_of_the_centres():
    rng = np.random.default_rng(24)
    n, d, gamma = 4, 16, 0.025
    edges = graph.complete(n)
    ev = _events(n, edges, 1.0, 10.0, 77, 120000)
    c, h, x_star = _diag_quadratics(rng, n, d)
    x0 = 3.0 * rng.normal(size=(n, d))
    p = graph.acid_params(n, edges, 10.0)
    row = np.where(ev.kind == 0, ev.i, -1).astype(np.int64)
    st = core.State(x0, None, p["eta"], p["alpha"], p["alpha_tilde"]).apply(ev, gamma, 1.0, c=c, c_row=row, h=h, h_row=row)
    x, xt = st.flushed(ev.t[-1])
    err, err0 = np.abs(x - x_star).max(), np.abs(x0 - x_star).max()
    assert err < 0.03 * err0                                  # a neighbourhood of size O(gamma) of the minimiser
    assert err < 0.5 * np.abs(x - c.mean(0)).max()            # ... and not of the mean of the centres
    assert np.allclose(x.sum(0), xt.sum(0), rtol=1e-10, atol=1e-10)     # Eq. (2): the two means stay together


def test_accelerated_parameters_reach_a_tighter_neighbourhood_of_the_optimum_on_the_ring():
    # Proposition 3.2, strongly convex case: the heterogeneity of the local objectives enters the bound with a
    # factor (1 + chi): chi_1 = 6.6 for plain averaging on the ring of 16, sqrt(chi_1 chi_2) = 1.8 with the
    # accelerated parameters.  Same events, same objectives: the distance to the optimum levels off lower.
    rng = np.random.default_rng(25)
    n, d, gamma = 16, 64, 0.05
    edges = graph.ring(n)
    ev = _events(n, edges, 1.0, 1.0, 77, 20000)
    c, h, x_star = _diag_quadratics(rng, n, d, 0.2, 2.0)
    x0 = np.tile(3.0 * rng.normal(size=d), (n, 1))            # the workers start in consensus, as in the paper
    p = graph.acid_params(n, edges, 1.0)
    row = np.where(ev.kind == 0, ev.i, -1).astype(np.int64)
    level = {}
    for label, (eta, alpha_t) in {"accelerated": (p["eta"], p["alpha_tilde"]), "baseline": (0.0, 0.5)}.items():
        st = core.State(x0, None, eta, 0.5, alpha_t)
        dist = []
        for lo in range(0, len(ev), 2000):
            part = ev[lo:lo + 2000]
            st.apply(part, gamma, 1.0, c=c, c_row=row[lo:lo + 2000], h=h, h_row=row[lo:lo + 2000])
            x, _ = st.flushed(part.t[-1])
            dist.append(np.sqrt(((x - x_star) ** 2).sum(1).mean()))
        assert dist[0] < 0.5 * np.sqrt(((x0 - x_star) ** 2).sum(1).mean())     # the transient is over early
        level[label] = np.mean(dist[2:])
    assert level["accelerated"] < 0.8 * level["baseline"]


# ---------------------------------------------------------------- worker clocks (time normalised per worker)

def test_worker_clocks_equal_dense_operators_with_flows_of_the_workers_own_durations():
    """Every worker's flow between two of its events lasts (speed of its clock) x (difference of the event times); a
    gradient event may set a new speed, which counts from that event on.  The speeds are tracked here by hand and
    handed to the dense operators as flow durations."""
    rng = np.random.default_rng(5)
    n, d = 4, 6
    edges = graph.ring(n)
    ev = _events(n, edges, 1.0, 1.3, 321, 160)
    m = len(ev)
    is_grad = ev.kind == 0
    speed = np.where(is_grad & (rng.random(m) < 0.7), rng.uniform(0.3, 2.5, m), 0.0)
    ev = core.Events(ev.t, ev.kind, ev.i, ev.j, ev.clock, speed)
    rate0 = rng.uniform(0.5, 2.0, n)
    eta, alpha, alpha_t = 0.6, 0.5, 1.2
    x0 = rng.normal(size=(n, d)); xt0 = rng.normal(size=(n, d))
    gamma = rng.uniform(0.01, 0.2, m); s = rng.uniform(0.0, 1.5, m)
    c = rng.normal(size=(n, d))
    c_row = np.where(is_grad, ev.i, -1).astype(np.int64)
    for order in (0, 1):
        st = core.State(x0, xt0, eta, alpha, alpha_t, order=order)
        st.rate[:] = rate0
        st.apply(ev, gamma, s, None, None, c, c_row)
        T = ev.t[-1] + 0.4
        ox, oxt = st.flushed(T)
        # by hand: the speed in force for worker w when event e (or the final flush) mixes it
        in_force = np.zeros((m + 1, n))
        cur = rate0.copy()
        for e in range(m):
            in_force[e] = cur
            if is_grad[e] and speed[e] > 0:
                cur[ev.i[e]] = speed[e]
        in_force[m] = cur
        assert np.array_equal(st.rate, cur)
        bx, bxt = dense_ops.run(x0, xt0, eta, alpha, alpha_t, list(zip(ev.t, ev.kind, ev.i, ev.j)), gamma, s, c,
                                [None] * m, t_final=T, order=order,
                                flow_time=lambda e, w, a, b: in_force[m if e is None else e, w] * (b - a))
        assert np.allclose(ox, bx, rtol=1e-10, atol=1e-12) and np.allclose(oxt, bxt, rtol=1e-10, atol=1e-12)
        assert not np.allclose(ox, core.State(x0, xt0, eta, alpha, alpha_t, order=order).apply(
            core.Events(ev.t, ev.kind, ev.i, ev.j), gamma, s, None, None, c, c_row).flushed(T)[0], rtol=1e-3)


def test_one_common_clock_speed_is_a_change_of_eta():
    """All clocks at the same constant speed s: eta only ever multiplies an elapsed time, so the run equals the plain
    dynamic with eta s; and the observables, which mix every worker to a common time, follow."""
    rng = np.random.default_rng(8)
    n, d = 5, 7
    ev = _events(n, graph.complete(n), 1.0, 0.8, 77, 300)
    x0 = rng.normal(size=(n, d))
    a = core.State(x0, None, 0.4, 0.5, 0.9)
    a.rate[:] = 1.75
    a.apply(ev, 0.05, 1.0)
    b = core.State(x0, None, 0.4 * 1.75, 0.5, 0.9).apply(ev, 0.05, 1.0)
    assert np.allclose(a.x, b.x, rtol=1e-12, atol=1e-14) and np.allclose(a.xt, b.xt, rtol=1e-12, atol=1e-14)
    T = ev.t[-1] + 1.0
    sa, sb = a.stats(T), b.stats(T)
    assert np.isclose(sa["consensus_xt"], sb["consensus_xt"], rtol=1e-11)
    assert np.allclose(sa["sum_x"], sb["sum_x"], rtol=1e-11)
    a.average(T); b.average(T)
    assert np.allclose(a.x, b.x, rtol=1e-12, atol=1e-14)
