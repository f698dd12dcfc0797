"""CPU tests of the library's host side: exported symbols, graph quantities, scheduler, planner.
No kernel is launched here."""
import ctypes as C
import math
import os
import re

import numpy as np
import pytest

import paper_2306_08289_amd as a2
from paper_2306_08289_amd import binding
from oracle import core, graph, levels

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _uv(edges):
    return [e[0] for e in edges], [e[1] for e in edges]


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "a2cid.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(a2cid_[a-z_]+)\s*\(", header))
    assert len(declared) >= 20
    lib = C.CDLL(binding.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name
    assert declared == set(binding.SIGNATURES), declared ^ set(binding.SIGNATURES)
    assert b"gfx950" in a2.load().a2cid_version()


@pytest.mark.parametrize("topo,n,rate", [("complete", 4, 1.0), ("ring", 16, 1.0), ("ring", 64, 2.0),
                                         ("exponential", 64, 1.0), ("exponential", 16, 0.4),
                                         ("complete", 64, 0.56), ("ring", 1024, 1.0), ("ring", 2, 3.0),
                                         ("exponential", 600, 0.7)])
def test_graph_params_match_oracle(topo, n, rate):
    edges = getattr(graph, topo)(n)
    u, v = _uv(edges)
    got = a2.a2cid_graph_params(n, u, v, rate)
    want = graph.acid_params(n, edges, rate)
    for k in ("chi1", "chi2", "eta", "alpha_tilde"):
        assert math.isclose(got[k], want[k], rel_tol=1e-9), k


def test_graph_params_heterogeneous_rates_and_errors():
    rng = np.random.default_rng(0)
    n = 9
    edges = sorted(set(graph.ring(n)) | {(0, 4), (2, 7), (1, 5)})
    rates = rng.uniform(0.2, 2.0, len(edges))
    u, v = _uv(edges)
    got = a2.a2cid_graph_params(n, u, v, rates)
    want = graph.acid_params(n, edges, rates)
    assert math.isclose(got["chi1"], want["chi1"], rel_tol=1e-9)
    assert math.isclose(got["chi2"], want["chi2"], rel_tol=1e-9)
    with pytest.raises(a2.A2cidError) as e:
        a2.a2cid_graph_params(4, [0, 2], [1, 3], 1.0)          # two components
    assert e.value.code == binding.EGRAPH
    with pytest.raises(a2.A2cidError) as e:
        a2.a2cid_graph_params(4, [1], [0], 1.0)                # u >= v
    assert e.value.code == binding.EGRAPH
    with pytest.raises(a2.A2cidError) as e:
        a2.a2cid_graph_params(4, [0, 0], [1, 1], 1.0)          # duplicate
    assert e.value.code == binding.EGRAPH
    with pytest.raises(a2.A2cidError) as e:
        a2.a2cid_graph_params(1, [], [], 1.0)
    assert e.value.code == binding.EINVAL


# ------------------------------------------------------------------ scheduler
@pytest.mark.parametrize("topo,n,node_rate,edge_rate,seed", [
    ("complete", 4, 1.0, 1.0, 0xA2C1D2), ("ring", 16, 1.0, 1.0, 0xA2C1D3), ("ring", 64, 1.0, 2.0, 0xA2C1D4),
    ("exponential", 64, 1.0, 1.0, (7 << 32) + 5), ("complete", 64, None, None, 0xA2C1D6)])
def test_schedule_is_bit_identical_to_the_oracle_stream(topo, n, node_rate, edge_rate, seed):
    edges = getattr(graph, topo)(n)
    u, v = _uv(edges)
    if node_rate is None:       # straggler clocks: log-normal node rates, edges at half their mean
        node_rate = np.exp(0.5 * np.random.default_rng(1).normal(size=n))
        edge_rate = 0.5 * node_rate.mean()
    node_rate = np.broadcast_to(node_rate, (n,)).astype(float)
    m = 20000
    ref = core.generate_events(n, u, v, node_rate, np.full(len(edges), edge_rate), seed, m)
    s = a2.Scheduler(n, u, v, edge_rate, node_rate, seed)
    got = []
    batch_size = 1024
    while sum(len(b.ops) for b in got) < m:
        got.append(s.next(min(batch_size, m - sum(len(b.ops) for b in got))))
    ref_batches = levels.pack(ref.kind, ref.i, ref.j, batch_size)
    assert len(got) == len(ref_batches)
    for b, rb in zip(got, ref_batches):
        order = [e for lev in rb for e in lev]
        assert b.n_levels == len(rb)
        assert list(b.level_off) == list(np.cumsum([0] + [len(lev) for lev in rb]))
        assert np.array_equal(b.ops["id"], order)
        assert np.array_equal(b.ops["t"], ref.t[order])          # bit-exact times
        assert np.array_equal(b.ops["kind"], ref.kind[order])
        assert np.array_equal(b.ops["i"], ref.i[order]) and np.array_equal(b.ops["j"], ref.j[order])
        assert np.all(b.ops["xi"] == 0) and np.all(b.ops["c"] == 0) and math.isnan(b.t_sync)
    counts = s.counts()
    assert counts.sum() == m and np.array_equal(counts, np.bincount(ref.clock, minlength=n + len(edges)))


def test_scheduler_skip_resumes_the_same_stream_and_dead_clocks():
    n = 8
    edges = graph.ring(n)
    u, v = _uv(edges)
    a = a2.Scheduler(n, u, v, 1.0, 1.0, 99)
    whole = a.next(500)
    b = a2.Scheduler(n, u, v, 1.0, 1.0, 99)
    b.skip(200)
    rest = b.next(300)
    ids = np.sort(rest.ops["id"])
    assert ids[0] == 200 and ids[-1] == 499
    by_id = {int(o["id"]): o for o in whole.ops}
    for o in rest.ops:
        w = by_id[int(o["id"])]
        assert o["t"] == w["t"] and o["i"] == w["i"] and o["j"] == w["j"] and o["kind"] == w["kind"]
    dead = a2.Scheduler(n, u, v, 0.0, 0.0, 1)
    assert len(dead.next(10).ops) == 0
    comm_only = a2.Scheduler(n, u, v, 1.0, 0.0, 1).next(100)
    assert np.all(comm_only.ops["kind"] == a2.KIND_GOSSIP)
    assert len(a.next(0).ops) == 0


# ------------------------------------------------------------------ planner
def _batch(ops, level_off, t_sync=float("nan")):
    arr = np.zeros(len(ops), a2.OP_DTYPE)
    for k, o in enumerate(ops):
        for key, val in o.items():
            arr[k][key] = val
    return a2.Batch(arr, level_off, t_sync)


def test_planner_coefficients_and_time_stamps():
    n, eta = 4, 0.7
    u, v = _uv(graph.complete(n))
    t0 = np.array([0.0, 0.5, 1.0, 0.25])
    b = _batch([dict(t=1.5, kind=1, i=0, j=1), dict(t=1.25, kind=0, i=2, j=-1, gamma=0.1),
                dict(t=2.0, kind=1, i=2, j=0), dict(t=2.5, kind=0, i=1, j=-1)], [0, 2, 4])
    t1, coef = a2.a2cid_plan_batch(n, u, v, 1.0, eta, t0, b)
    assert list(t1) == [2.0, 2.5, 2.0, 0.25]
    bco = lambda tau: np.float32(0.5 * (1 - math.exp(-2 * eta * tau)))
    assert coef["b_pre_i"][0] == bco(1.5) and coef["b_pre_j"][0] == bco(1.0)
    assert coef["b_pre_i"][1] == bco(0.25) and coef["b_pre_j"][1] == 0
    assert coef["b_pre_i"][2] == bco(0.75) and coef["b_pre_j"][2] == bco(0.5)
    assert coef["b_pre_i"][3] == bco(1.0)
    assert np.all(coef["b_post_i"] == 0) and np.all(coef["b_post_j"] == 0)
    # the closed form against the matrix exponential (independent route)
    from scipy.linalg import expm
    assert math.isclose(float(coef["b_pre_i"][0]), expm(1.5 * np.array([[-eta, eta], [eta, -eta]]))[0, 1], rel_tol=1e-6)
    # eta = 0: identity flow
    _, c0 = a2.a2cid_plan_batch(n, u, v, 1.0, 0.0, t0, b)
    assert np.all(c0["b_pre_i"] == 0) and np.all(c0["b_pre_j"] == 0)
    # tiny eta * tau keeps relative accuracy (expm1 form)
    t2, c2 = a2.a2cid_plan_batch(n, u, v, 1.0, 1e-9, np.zeros(n), _batch([dict(t=1e-3, kind=0, i=0, j=-1)], [0, 1]))
    assert math.isclose(float(c2["b_pre_i"][0]), 1e-12, rel_tol=1e-6)


def test_planner_trailing_mix_goes_to_each_workers_last_operation():
    n, eta = 4, 0.3
    u, v = _uv(graph.complete(n))
    b = _batch([dict(t=1.0, kind=1, i=0, j=1), dict(t=2.0, kind=0, i=1, j=-1), dict(t=2.5, kind=1, i=2, j=0)],
               [0, 1, 2, 3], t_sync=4.0)
    t1, coef = a2.a2cid_plan_batch(n, u, v, 1.0, eta, np.zeros(n), b)
    assert list(t1) == [4.0, 4.0, 4.0, 0.0]            # worker 3 is not touched by the batch
    bco = lambda tau: np.float32(0.5 * (1 - math.exp(-2 * eta * tau)))
    assert coef["b_post_i"][0] == 0 and coef["b_post_j"][0] == 0     # both have later operations
    assert coef["b_post_i"][1] == bco(2.0)
    assert coef["b_post_i"][2] == bco(1.5) and coef["b_post_j"][2] == bco(1.5)


@pytest.mark.parametrize("ops,level_off,t_sync,code", [
    ([dict(t=1.0, kind=1, i=0, j=1), dict(t=1.0, kind=0, i=1, j=-1)], [0, 2], float("nan"), binding.EMATCHING),
    ([dict(t=1.0, kind=1, i=0, j=2)], [0, 1], float("nan"), binding.EGRAPH),           # not an edge of the ring
    ([dict(t=0.4, kind=0, i=3, j=-1)], [0, 1], float("nan"), binding.EORDER),           # worker 3 is at t = 0.5
    ([dict(t=1.0, kind=0, i=0, j=-1), dict(t=0.9, kind=0, i=0, j=-1)], [0, 1, 2], float("nan"), binding.EORDER),
    ([dict(t=1.0, kind=7, i=0, j=-1)], [0, 1], float("nan"), binding.EINVAL),
    ([dict(t=1.0, kind=0, i=9, j=-1)], [0, 1], float("nan"), binding.EINVAL),
    ([dict(t=1.0, kind=1, i=1, j=1)], [0, 1], float("nan"), binding.EINVAL),
    ([dict(t=float("inf"), kind=0, i=0, j=-1)], [0, 1], float("nan"), binding.EINVAL),
    ([dict(t=1.0, kind=0, i=0, j=-1, gamma=float("nan"))], [0, 1], float("nan"), binding.EINVAL),
    ([dict(t=1.0, kind=0, i=0, j=-1, xi=8)], [0, 1], float("nan"), binding.EALIGN),
    ([dict(t=1.0, kind=0, i=0, j=-1, h=4100)], [0, 1], float("nan"), binding.EALIGN),
    ([dict(t=1.0, kind=0, i=0, j=-1)], [0, 2], float("nan"), binding.EMATCHING),        # table does not end at n_ops
    ([dict(t=1.0, kind=0, i=0, j=-1)], [0, 1], 0.5, binding.EORDER),                    # t_sync before an event
    ([dict(t=1.0, kind=0, i=0, j=-1)], [0, 1], float("inf"), binding.EINVAL),
])
def test_planner_rejects_bad_batches_and_leaves_times_untouched(ops, level_off, t_sync, code):
    n = 4
    u, v = _uv(graph.ring(n))
    t0 = np.array([0.0, 0.0, 0.0, 0.5])
    with pytest.raises(a2.A2cidError) as e:
        a2.a2cid_plan_batch(n, u, v, 1.0, 0.5, t0, _batch(ops, level_off, t_sync))
    assert e.value.code == code, str(e.value)
    assert list(t0) == [0.0, 0.0, 0.0, 0.5]


def test_empty_batch_is_fine():
    n = 4
    u, v = _uv(graph.ring(n))
    t1, coef = a2.a2cid_plan_batch(n, u, v, 1.0, 0.5, np.zeros(n), _batch([], [0]))
    assert len(coef) == 0 and np.all(t1 == 0)


# ------------------------------------------------------------------ first-in-first-out pairing source
@pytest.mark.parametrize("normalize", [False, True, "worker"])
@pytest.mark.parametrize("topo,n,rho,comm_time,jitter,seed", [
    ("ring", 16, 1.0, 0.05, 0.2, 3), ("exponential", 64, 1.0, 0.02, 0.1, (5 << 32) + 1),
    ("complete", 8, 2.0, 0.0, 0.0, 7), ("ring", 64, 2.0, 0.01, 0.5, 11)])
def test_fifo_schedule_is_bit_identical_to_the_oracle_stream(topo, n, rho, comm_time, jitter, seed, normalize):
    from oracle import fifo
    edges = getattr(graph, topo)(n)
    u, v = _uv(edges)
    rate = np.exp(0.3 * np.random.default_rng(2).normal(size=n)) if jitter > 0 else np.ones(n)
    m = 6000
    ref = fifo.generate(n, edges, rate, rho, comm_time, jitter, seed, m, normalize=normalize)
    s = a2.Scheduler(n, u, v, 1.0, rate, seed, fifo=dict(comm_per_grad=rho, comm_time=comm_time, jitter=jitter,
                                                         normalize=normalize))
    got = [s.next(1500) for _ in range(4)]
    ref_batches = levels.pack(ref.kind, ref.i, ref.j, 1500)
    for b, rb in zip(got, ref_batches):
        order = [e for lev in rb for e in lev]
        assert list(b.level_off) == list(np.cumsum([0] + [len(lev) for lev in rb]))
        assert np.array_equal(b.ops["id"], order)
        assert np.array_equal(b.ops["t"], ref.t[order])
        assert np.array_equal(b.ops["kind"], ref.kind[order])
        assert np.array_equal(b.ops["i"], ref.i[order]) and np.array_equal(b.ops["j"], ref.j[order])
        # the speeds of the workers' own clocks: bit-equal fp32 values on gradient events, 0 elsewhere
        want = ref.speed[order] if normalize == "worker" else np.zeros(len(order))
        assert np.array_equal(b.ops["clock_rate"].astype(np.float64), want)
    assert np.array_equal(s.counts(), np.bincount(ref.clock, minlength=n + len(edges)))


def test_plan_batch_with_worker_clocks_scales_every_workers_elapsed_time_by_its_own_speed():
    n = 4
    u, v = _uv(graph.ring(n))
    eta = 0.8
    ops = np.zeros(5, binding.OP_DTYPE)
    ops["kind"] = [binding.KIND_GRADIENT, binding.KIND_GOSSIP, binding.KIND_GRADIENT, binding.KIND_GOSSIP, binding.KIND_GRADIENT]
    ops["i"], ops["j"] = [0, 0, 2, 1, 0], [-1, 1, -1, 2, -1]
    ops["t"] = [0.5, 0.9, 1.0, 1.6, 2.0]
    ops["clock_rate"] = [2.5, 0.0, 0.0, 0.0, 0.25]        # worker 0 changes speed twice, worker 2 keeps its own
    b = binding.Batch(ops, [0, 1, 2, 3, 4, 5], t_sync=3.0)
    rate0 = np.array([0.5, 1.0, 3.0, 1.0])
    t1, coef, rate1 = a2.a2cid_plan_batch(n, u, v, 1.0, eta, np.zeros(n), b, clock_rates=rate0)
    bcoef = lambda tau: np.float32(0.5 * -np.expm1(-2.0 * eta * tau))
    # worker 0: 0.5 elapsed at speed 0.5 (the new speed counts after the event), then 0.4 at 2.5, then 1.1 at 2.5, then
    # the trailing mix of 1.0 at 0.25; worker 1: speed 1 throughout; worker 2: speed 3 throughout
    assert coef["b_pre_i"][0] == bcoef(0.5 * 0.5)
    assert coef["b_pre_i"][1] == bcoef(2.5 * 0.4) and coef["b_pre_j"][1] == bcoef(1.0 * 0.9)
    assert coef["b_pre_i"][2] == bcoef(3.0 * 1.0)
    assert coef["b_pre_i"][3] == bcoef(1.0 * 0.7) and coef["b_pre_j"][3] == bcoef(3.0 * 0.6)
    assert coef["b_pre_i"][4] == bcoef(2.5 * 1.1)
    assert coef["b_post_i"][4] == bcoef(0.25 * 1.0)
    assert coef["b_post_i"][3] == bcoef(1.0 * 1.4) and coef["b_post_j"][3] == bcoef(3.0 * 1.4)
    assert np.array_equal(rate1, [0.25, 1.0, 3.0, 1.0]) and np.all(t1[:3] == 3.0) and t1[3] == 0.0
    # without speeds given every clock runs at 1, and changes made by the batch still count inside it
    _, plain = a2.a2cid_plan_batch(n, u, v, 1.0, eta, np.zeros(n), b)
    assert plain["b_pre_i"][0] == bcoef(0.5) and plain["b_pre_i"][1] == bcoef(2.5 * 0.4)
    for bad in (-1.0, float("nan"), float("inf")):
        wrong = ops.copy()
        wrong["clock_rate"][2] = bad
        with pytest.raises(a2.A2cidError):
            a2.a2cid_plan_batch(n, u, v, 1.0, eta, np.zeros(n), binding.Batch(wrong, [0, 1, 2, 3, 4, 5]))
    with pytest.raises(a2.A2cidError):
        a2.a2cid_plan_batch(n, u, v, 1.0, eta, np.zeros(n), b, clock_rates=[1.0, 0.0, 1.0, 1.0])


def test_fifo_scheduler_rejects_bad_parameters():
    u, v = _uv(graph.ring(4))
    for kw in (dict(comm_per_grad=-1.0, comm_time=0.0, jitter=0.0), dict(comm_per_grad=1.0, comm_time=-0.1, jitter=0.0),
               dict(comm_per_grad=1.0, comm_time=0.0, jitter=1.0), dict(comm_per_grad=float("nan"), comm_time=0.0, jitter=0.0)):
        with pytest.raises(a2.A2cidError) as e:
            a2.Scheduler(4, u, v, 1.0, 1.0, 1, fifo=kw)
        assert e.value.code == binding.EINVAL


def test_engine_entry_points_fail_cleanly_without_touching_memory():
    # argument checks come before any GPU call, so these run on a machine without a GPU
    lib = a2.load()
    g = binding._GraphArg([0, 1], [1, 2], 1.0)
    h = C.c_void_p()
    for buf, code in [(binding.a2cid_buffers(0x1004, 0x2000, 8, None), binding.EALIGN),
                      (binding.a2cid_buffers(0x1000, 0x2000, 6, None), binding.EINVAL),       # ld < d
                      (binding.a2cid_buffers(0x1000, 0x2000, 10, None), binding.EALIGN),      # ld % 4 != 0
                      (binding.a2cid_buffers(0x1000, 0x1000, 8, None), binding.EINVAL),       # x == xt
                      (binding.a2cid_buffers(0, 0x2000, 8, None), binding.EINVAL)]:
        assert lib.a2cid_create(C.byref(h), 3, 8, C.byref(g.struct), 0.5, 0.5, 0.5, C.byref(buf)) == code
        assert h.value is None and len(lib.a2cid_last_error()) > 0
    good = binding.a2cid_buffers(0x1000, 0x2000, 8, None)
    assert lib.a2cid_create(C.byref(h), 3, 0, C.byref(g.struct), 0.5, 0.5, 0.5, C.byref(good)) == binding.EINVAL
    assert lib.a2cid_create(C.byref(h), 3, 8, C.byref(g.struct), -1.0, 0.5, 0.5, C.byref(good)) == binding.EINVAL
    assert lib.a2cid_create(C.byref(h), 3, 8, C.byref(g.struct), 0.5, float("nan"), 0.5, C.byref(good)) == binding.EINVAL
    assert lib.a2cid_create(C.byref(h), 3, 8, None, 0.5, 0.5, 0.5, C.byref(good)) == binding.EINVAL
    assert lib.a2cid_create(C.byref(h), 3, 8, C.byref(g.struct), 0.5, 0.5, 0.5, None) == binding.EINVAL
    assert lib.a2cid_apply_events(None, None) == binding.EINVAL
    assert lib.a2cid_stats(None, 0.0, None) == binding.EINVAL
    assert lib.a2cid_flush(None, 0.0) == binding.EINVAL and lib.a2cid_average(None, 0.0) == binding.EINVAL
    assert lib.a2cid_stats_static(None, 0.0, None) == binding.EINVAL
    assert lib.a2cid_inplace_probe(None, 2, 8, None) == binding.EINVAL
    assert lib.a2cid_set_walk_occupancy(None, 4) == binding.EINVAL
    assert lib.a2cid_set_resident_group(None, 8, 1) == binding.EINVAL
    assert lib.a2cid_set_clock_rates(None, None) == binding.EINVAL and lib.a2cid_get_clock_rates(None, None) == binding.EINVAL
    assert lib.a2cid_profile_read_stats(None, None, None) == binding.EINVAL
    assert lib.a2cid_stream_probe(None, None, 16, None) == binding.EINVAL
    assert lib.a2cid_stream_probe(0x1000, 0x2000, 18, None) == binding.EINVAL
    assert lib.a2cid_stream_probe(0x1004, 0x2000, 16, None) == binding.EALIGN
    lib.a2cid_destroy(None)
    lib.a2cid_sched_destroy(None)


# ---- chain programme (order of application and placement of the workers' columns) ------------------

def _run_chain_programme(n, ops, steps, slots):
    """Executes the programme symbolically with a version counter per worker: every read must find the worker's
    current version where the step says it is, a slot or the registers never hold two things, and memory must be
    complete at the end.  Returns the bytes per column that the programme moves."""
    m = len(ops)
    ends = [([int(o["i"]), int(o["j"])] if o["kind"] == binding.KIND_GOSSIP else [int(o["i"])]) for o in ops]
    version = [0] * n
    in_memory = [0] * n
    carry, parked = None, [None] * slots
    applied, seen, moved = [], {}, 0.0
    for st in steps:
        if st["op"] < 0:                                                  # spill
            slot = int(st["src_i"]) - binding.LOC_SLOT0
            w = int(st["row_i"])
            assert 0 <= slot < slots and parked[slot] == (w, version[w]), ("spill", st, parked)
            in_memory[w] = version[w]
            parked[slot] = None
            moved += 8
            continue
        k = int(st["op"])
        ws = [int(st["row_i"])] + ([int(st["row_j"])] if ops[k]["kind"] == binding.KIND_GOSSIP else [])
        assert sorted(ws) == sorted(ends[k]), (k, ws, ends[k])
        applied.append(k)
        for w in ws:                                                      # every worker sees its operations in order
            assert seen.get(w, -1) < k
            seen[w] = k
        srcs = [int(st["src_i"]), int(st["src_j"])][:len(ws)]
        dsts = [int(st["dst_i"]), int(st["dst_j"])][:len(ws)]
        assert srcs[1:] != [binding.LOC_CARRY]                            # the carried worker is always row_i
        for w, src in zip(ws, srcs):
            if src == binding.LOC_MEMORY:
                assert in_memory[w] == version[w], ("stale memory", k, w)
                moved += 8
            elif src == binding.LOC_CARRY:
                assert carry == (w, version[w]), ("stale registers", k, w, carry)
            else:
                assert 0 <= src - binding.LOC_SLOT0 < slots and parked[src - binding.LOC_SLOT0] == (w, version[w]), k
        if ops[k]["kind"] == binding.KIND_GRADIENT:
            moved += (4 if ops[k]["xi"] else 0) + (4 if ops[k]["c"] and ops[k]["gscale"] != 0 else 0) + \
                     (4 if ops[k]["h"] and ops[k]["gscale"] != 0 else 0)
        for w in ws:
            version[w] += 1
        for w, src, dst in zip(ws, srcs, dsts):                           # a slot that is left becomes free
            if src >= binding.LOC_SLOT0 and dst != src:
                parked[src - binding.LOC_SLOT0] = None
        carry = None
        for w, dst in zip(ws, dsts):
            if dst == binding.LOC_MEMORY:
                in_memory[w] = version[w]
                moved += 8
            elif dst == binding.LOC_CARRY:
                assert carry is None, ("two workers in the registers", k)
                carry = (w, version[w])
            else:
                slot = dst - binding.LOC_SLOT0
                assert 0 <= slot < slots and (parked[slot] is None or parked[slot][0] == w), ("slot busy", k, parked)
                parked[slot] = (w, version[w])
    assert carry is None and all(p is None for p in parked)
    assert sorted(applied) == list(range(m))                              # every operation exactly once
    assert in_memory == version                                           # memory is complete when the launch ends
    return moved


def _random_ops(rng, n, m, p_grad):
    ops = np.zeros(m, binding.OP_DTYPE)
    for k in range(m):
        if rng.random() < p_grad or n < 2:
            ops["kind"][k], ops["i"][k], ops["j"][k] = binding.KIND_GRADIENT, rng.integers(n), -1
            ops["xi"][k] = 4096 if rng.random() < 0.7 else 0
            ops["c"][k] = 8192 if rng.random() < 0.5 else 0
            ops["h"][k] = 12288 if rng.random() < 0.4 else 0
            ops["gscale"][k] = 1.0 if rng.random() < 0.8 else 0.0
        else:
            i, j = rng.choice(n, 2, replace=False)
            ops["kind"][k], ops["i"][k], ops["j"][k] = binding.KIND_GOSSIP, i, j
    return ops


@pytest.mark.parametrize("n,m,p_grad,seed", [(2, 50, 0.3, 0), (3, 200, 0.0, 1), (5, 300, 0.5, 2), (64, 1024, 0.15, 3),
                                             (64, 5000, 1.0, 4), (1024, 3000, 0.2, 5), (1, 10, 1.0, 6),
                                             (8, 2000, 0.1, 7)])
@pytest.mark.parametrize("slots", [0, 1, 2, 3, 16])
def test_chain_programme_reads_current_values_and_completes_memory(n, m, p_grad, seed, slots):
    ops = _random_ops(np.random.default_rng(seed), n, m, p_grad)
    steps, per_col = binding.a2cid_plan_chain(n, binding.Batch(ops, [0, m]), slots)
    assert len(steps) <= 3 * m + slots
    assert _run_chain_programme(n, ops, steps, slots) == per_col


@pytest.mark.parametrize("topo,n,edge_rate,limits", [("ring", 64, 2.0, (16.5, 10.5)), ("exponential", 64, 1.0, (20.0, 16.0)),
                                                     ("complete", 64, 0.56, (21.0, 17.0))])
def test_chain_programme_on_scheduler_batches(topo, n, edge_rate, limits):
    """On the paper's topologies the programme moves far fewer bytes than one pass per event (about 30 per column
    and event); the limits guard the greedy order and the parking rule against regressions."""
    edges = getattr(graph, topo)(n)
    u, v = _uv(edges)
    s = binding.Scheduler(n, u, v, edge_rate, 1.0, 11)
    for size in (1, 7, 1024, 4096):
        b = s.next(size)
        for slots, limit in zip((0, 2), limits):
            steps, per_col = binding.a2cid_plan_chain(n, b, slots)
            assert _run_chain_programme(n, b.ops, steps, slots) == per_col
            if size >= 1024:
                assert per_col / size <= limit, (topo, size, slots, per_col / size)
    s.close()


def test_chain_programme_without_slots_carries_whenever_neighbours_share_a_worker():
    ops = _random_ops(np.random.default_rng(9), 16, 800, 0.2)
    steps, _ = binding.a2cid_plan_chain(16, binding.Batch(ops, [0, 800]), 0)
    assert len(steps) == 800 and (steps["op"] >= 0).all()
    for p, q in zip(steps[:-1], steps[1:]):
        pw = {int(p["row_i"]), int(p["row_j"])} - {-1}
        qw = {int(q["row_i"]), int(q["row_j"])} - {-1}
        carried = binding.LOC_CARRY in (p["dst_i"], p["dst_j"])
        assert carried == bool(pw & qw) and carried == (q["src_i"] == binding.LOC_CARRY)


def test_chain_programme_rejects_malformed_batches_and_accepts_empty_ones():
    empty = binding.Batch(np.zeros(0, binding.OP_DTYPE), [0])
    steps, per_col = binding.a2cid_plan_chain(4, empty)
    assert len(steps) == 0 and per_col == 0.0
    for field, value in (("i", 4), ("i", -1), ("j", 9), ("kind", 7)):
        ops = _random_ops(np.random.default_rng(0), 4, 20, 0.0)
        ops[field][11] = value
        with pytest.raises(a2.A2cidError) as e:
            binding.a2cid_plan_chain(4, binding.Batch(ops, [0, 20]))
        assert e.value.code == binding.EINVAL
    ops = _random_ops(np.random.default_rng(0), 4, 20, 0.0)
    ops["j"][3] = ops["i"][3]                                             # a worker cannot gossip with itself
    with pytest.raises(a2.A2cidError):
        binding.a2cid_plan_chain(4, binding.Batch(ops, [0, 20]))
    with pytest.raises(a2.A2cidError):
        binding.a2cid_plan_chain(4, binding.Batch(ops, [0, 20]), lds_slots=17)


def test_chain_programme_on_arbitrary_small_batches():
    """Property test: whatever the batch, the programme is executable and leaves memory complete."""
    hyp = pytest.importorskip("hypothesis")
    from hypothesis import strategies as st

    @st.composite
    def batches(draw):
        n = draw(st.integers(1, 9))
        m = draw(st.integers(0, 40))
        ops = np.zeros(m, binding.OP_DTYPE)
        for k in range(m):
            i = draw(st.integers(0, n - 1))
            if n == 1 or draw(st.booleans()):
                ops["kind"][k], ops["i"][k], ops["j"][k] = binding.KIND_GRADIENT, i, -1
                ops["xi"][k] = draw(st.sampled_from([0, 4096]))
            else:
                j = draw(st.integers(0, n - 2))
                ops["kind"][k], ops["i"][k], ops["j"][k] = binding.KIND_GOSSIP, i, j + (j >= i)
        return n, ops, draw(st.integers(0, 6))

    @hyp.settings(max_examples=300, deadline=None)
    @hyp.given(batches())
    def check(case):
        n, ops, slots = case
        steps, per_col = binding.a2cid_plan_chain(n, binding.Batch(ops, [0, len(ops)]), slots)
        assert _run_chain_programme(n, ops, steps, slots) == per_col

    check()


# ---- the resident kernel's programmes ---------------------------------------------------------------------------

def _f32_bits(v):
    return int(np.float32(v).view(np.uint32))


def _run_resident_launch(n, batch, coef, plan, first_op, trailing):
    """Walks the W programmes of one launch the way the kernel does and checks them against the batch: returns the
    set of operations the launch applies.  Levels are executed in lock step (every wave passes the same number of
    barriers); within a level the rows touched by all waves must be disjoint; per worker the operations must come
    in batch order; every operation carries its own rows, coefficients and inputs; a gradient operation's inputs are
    the ones its wave was told to request by its previous gradient operation (or by its first slot)."""
    W, cols, slots = plan["waves"], plan["cols"], plan["slots"]
    per_wave = slots.shape[1]
    assert per_wave == (256 if W >= 16 else 512)
    row_bytes = 512 * cols
    rows = [int(r) for r in plan["rows"]]
    assert len(set(rows)) == len(rows) and all(0 <= r < n for r in rows)
    ops = batch.ops
    level_of = np.zeros(len(ops), np.int64)
    for l in range(len(batch.level_off) - 1):
        level_of[batch.level_off[l]:batch.level_off[l + 1]] = l
    gops = [int(g) for g in plan["gradient_ops"]]
    # per wave: list of levels, each a list of (kind, op index)
    per_wave_levels, requested = [], []
    applied = {}
    for w in range(W):
        prog = slots[w]
        pos, levels = 0, []
        first = prog[0]
        pending = None                                      # (ordinal, xi) the wave has been told to request
        if first["x"] < binding.RES_JUMP or first["x"] == binding.RES_END:
            if first["y"] != binding.RES_NONE:
                pending = (int(first["y"]), int(first["z"]) | int(first["w"]) << 32)
        seen_end = False
        while not seen_end:
            ctl = int(prog[pos]["x"])
            if ctl == binding.RES_END:
                seen_end = True
                break
            if ctl == binding.RES_JUMP:
                pos = (pos // 64 + 1) * 64                  # the next set
                assert pos < per_wave
                continue
            assert ctl < binding.RES_JUMP
            n_gos, n_grad = ctl & 255, ctl >> 8
            need = 1 + n_gos * (2 if trailing else 1) + 2 * n_grad
            assert pos % 64 + need <= 63, "a level straddles a set (or leaves no room for the next control slot)"
            pos += 1
            this = []
            for _ in range(n_gos):
                sl = prog[pos]
                ri, rj = int(sl["x"]), int(sl["y"])
                assert ri % row_bytes == 0 and rj % row_bytes == 0
                wi, wj = rows[ri // row_bytes], rows[rj // row_bytes]
                this.append(("gossip", wi, wj, int(sl["z"]), int(sl["w"]),
                             (int(prog[pos + 1]["x"]), int(prog[pos + 1]["y"])) if trailing else (0, 0)))
                pos += 2 if trailing else 1
            for _ in range(n_grad):
                sl, sl2 = prog[pos], prog[pos + 1]
                ri = int(sl["x"])
                assert ri % row_bytes == 0
                assert pending is not None, "a gradient operation whose inputs nobody requested"
                this.append(("gradient", rows[ri // row_bytes], pending, int(sl["y"]), int(sl["z"]), int(sl["w"]), int(sl2["y"])))
                pending = None if sl2["x"] == binding.RES_NONE else (int(sl2["x"]), int(sl2["z"]) | int(sl2["w"]) << 32)
                pos += 2
            levels.append(this)
        assert pending is None, "a requested gradient input that no operation uses"
        per_wave_levels.append(levels)
    n_levels = len(per_wave_levels[0])
    assert all(len(lv) == n_levels for lv in per_wave_levels), "waves pass different numbers of barriers"
    last_op_of_worker = {}
    # which operation is it?  match by (workers, level order): walk the batch from first_op in order per worker
    next_of_worker = {}
    for k in range(first_op, len(ops)):
        for wkr in ([int(ops["i"][k]), int(ops["j"][k])] if ops["kind"][k] == binding.KIND_GOSSIP else [int(ops["i"][k])]):
            next_of_worker.setdefault(wkr, []).append(k)
    cursor = {wkr: 0 for wkr in next_of_worker}
    for l in range(n_levels):
        touched = set()
        for w in range(W):
            for rec in per_wave_levels[w][l]:
                ws = [rec[1], rec[2]] if rec[0] == "gossip" else [rec[1]]
                assert not (touched & set(ws)), "two operations of a level share a worker"
                touched |= set(ws)
                # the operation must be the next one of each of its workers
                ks = {next_of_worker[wkr][cursor[wkr]] for wkr in ws}
                assert len(ks) == 1, ("not the next operation of both workers", rec)
                k = ks.pop()
                for wkr in ws:
                    cursor[wkr] += 1
                assert k not in applied
                applied[k] = (l, w)
                op, cf = ops[k], coef[k]
                if rec[0] == "gossip":
                    assert op["kind"] == binding.KIND_GOSSIP and (rec[1], rec[2]) == (int(op["i"]), int(op["j"]))
                    assert (rec[3], rec[4]) == (_f32_bits(cf["b_pre_i"]), _f32_bits(cf["b_pre_j"]))
                    if trailing:
                        assert rec[5] == (_f32_bits(cf["b_post_i"]), _f32_bits(cf["b_post_j"]))
                else:
                    assert op["kind"] == binding.KIND_GRADIENT and rec[1] == int(op["i"])
                    ordinal, xi = rec[2]
                    assert gops[ordinal] == k, "the requested inputs belong to another event"
                    assert xi == (int(op["xi"]) if op["xi"] else 1)
                    assert (rec[3], rec[4], rec[5]) == (_f32_bits(cf["b_pre_i"]), _f32_bits(op["gamma"]), _f32_bits(op["gscale"]))
                    if trailing:
                        assert rec[6] == _f32_bits(cf["b_post_i"])
    ks = sorted(applied)
    assert ks == list(range(first_op, plan["next_op"])), "the launch must apply a contiguous range of the batch"
    assert sorted(set(rows)) == sorted({int(x) for k in ks for x in
                                        ([ops["i"][k], ops["j"][k]] if ops["kind"][k] == binding.KIND_GOSSIP else [ops["i"][k]])})
    assert sorted(gops) == [k for k in ks if ops["kind"][k] == binding.KIND_GRADIENT]
    return ks


def _resident_plans_cover(n, batch, coef, waves, cols):
    trailing = bool(((coef["b_post_i"] != 0) | (coef["b_post_j"] != 0)).any())
    k, launches = 0, 0
    while k < len(batch.ops):
        plan = binding.a2cid_plan_resident(n, batch, coef, first_op=k, waves=waves, cols=cols)
        ks = _run_resident_launch(n, batch, coef, plan, k, trailing)
        assert ks and plan["next_op"] > k
        k = plan["next_op"]
        launches += 1
    return launches


@pytest.mark.parametrize("topo,n,edge_rate", [("ring", 64, 2.0), ("exponential", 64, 1.0), ("complete", 64, 0.56),
                                              ("ring", 16, 1.0), ("complete", 4, 1.0), ("ring", 320, 1.0)])
@pytest.mark.parametrize("waves,cols", [(0, 1), (1, 1), (2, 4), (8, 1), (16, 2)])
def test_resident_programmes_on_scheduler_batches(topo, n, edge_rate, waves, cols):
    edges = getattr(graph, topo)(n)
    u, v = _uv(edges)
    s = binding.Scheduler(n, u, v, edge_rate, 1.0, 5)
    t = np.zeros(n)
    for size, sync in ((1, False), (300, False), (4096, False), (1024, True)):   # a trailing mix only in the last one
        b = s.next(size)
        b.ops["gamma"], b.ops["gscale"] = 0.1, 1.0
        grad = b.ops["kind"] == binding.KIND_GRADIENT
        b.ops["xi"][grad] = 4096 * (1 + np.arange(int(grad.sum())))        # distinct, 16-byte aligned stand-ins
        if sync:
            b.t_sync = float(b.ops["t"].max()) + 0.5
        t, coef = binding.a2cid_plan_batch(n, u, v, edge_rate, 0.7, t, b)
        launches = _resident_plans_cover(n, b, coef, waves, cols)
        if size <= 300:
            assert launches <= 2
    s.close()


def test_resident_shape_follows_the_operations_per_level():
    for topo, n, rate, want in (("ring", 64, 2.0, (16, 2)), ("exponential", 64, 1.0, (8, 1)), ("ring", 16, 1.0, (4, 2))):
        u, v = _uv(getattr(graph, topo)(n))
        s = binding.Scheduler(n, u, v, rate, 1.0, 5)
        b = s.next(1024)
        _, coef = binding.a2cid_plan_batch(n, u, v, rate, 0.5, np.zeros(n), b)
        plan = binding.a2cid_plan_resident(n, b, coef)
        assert (plan["waves"], plan["cols"]) == want
        s.close()


def test_resident_programme_of_wide_levels_is_cut_into_parts():
    """A level with more operations than a wave may hold between two control slots (31) is applied in parts."""
    n = 320
    ops = np.zeros(160, binding.OP_DTYPE)
    ops["kind"], ops["i"], ops["j"] = binding.KIND_GOSSIP, 2 * np.arange(160), 2 * np.arange(160) + 1
    ops["t"] = 1.0
    b = binding.Batch(ops, [0, 160])
    u, v = list(range(0, 320, 2)), list(range(1, 320, 2))
    _, coef = binding.a2cid_plan_batch(n, u, v, 1.0, 0.5, np.zeros(n), b)
    for waves in (1, 2, 16):
        plan = binding.a2cid_plan_resident(n, b, coef, waves=waves, cols=1)
        assert _run_resident_launch(n, b, coef, plan, 0, False) == list(range(160))
        prog, pos, levels = plan["slots"][0], 0, 0
        while prog[pos]["x"] != binding.RES_END:
            ctl = int(prog[pos]["x"])
            if ctl == binding.RES_JUMP:
                pos = (pos // 64 + 1) * 64
            else:
                levels += 1
                pos += 1 + (ctl & 255) + 2 * (ctl >> 8)
        assert levels == -(-160 // (31 * waves))


def test_resident_planner_rejects_malformed_input():
    ops = _random_ops(np.random.default_rng(0), 4, 20, 0.3)
    coef = np.zeros(20, binding.COEF_DTYPE)
    good = binding.Batch(ops, [0, 20])
    for kwargs in ({"waves": 3}, {"waves": 8, "cols": 3}, {"first_op": 21}, {"first_op": -1}):
        with pytest.raises(a2.A2cidError):
            binding.a2cid_plan_resident(4, good, coef, **kwargs)
    bad = ops.copy()
    bad["i"][5] = 4
    with pytest.raises(a2.A2cidError):
        binding.a2cid_plan_resident(4, binding.Batch(bad, [0, 20]), coef)


def test_resident_programme_checker_notices_planted_mistakes():
    """The checker above is only worth something if a wrong programme fails it."""
    n = 16
    u, v = _uv(graph.ring(n))
    s = binding.Scheduler(n, u, v, 1.0, 1.0, 3)
    b = s.next(400)
    b.ops["gamma"], b.ops["gscale"] = 0.1, 1.0
    grad = b.ops["kind"] == binding.KIND_GRADIENT
    b.ops["xi"][grad] = 4096 * (1 + np.arange(int(grad.sum())))
    _, coef = binding.a2cid_plan_batch(n, u, v, 1.0, 0.7, np.zeros(n), b)
    good = binding.a2cid_plan_resident(n, b, coef, waves=4, cols=2)
    _run_resident_launch(n, b, coef, good, 0, False)

    def first_slot(kind_wanted):
        """(wave, position) of the first gossip / gradient operation slot of wave 1's programme."""
        prog, pos = good["slots"][1], 0
        while True:
            ctl = int(prog[pos]["x"])
            assert ctl != binding.RES_END
            if ctl == binding.RES_JUMP:
                pos = (pos // 64 + 1) * 64
                continue
            n_gos, n_grad = ctl & 255, ctl >> 8
            if kind_wanted == "gossip" and n_gos:
                return pos + 1
            if kind_wanted == "gradient" and n_grad:
                return pos + 1 + n_gos
            pos += 1 + n_gos + 2 * n_grad

    def mutated(change):
        plan = dict(good)
        plan["slots"] = good["slots"].copy()
        change(plan["slots"])
        return plan

    g, d = first_slot("gossip"), first_slot("gradient")
    mistakes = {
        "wrong row": lambda sl: sl[1].__setitem__(g, (sl[1][g]["x"], sl[1][g]["x"] ^ 1024, sl[1][g]["z"], sl[1][g]["w"])),
        "wrong coefficient": lambda sl: sl[1].__setitem__(g, (sl[1][g]["x"], sl[1][g]["y"], sl[1][g]["z"] ^ 1, sl[1][g]["w"])),
        "wrong step size": lambda sl: sl[1].__setitem__(d, (sl[1][d]["x"], sl[1][d]["y"], sl[1][d]["z"] ^ 1, sl[1][d]["w"])),
        "wrong next input": lambda sl: sl[1].__setitem__(d + 1, (sl[1][d + 1]["x"] ^ 1, sl[1][d + 1]["y"], sl[1][d + 1]["z"], sl[1][d + 1]["w"])),
        "missing barrier": lambda sl: sl[2].__setitem__(0, (binding.RES_END, sl[2][0]["y"], 0, 0)),
    }
    for what, change in mistakes.items():
        with pytest.raises((AssertionError, IndexError, KeyError)):
            _run_resident_launch(n, b, coef, mutated(change), 0, False)
    s.close()


def test_resident_programmes_on_arbitrary_small_batches():
    """Property test: whatever the batch and the launch shape, the launches together apply every operation once, in an
    order the checker accepts."""
    hyp = pytest.importorskip("hypothesis")
    from hypothesis import strategies as st

    @st.composite
    def cases(draw):
        n = draw(st.integers(2, 9))
        m = draw(st.integers(1, 60))
        rng = np.random.default_rng(draw(st.integers(0, 2 ** 20)))
        ops = _random_ops(rng, n, m, draw(st.sampled_from([0.0, 0.3, 1.0])))
        ops["gamma"], ops["t"] = 0.1, np.sort(rng.uniform(0.0, 5.0, m))
        ops["xi"] = np.where(ops["kind"] == binding.KIND_GRADIENT, 4096 * (1 + np.arange(m)), 0)
        ops["c"] = ops["h"] = 0
        # levels: greedy, as the scheduler packs them
        level, last = np.zeros(m, np.int64), {}
        for k in range(m):
            ws = [int(ops["i"][k])] + ([int(ops["j"][k])] if ops["kind"][k] == binding.KIND_GOSSIP else [])
            level[k] = 1 + max([last.get(w, -1) for w in ws])
            for w in ws:
                last[w] = level[k]
        order = np.argsort(level, kind="stable")
        ops = ops[order]
        off = np.concatenate([[0], np.cumsum(np.bincount(level))])
        sync = draw(st.booleans())
        return n, ops, off, sync, draw(st.sampled_from([1, 2, 4, 8, 16])), draw(st.sampled_from([1, 2, 4]))

    @hyp.settings(max_examples=150, deadline=None)
    @hyp.given(cases())
    def check(case):
        n, ops, off, sync, waves, cols = case
        if waves == 1:
            cols = 1
        b = binding.Batch(ops, off, t_sync=6.0 if sync else float("nan"))
        u, v = _uv(graph.complete(n))
        _, coef = binding.a2cid_plan_batch(n, u, v, 1.0, 0.7, np.zeros(n), b)
        _resident_plans_cover(n, b, coef, waves, cols)

    check()


# ---- the register-file kernel's programme ------------------------------------------------------------------------

REG_ZERO_ONE = 0x7000                   # stand-in for the device address of the constants 0.0 and 1.0


def _run_register_launch(n, batch, coef, plan, first_op, max_slots, full=False):
    """Interprets one launch the way regfile_kernel does and checks it against the batch.  The programme starts with
    the request blocks of chunks 0 and 1 (8 gradient events to a chunk; set of registers = chunk % 2); a switch block
    (first slot of a block) precedes the first event of every later chunk: the kernel requests its pointers into the
    set just used up and turns to the other set; nothing else of a request block (nor, with centres and curvatures,
    of the block after it) is executed.  Returns the indices of the operations applied, in order."""
    ops, slots, gops = batch.ops, plan["slots"], [int(k) for k in plan["gradient_ops"]]
    B, K = binding.REG_BLOCK, binding.REG_CHUNK
    per_request = 2 * B if full else B
    assert len(slots) % B == 0 and 0 < len(slots) <= max_slots

    def pointers(at):
        """The three lists of 8 pointers a request block at slot `at` names."""
        def eight(first):
            out = []
            for s in slots[first:first + 4]:
                out += [int(s["x"]) | int(s["y"]) << 32, int(s["z"]) | int(s["w"]) << 32]
            return out
        none = [None] * K
        return eight(at + 1), eight(at + B) if full else none, eight(at + B + 4) if full else none

    def expected(k_op):
        """What the registers must hold for gradient event k_op: (xi, c, h) as the kernel reads them."""
        op = ops[k_op]
        affine = op["gscale"] != 0
        want = (int(op["xi"]) if op["xi"] else REG_ZERO_ONE | 1,
                int(op["c"]) if op["c"] and affine else REG_ZERO_ONE | 1,
                int(op["h"]) if op["h"] and affine else (REG_ZERO_ONE + 4) | 1)
        return want if full else (want[0], None, None)

    for q in (0, 1):                                   # the two first requests
        ctl = slots[q * per_request]
        assert (int(ctl["x"]) >> 8, int(ctl["y"])) == (binding.REG_CONTROL, binding.REG_REQUEST)
    sets = {0: pointers(0), 8: pointers(per_request)}  # set offset -> the pointers it was filled from
    applied, touched = [], 0
    k = first_op                                       # the next operation of the batch
    pending_mix = []                                   # trailing mixes the last operation still owes: (worker, bits)
    sel, q, n_grad, ended = 0, 0, 0, False
    pos = 2 * per_request
    while pos < len(slots) and not ended:
        block, at, pos = slots[pos:pos + B], pos, pos + B
        for j, s in enumerate(block):
            kind, x, y = int(s["x"]) >> 8, int(s["x"]), int(s["y"])
            if kind != binding.REG_MIX:
                assert not pending_mix, "a trailing mix is missing"
            if kind == binding.REG_GOSSIP:
                op, cf = ops[k], coef[k]
                assert op["kind"] == binding.KIND_GOSSIP and (x, y) == (int(op["i"]), int(op["j"]))
                assert (int(s["z"]), int(s["w"])) == (_f32_bits(cf["b_pre_i"]), _f32_bits(cf["b_pre_j"]))
                pending_mix = [(int(op[e]), _f32_bits(cf[b])) for e, b in (("i", "b_post_i"), ("j", "b_post_j")) if cf[b] != 0]
                touched |= 1 << x | 1 << y
                applied.append(k); k += 1
            elif kind == binding.REG_GRADIENT:
                op, cf = ops[k], coef[k]
                assert op["kind"] == binding.KIND_GRADIENT and (x & 255) == int(op["i"])
                assert (y, int(s["z"]), int(s["w"])) == (_f32_bits(cf["b_pre_i"]), _f32_bits(op["gamma"]), _f32_bits(op["gscale"]))
                assert q - sel < K, "more gradient events than a set of inputs holds"
                have = tuple(p[q - sel] for p in sets[sel])
                assert have == expected(k), "the inputs in the registers belong to another event"
                assert gops[n_grad] == k
                q += 1; n_grad += 1
                pending_mix = [(int(op["i"]), _f32_bits(cf["b_post_i"]))] if cf["b_post_i"] != 0 else []
                touched |= 1 << (x & 255)
                applied.append(k); k += 1
            elif kind == binding.REG_MIX:
                assert pending_mix and pending_mix.pop(0) == (x & 255, y), "a trailing mix nobody owes"
            else:
                assert kind == binding.REG_CONTROL and (x & 255) == 0
                if y == binding.REG_SWITCH:
                    assert j == 0, "a switch slot anywhere but at the head of a block is not acted on"
                    sets[sel] = pointers(at)           # the set just used up receives the pointers of this block
                    sel = 8 - sel
                    q = sel
                    if full:
                        pos += B                       # the block of c and h pointers is passed over
                    break                              # and so is the rest of this one
                if y == binding.REG_END:
                    ended = True
                    break
                assert y == 0
    assert ended and not pending_mix, "the programme has no end slot"
    assert pos == len(slots), "blocks after the end"
    assert k == plan["next_op"] and applied == list(range(first_op, k))
    assert gops == [j for j in applied if ops["kind"][j] == binding.KIND_GRADIENT]
    assert touched == plan["touched"]
    return applied


def _register_plans_cover(n, batch, coef, max_slots=8192, full=False):
    k, launches = 0, 0
    while k < len(batch.ops):
        plan = binding.a2cid_plan_registers(n, batch, coef, first_op=k, max_slots=max_slots, full=full,
                                            zero_one=REG_ZERO_ONE)
        assert _run_register_launch(n, batch, coef, plan, k, max_slots, full), "a launch must take at least one operation"
        k = plan["next_op"]
        launches += 1
    return launches


@pytest.mark.parametrize("topo,n,edge_rate", [("ring", 64, 2.0), ("exponential", 64, 1.0), ("complete", 64, 0.56),
                                              ("ring", 16, 1.0), ("complete", 4, 1.0)])
def test_register_programmes_on_scheduler_batches(topo, n, edge_rate):
    u, v = _uv(getattr(graph, topo)(n))
    s = binding.Scheduler(n, u, v, edge_rate, 1.0, 5)
    t = np.zeros(n)
    for size, sync in ((1, False), (300, False), (4096, False), (12000, False), (1024, True)):   # the sync batch last
        b = s.next(size)
        b.ops["gamma"], b.ops["gscale"] = 0.1, 1.0
        grad = b.ops["kind"] == binding.KIND_GRADIENT
        b.ops["xi"][grad] = 4096 * (1 + np.arange(int(grad.sum())))
        if sync:
            b.t_sync = float(b.ops["t"].max()) + 0.5
        t, coef = binding.a2cid_plan_batch(n, u, v, edge_rate, 0.7, t, b)
        launches = _register_plans_cover(n, b, coef)
        assert launches == 1 if size <= 4096 else launches in (2, 3)
        assert _register_plans_cover(n, b, coef, max_slots=64) >= size // 64     # short programmes: many launches
        assert _register_plans_cover(n, b, coef, max_slots=32) >= size // 32
        # with centres and curvatures on some events: request blocks of two blocks
        b.ops["c"][grad] = np.where(np.arange(int(grad.sum())) % 3 == 0, 0, (1 << 40) + 16 * np.arange(int(grad.sum())))
        b.ops["h"][grad] = np.where(np.arange(int(grad.sum())) % 2 == 0, 0, (1 << 41) + 16 * np.arange(int(grad.sum())))
        _register_plans_cover(n, b, coef, full=True)
        _register_plans_cover(n, b, coef, max_slots=48, full=True)
        if grad.any() and size > 1:
            with pytest.raises(a2.A2cidError):                                    # centres need the two-block requests
                binding.a2cid_plan_registers(n, b, coef)
    s.close()


def test_register_programme_of_an_empty_range_and_of_gradient_events_only():
    n = 8
    ops = np.zeros(40, binding.OP_DTYPE)
    ops["kind"], ops["i"], ops["j"], ops["t"] = binding.KIND_GRADIENT, np.arange(40) % n, -1, 1.0 + np.arange(40) // n
    ops["gamma"], ops["xi"] = 0.1, 4096 * (1 + np.arange(40))
    ops["xi"][5] = 0                                                 # an event without xi
    b = binding.Batch(ops, list(range(0, 41, 8)))
    u, v = _uv(graph.ring(n))
    _, coef = binding.a2cid_plan_batch(n, u, v, 1.0, 0.5, np.zeros(n), b)
    plan = binding.a2cid_plan_registers(n, b, coef, zero_one=REG_ZERO_ONE)
    assert _run_register_launch(n, b, coef, plan, 0, 8192) == list(range(40))
    # 40 events in chunks of 8: two first request blocks, then a switch block (requesting chunks 2, 3, 4, 5) before
    # events 8, 16, 24, 32, each block of 8 events in a block of its own, the end slot in the last
    sl = plan["slots"]
    kinds = [int(x) >> 8 for x in sl["x"]]
    heads = [(kinds[at], int(sl["y"][at])) for at in range(0, len(sl), 8)]
    req, sw, ctl = binding.REG_REQUEST, binding.REG_SWITCH, binding.REG_CONTROL
    assert heads == [(ctl, req), (ctl, req), (1, heads[2][1]), (ctl, sw), (1, heads[4][1]), (ctl, sw), (1, heads[6][1]),
                     (ctl, sw), (1, heads[8][1]), (ctl, sw), (1, heads[10][1]), (ctl, binding.REG_END)]
    assert kinds.count(binding.REG_GRADIENT) == 40
    xi_of_chunk_0 = [int(s["x"]) | int(s["y"]) << 32 for s in sl[1:5]] + [int(s["z"]) | int(s["w"]) << 32 for s in sl[1:5]]
    assert sorted(xi_of_chunk_0) == sorted([4096 * (1 + g) for g in range(8) if g != 5] + [REG_ZERO_ONE | 1])
    last_request = 9 * 8                                             # chunk 5: no such events
    assert all(int(s["x"]) == REG_ZERO_ONE | 1 and int(s["z"]) == REG_ZERO_ONE | 1 for s in sl[last_request + 1:last_request + 5])
    empty = binding.a2cid_plan_registers(n, b, coef, first_op=40)
    assert empty["next_op"] == 40 and empty["touched"] == 0 and len(empty["slots"]) == 24
    assert (int(empty["slots"][16]["x"]) >> 8, int(empty["slots"][16]["y"])) == (binding.REG_CONTROL, binding.REG_END)


def test_register_planner_rejects_malformed_input():
    ops = _random_ops(np.random.default_rng(0), 4, 20, 0.3)
    ops["c"] = ops["h"] = 0
    coef = np.zeros(20, binding.COEF_DTYPE)
    good = binding.Batch(ops, [0, 20])
    for kwargs in ({"first_op": 21}, {"first_op": -1}, {"max_slots": 24}, {"max_slots": 36}, {"max_slots": 0},
                   {"max_slots": 40, "full": True}, {"zero_one": 0x1002}):
        with pytest.raises(a2.A2cidError):
            binding.a2cid_plan_registers(4, good, coef, **kwargs)
    binding.a2cid_plan_registers(4, good, coef, max_slots=32)
    binding.a2cid_plan_registers(4, good, coef, max_slots=48, full=True)
    with pytest.raises(a2.A2cidError):
        binding.a2cid_plan_registers(65, good, coef)                 # more workers than registers
    bad = ops.copy()
    bad["i"][5] = 4
    with pytest.raises(a2.A2cidError):
        binding.a2cid_plan_registers(4, binding.Batch(bad, [0, 20]), coef)
    odd = ops.copy()
    odd["xi"][np.flatnonzero(odd["kind"] == binding.KIND_GRADIENT)[0]] = 4097      # bit 0 is the library's own mark
    with pytest.raises(a2.A2cidError):
        binding.a2cid_plan_registers(4, binding.Batch(odd, [0, 20]), coef)


def test_register_programme_checker_notices_planted_mistakes():
    n = 16
    u, v = _uv(graph.ring(n))
    s = binding.Scheduler(n, u, v, 1.0, 1.0, 3)
    b = s.next(400)
    b.ops["gamma"], b.ops["gscale"] = 0.1, 1.0
    grad = b.ops["kind"] == binding.KIND_GRADIENT
    b.ops["xi"][grad] = 4096 * (1 + np.arange(int(grad.sum())))
    b.t_sync = float(b.ops["t"].max()) + 0.5
    _, coef = binding.a2cid_plan_batch(n, u, v, 1.0, 0.7, np.zeros(n), b)
    good = binding.a2cid_plan_registers(n, b, coef, zero_one=REG_ZERO_ONE)
    _run_register_launch(n, b, coef, good, 0, 8192)
    kinds = good["slots"]["x"] >> 8
    ctl = (kinds == binding.REG_CONTROL) & (np.arange(len(kinds)) % 8 == 0)
    g = int(np.flatnonzero(kinds == binding.REG_GOSSIP)[3])
    d = int(np.flatnonzero(kinds == binding.REG_GRADIENT)[9])
    m = int(np.flatnonzero(kinds == binding.REG_MIX)[0])
    sw = int(np.flatnonzero(ctl & (good["slots"]["y"] == binding.REG_SWITCH))[0])
    end = int(np.flatnonzero((kinds == binding.REG_CONTROL) & (good["slots"]["y"] == binding.REG_END))[-1])

    def mutated(change):
        plan = dict(good)
        plan["slots"] = good["slots"].copy()
        change(plan["slots"])
        return plan

    def swap(sl, a, b):
        sl[[a, b]] = sl[[b, a]]

    mistakes = {
        "wrong worker": lambda sl: sl["y"].__setitem__(g, sl["y"][g] ^ 1),
        "wrong coefficient": lambda sl: sl["z"].__setitem__(g, sl["z"][g] ^ 1),
        "wrong step size": lambda sl: sl["z"].__setitem__(d, sl["z"][d] ^ 1),
        "missing switch": lambda sl: sl["y"].__setitem__(sw, 0),
        "wrong pointer in a request": lambda sl: sl["z"].__setitem__(sw + 2, sl["z"][sw + 2] ^ 64),
        "pointers of two events exchanged": lambda sl: swap(sl, 1, 2),
        "dropped trailing mix": lambda sl: sl.__setitem__(m, (binding.REG_CONTROL << 8, 0, 0, 0)),
        "operations exchanged": lambda sl: swap(sl, g, d),
        "no end": lambda sl: sl["y"].__setitem__(end, 0),
    }
    for what, change in mistakes.items():
        with pytest.raises((AssertionError, IndexError, KeyError)):
            _run_register_launch(n, b, coef, mutated(change), 0, 8192)
    s.close()


def test_register_programme_check_refuses_what_the_kernel_could_not_run():
    """The kernel adds worker indices to register numbers and trusts the block structure; the library checks every
    programme before launching it, and this is that check."""
    n = 16
    u, v = _uv(graph.ring(n))
    s = binding.Scheduler(n, u, v, 1.0, 1.0, 3)
    b = s.next(400)
    b.ops["gamma"], b.ops["gscale"] = 0.1, 1.0
    grad = b.ops["kind"] == binding.KIND_GRADIENT
    b.ops["xi"][grad] = 4096 * (1 + np.arange(int(grad.sum())))
    _, coef = binding.a2cid_plan_batch(n, u, v, 1.0, 0.7, np.zeros(n), b)
    for full in (False, True):
        good = binding.a2cid_plan_registers(n, b, coef, full=full)["slots"]
        binding.a2cid_check_registers(n, good, full)
        binding.a2cid_check_registers(64, good, full)
        kinds = good["x"] >> 8
        heads = np.arange(len(good)) % 8 == 0
        g = int(np.flatnonzero(kinds == binding.REG_GOSSIP)[5])
        d = int(np.flatnonzero(kinds == binding.REG_GRADIENT)[3])
        sw = int(np.flatnonzero((kinds == binding.REG_CONTROL) & heads & (good["y"] == binding.REG_SWITCH))[0])
        end = int(np.flatnonzero((kinds == binding.REG_CONTROL) & (good["y"] == binding.REG_END))[-1])
        filler = (binding.REG_CONTROL << 8, 0, 0, 0)

        def bad(change, workers=n):
            sl = good.copy()
            sl = change(sl)
            with pytest.raises(a2.A2cidError):
                binding.a2cid_check_registers(workers, sl, full)

        def put(sl, at, field, value):
            sl[field][at] = value
            return sl

        bad(lambda sl: put(sl, g, "x", n))                                      # worker i out of range
        bad(lambda sl: put(sl, g, "y", 200))                                    # worker j out of range
        bad(lambda sl: put(sl, d, "x", (binding.REG_GRADIENT << 8) | 77))
        bad(lambda sl: sl, workers=int(max(good["x"][kinds == 0].max(), good["y"][kinds == 0].max())))  # n too small
        bad(lambda sl: sl, workers=65)
        bad(lambda sl: put(sl, sw, "y", 0))                                     # the pointers would run as operations
        bad(lambda sl: put(sl, end, "y", 0))                                    # no end
        bad(lambda sl: sl[:-8])                                                 # the end slot's block is gone
        bad(lambda sl: sl[:-3])                                                 # not whole blocks
        bad(lambda sl: np.concatenate([sl, np.array([filler] * 8, binding.SLOT_DTYPE)]))   # blocks after the end
        bad(lambda sl: put(sl, 0, "y", binding.REG_SWITCH))                     # the first requests are missing
        bad(lambda sl: put(sl, g, "x", 9 << 8))                                 # no such kind
        moved = good.copy()                                                     # a switch slot away from a block's head
        moved[[sw, sw + 1]] = moved[[sw + 1, sw]]
        bad(lambda sl: moved)
    bad_full = binding.a2cid_plan_registers(n, b, coef, full=False)["slots"]
    with pytest.raises(a2.A2cidError):                                          # read with the other block layout
        binding.a2cid_check_registers(n, bad_full, True)
    # nine gradient events in one chunk: index 8 of a set of 8 registers
    ops = np.zeros(9, binding.OP_DTYPE)
    ops["kind"], ops["i"], ops["j"], ops["t"], ops["gamma"] = binding.KIND_GRADIENT, np.arange(9), -1, 1.0, 0.1
    nine = binding.Batch(ops, [0, 9])
    _, c9 = binding.a2cid_plan_batch(n, u, v, 1.0, 0.7, np.zeros(n), nine)
    sl = binding.a2cid_plan_registers(n, nine, c9)["slots"]
    binding.a2cid_check_registers(n, sl)
    assert len(sl) == 40                   # two requests, eight events, the switch block, the ninth event and the end
    merged = np.concatenate([sl[:24], sl[32:]])                                 # ... without the switch block
    with pytest.raises(a2.A2cidError):
        binding.a2cid_check_registers(n, merged)
    s.close()


def test_register_programmes_on_arbitrary_small_batches():
    """Property test: whatever the batch and the programme length, the launches together apply every operation once,
    in the batch's order, with the inputs of the right gradient event in the registers."""
    hyp = pytest.importorskip("hypothesis")
    from hypothesis import strategies as st

    @st.composite
    def cases(draw):
        n = draw(st.integers(2, 9))
        m = draw(st.integers(1, 120))
        rng = np.random.default_rng(draw(st.integers(0, 2 ** 20)))
        ops = _random_ops(rng, n, m, draw(st.sampled_from([0.0, 0.3, 0.8, 1.0])))
        ops["gamma"], ops["t"] = 0.1, np.sort(rng.uniform(0.0, 5.0, m))
        grad = ops["kind"] == binding.KIND_GRADIENT
        for name, base in (("xi", 1 << 20), ("c", 2 << 20), ("h", 3 << 20)):     # distinct addresses where the event has the input
            ops[name] = np.where(grad & (ops[name] != 0), base + 16 * np.arange(m), 0)
        full = draw(st.booleans())
        if not full:
            ops["c"] = ops["h"] = 0
        return n, ops, draw(st.booleans()), draw(st.sampled_from([48, 56, 64, 8192])), full

    @hyp.settings(max_examples=200, deadline=None)
    @hyp.given(cases())
    def check(case):
        n, ops, sync, max_slots, full = case
        b = binding.Batch(ops, list(range(len(ops) + 1)), t_sync=6.0 if sync else float("nan"))   # one operation per level
        u, v = _uv(graph.complete(n))
        _, coef = binding.a2cid_plan_batch(n, u, v, 1.0, 0.7, np.zeros(n), b)
        _register_plans_cover(n, b, coef, max_slots, full)

    check()
