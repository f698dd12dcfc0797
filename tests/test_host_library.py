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
@pytest.mark.parametrize("normalize", [False, True])
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
    assert np.array_equal(s.counts(), np.bincount(ref.clock, minlength=n + len(edges)))


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
