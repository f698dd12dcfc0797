"""Pins for the level packing definition: it is a re-ordering that no worker can observe."""
import numpy as np

from oracle import core, graph, levels


def _events(n, edges, seed, m):
    return core.generate_events(n, [e[0] for e in edges], [e[1] for e in edges],
                                np.ones(n), np.ones(len(edges)), seed, m)


def test_levels_are_vertex_disjoint_cover_the_batch_and_keep_worker_order():
    n = 16
    ev = _events(n, graph.exponential(n), 2, 3000)
    batches = levels.pack(ev.kind, ev.i, ev.j, 257)
    seen = []
    for b, batch in enumerate(batches):
        for level in batch:
            touched = set()
            assert level == sorted(level) and len(level) > 0
            for e in level:
                ws = {int(ev.i[e])} | ({int(ev.j[e])} if ev.kind[e] == 1 else set())
                assert not (touched & ws)
                touched |= ws
            assert len(level) <= n
        flat = [e for level in batch for e in level]
        assert sorted(flat) == list(range(b * 257, min(len(ev), (b + 1) * 257)))
        seen += flat
    assert sorted(seen) == list(range(len(ev)))
    # per-worker subsequence in packed order == per-worker subsequence in serial order
    for w in range(n):
        packed = [e for e in seen if ev.i[e] == w or ev.j[e] == w]
        assert packed == sorted(packed)


def test_applying_levels_in_any_inner_order_equals_the_serial_stream_bit_for_bit():
    rng = np.random.default_rng(0)
    n, d = 8, 6
    edges = graph.ring(n)
    ev = _events(n, edges, 5, 600)
    x0 = rng.normal(size=(n, d)); c = rng.normal(size=(n, d))
    kw = dict(gamma=0.1, gscale=1.0)
    c_row = np.where(ev.kind == 0, ev.i, -1)
    serial = core.State(x0, None, 0.3, 0.5, 1.7).apply(ev, c=c, c_row=c_row, **kw)
    order = []
    for batch in levels.pack(ev.kind, ev.i, ev.j, 100):
        for level in batch:
            order += list(rng.permutation(level))
    order = np.array(order)
    perm = core.Events(ev.t[order], ev.kind[order], ev.i[order], ev.j[order])
    packed = core.State(x0, None, 0.3, 0.5, 1.7).apply(perm, c=c, c_row=c_row[order], **kw)
    assert np.array_equal(serial.x, packed.x) and np.array_equal(serial.xt, packed.xt)
    assert np.array_equal(serial.t, packed.t)
