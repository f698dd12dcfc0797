"""GPU test of a2cid_stats_static, the observables entry point that allocates nothing (its partial sums live in a
fixed array inside the library), against a2cid_stats through the C ABI: same kernels, same state, same time."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from paper_2306_08289_amd import A2cidError, binding            # noqa: E402
from paper_2306_08289_amd import workloads as wl                # noqa: E402


def _say(msg):
    print(msg, flush=True)


def _both(w, t_now):
    """(a2cid_stats result, a2cid_stats_static result as a host array) for the same state and time."""
    ref = w.engine.stats(t_now)
    out = torch.full((2 * w.cfg.n + 2,), float("nan"), dtype=torch.float64, device=w.device)
    w.engine.stats_static(t_now, out)
    w.engine.synchronize()
    return ref, out.cpu().numpy()


def _assert_same(ref, got, n, exact):
    want = np.concatenate([ref["sum_x"], ref["sum_xt"], [ref["consensus_x"], ref["consensus_xt"]]])
    assert np.all(np.isfinite(got))
    if exact:                       # same launch shape, same summation order: the same bits
        assert np.array_equal(got, want), np.abs(got - want).max()
        return
    # fewer workgroups share the fixed scratch: another order of the same fp64 additions
    scale = max(np.abs(want[:2 * n]).max(), 1.0)
    assert np.all(np.abs(got[:2 * n] - want[:2 * n]) <= 1e-11 * scale * n)
    assert np.allclose(got[2 * n:], want[2 * n:], rtol=1e-11, atol=0.0)


def test_static_scratch_observables_equal_a2cid_stats_on_calls_in_a_row():
    # first call: 64 workers, rows long enough that every one of the 2048 workgroups walks several tiles, a ragged
    # tail, mixing pending for every worker
    big = wl.scaled(wl.CONFIGS["C4"], d=2048 * 512 * 4 * 2 + 4 * 777 + 3, events=600)
    _say(f"stats_static first call: n={big.n} d={big.d}")
    wb = wl.Workload(big, batch_events=300)
    wb.run(600)
    ref, got = _both(wb, wb.t_last + 0.37)
    _assert_same(ref, got, big.n, exact=True)
    # second call, smaller input, while the scratch still holds the partial sums of the first
    small = wl.scaled(wl.CONFIGS["C2"], d=5003, events=400)
    _say(f"stats_static second call: n={small.n} d={small.d}")
    ws = wl.Workload(small, batch_events=200)
    ws.run(400)
    ref, got = _both(ws, ws.t_last + 1.5)
    _assert_same(ref, got, small.n, exact=True)
    # and the large one again after the small one, later in time
    ref, got = _both(wb, wb.t_last + 2.0)
    _assert_same(ref, got, big.n, exact=True)
    ws.close()
    wb.close()


def test_static_scratch_observables_with_more_workers_than_full_width_and_beyond_the_limit():
    def ring(n, d):
        return wl.Config(name=f"ring-{n}", n=n, topology="ring", d=d, init_sigma=1.0, gscale=1.0, use_c=True,
                         xi_sigma=0.1, edge_rate=1.0, events=1000, seed=0xA2C1D2 + 91, eta=0.3, alpha_tilde=1.5)
    cfg = ring(binding.STATS_STATIC_MAX_WORKERS, 40000 * 4 + 2)
    _say(f"stats_static at the worker limit: n={cfg.n} d={cfg.d}")
    w = wl.Workload(cfg, batch_events=500)
    w.run(1000)
    ref, got = _both(w, w.t_last + 0.1)
    _assert_same(ref, got, cfg.n, exact=False)
    out = torch.zeros(2 * cfg.n + 4, dtype=torch.float64, device=w.device)
    for what, ptr in (("host pointer", np.zeros(2 * cfg.n + 2).ctypes.data), ("misaligned", out.data_ptr() + 4),
                      ("null", 0)):
        _say(f"stats_static rejects: {what}")
        rc = binding.load().a2cid_stats_static(w.engine._h, w.t_last + 0.2, ptr)
        assert rc in (binding.EINVAL, binding.EALIGN), (what, rc)
    with pytest.raises(A2cidError):                       # a time before a worker's stamp
        w.engine.stats_static(0.0, out[:2 * cfg.n + 2])
    w.close()
    cfg = ring(binding.STATS_STATIC_MAX_WORKERS + 1, 64)
    w = wl.Workload(cfg, batch_events=100)
    out = torch.zeros(2 * cfg.n + 2, dtype=torch.float64, device=w.device)
    with pytest.raises(A2cidError) as e:
        w.engine.stats_static(0.5, out)
    assert e.value.code == binding.EINVAL and "at most" in str(e.value)
    w.close()
