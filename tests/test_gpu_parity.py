"""GPU parity: the HIP path through the C ABI against the CPU oracle, element by element."""
import math

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import parity_util as pu                                        # noqa: E402
from paper_2306_08289_amd import workloads as wl                # noqa: E402
from synth import gen                                           # noqa: E402


def _say(msg):
    print(msg, flush=True)


def test_input_generator_device_equals_host():
    from synth import fill
    for d, seed, domain, row, sigma, mean in [(1, 3, gen.DOMAIN_INIT, 0, 1.0, 0.0),
                                              (4099, 0xA2C1D5, gen.DOMAIN_XI, (1 << 33) + 7, 1e-3, 0.0),
                                              (100003, 5 + (9 << 32), gen.DOMAIN_C, 63, 2.0, 0.5)]:
        _say(f"fill d={d} seed={seed} domain={domain} row={row}")
        t = torch.empty((d + 3) // 4 * 4, dtype=torch.float32, device="cuda:0")
        fill.fill_normal(t[:d], seed, domain, row, sigma, mean)
        torch.cuda.synchronize()
        host = gen.normal(seed, domain, row, np.arange(d), sigma, mean)
        assert np.array_equal(t[:d].cpu().numpy().view(np.uint32), host.view(np.uint32))


def _compare(cfg, n_events, batch_events, cols=None, tuning=None):
    _say(f"parity {cfg.name} n={cfg.n} d={cfg.d} events={n_events} batch={batch_events} tuning={tuning}")
    w = wl.Workload(cfg, batch_events=batch_events)
    if tuning:
        w.engine.set_tuning(*tuning)
    w.run(n_events)
    cols = np.arange(cfg.d) if cols is None else cols
    gx, gxt = w.columns(cols)
    st, ev = pu.oracle_run(cfg, cols, n_events)
    assert np.array_equal(w.engine.times(), st.t)               # time stamps are bit-exact
    ex, ext = pu.rel_err(gx, st.x), pu.rel_err(gxt, st.xt)
    _say(f"  rel err x {ex:.3g} xt {ext:.3g}")
    assert ex <= pu.TOL and ext <= pu.TOL
    if w.ld != cfg.d:                                           # padding columns were never written
        assert torch.isnan(w.x[:, cfg.d:]).all() and torch.isnan(w.xt[:, cfg.d:]).all()
    # observables at a common later time, against the oracle's on the same columns when complete
    t_now = float(ev.t[-1]) + 0.5
    gs = w.engine.stats(t_now)
    if len(cols) == cfg.d:
        os_ = st.stats(t_now)
        for k in ("consensus_x", "consensus_xt"):
            assert math.isclose(gs[k], os_[k], rel_tol=1e-4), (k, gs[k], os_[k])
        l1x = np.abs(st.x).sum(1); l1xt = np.abs(st.xt).sum(1)
        assert np.all(np.abs(gs["sum_x"] - os_["sum_x"]) <= 1e-5 * l1x)
        assert np.all(np.abs(gs["sum_xt"] - os_["sum_xt"]) <= 1e-5 * l1xt)
    # flush, then the same columns once more
    w.engine.flush(t_now)
    fx, fxt = w.columns(cols)
    ox, oxt = st.flushed(t_now)
    assert pu.rel_err(fx, ox) <= pu.TOL and pu.rel_err(fxt, oxt) <= pu.TOL
    assert np.all(w.engine.times() == t_now)
    w.close()
    return w


@pytest.mark.parametrize("name,d,events,batch", [
    ("C1", 1000, 10000, 512),          # config 1 in full
    ("C1", 3, 300, 64),                # d < 4: only the scalar tail path
    ("C1", 4, 300, 64),
    ("C2", 4 * 1024 * 3 + 1027, 3000, 1000),   # several tiles and a ragged tail, noise + centres
    ("C3", 9001, 3000, 1024),
    ("C4", 12345, 4000, 1024),
    ("C4-baseline", 4098, 2000, 700),
    ("C5", 8191, 4000, 1024),
])
def test_small_configs_match_oracle_everywhere(name, d, events, batch):
    _compare(wl.scaled(wl.CONFIGS[name], d=d, events=events), events, batch)


@pytest.mark.parametrize("unroll,nt,threads,walk", [(1, 0, 64, 0), (2, 1, 128, 0), (4, 1, 256, 1), (4, 0, 64, 0),
                                                   (2, 0, 512, 1), (1, 1, 128, 1), (4, 1, 64, 0),
                                                   (1, 0, 1024, 1), (2, 1, 1024, 0)])
def test_launch_shapes_give_the_same_answer(unroll, nt, threads, walk):
    # rows long enough that the engine keeps the requested unroll (it shrinks tiles for short rows)
    cfg = wl.scaled(wl.CONFIGS["C2"], d=2048 * 1024 * 4 * 4 + 517, events=600)
    _compare(cfg, 600, 300, cols=pu.sample_columns(cfg.d, 4096, seed=2), tuning=(unroll, nt, threads, walk))


@pytest.mark.parametrize("name,events,batch", [("C2", 3000, 1024), ("C3", 600, 512), ("C4", 400, 400),
                                               ("C5", 400, 400)])
def test_full_size_configs_on_sampled_columns(name, events, batch):
    cfg = wl.scaled(wl.CONFIGS[name], events=events)
    _compare(cfg, events, batch, cols=pu.sample_columns(cfg.d, 4096, seed=1))
