"""Full-length parity runs of the five configurations (not collected by pytest: minutes of GPU time each).

    python tests/full_stream_parity.py C1 C2 C3 C4 C4-baseline C5 [--events N] [--out gpurun_out/full_stream.json]

For each configuration the engine runs the WHOLE event stream at full size with freshly generated per-event
noise, while the CPU oracle follows 4096 sampled columns (first 1024, last 1024, seeded random ones) through the
same stream; the two are compared every `--check-every` events (state on the sampled columns, time stamps) and at
the end (after a flush).  Observables are recorded along the way (consensus-distance trace).
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

import parity_util as pu                                  # noqa: E402
from paper_2306_08289_amd import workloads as wl          # noqa: E402


def run(name, events, check_every, batch, mode=3, order=0, fifo=None):
    cfg = wl.CONFIGS[name]
    events = events or cfg.events
    cols = pu.sample_columns(cfg.d, 4096, seed=7)
    print(f"[{name}] n={cfg.n} d={cfg.d} events={events} sampled columns={len(cols)}", flush=True)
    t0 = time.perf_counter()
    o = pu.OracleStream(cfg, cols, order=order, fifo=fifo)
    ev = o.generate(events)
    print(f"[{name}] oracle stream generated in {time.perf_counter() - t0:.1f} s, T = {ev.t[-1]:.3f}", flush=True)
    w = wl.Workload(cfg, batch_events=batch, fifo=fifo)
    w.engine.set_tuning(1, 0, 256, mode)
    w.engine.set_order(order)
    rec = {"config": name, "mode": mode, "order": order, "fifo": fifo, "n": cfg.n, "d": cfg.d, "events": events, "eta": w.eta, "alpha_tilde": w.alpha_tilde,
           "checks": [], "trace": []}
    gpu_s = 0.0
    done = 0
    while done < events:
        upto = min(events, done + check_every)
        t1 = time.perf_counter()
        w.run(upto - done)
        w.engine.synchronize()
        gpu_s += time.perf_counter() - t1
        st = o.advance(upto)
        gx, gxt = w.columns(cols)
        ex, ext = pu.rel_err(gx, st.x), pu.rel_err(gxt, st.xt)
        same_t = bool(np.array_equal(w.engine.times(), st.t))
        t_now = float(ev.t[upto - 1])
        gs = w.engine.stats(t_now)
        rec["checks"].append({"events": upto, "rel_err_x": ex, "rel_err_xt": ext, "times_equal": same_t})
        rec["trace"].append({"events": upto, "t": t_now, "consensus_x": gs["consensus_x"],
                             "consensus_xt": gs["consensus_xt"]})
        print(f"[{name}] {upto:>8} events  rel err x {ex:.2e} xt {ext:.2e}  times equal {same_t}  "
              f"consensus_x {gs['consensus_x']:.6g}  (gpu {gpu_s:.1f} s)", flush=True)
        done = upto
    t_end = float(ev.t[-1]) + 1.0
    w.engine.flush(t_end)
    fx, fxt = w.columns(cols)
    ox, oxt = o.state.flushed(t_end)
    gs = w.engine.stats(t_end)
    rec["final"] = {"rel_err_x": pu.rel_err(fx, ox), "rel_err_xt": pu.rel_err(fxt, oxt),
                    "mean_gap": float(abs(gs["sum_x"].sum() - gs["sum_xt"].sum()) /
                                      max(1e-30, np.abs(gs["sum_x"]).sum())),
                    "gpu_seconds_incl_noise_generation": gpu_s, "wall_seconds": time.perf_counter() - t0}
    rec["max_rel_err"] = max([c["rel_err_x"] for c in rec["checks"]] + [c["rel_err_xt"] for c in rec["checks"]] +
                             [rec["final"]["rel_err_x"], rec["final"]["rel_err_xt"]])
    rec["pass"] = bool(rec["max_rel_err"] <= pu.TOL and all(c["times_equal"] for c in rec["checks"]))
    print(f"[{name}] final: {rec['final']}  max rel err {rec['max_rel_err']:.2e}  PASS={rec['pass']}", flush=True)
    w.close()
    return rec


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("configs", nargs="+")
    ap.add_argument("--events", type=int, default=None)
    ap.add_argument("--check-every", type=int, default=100000)
    ap.add_argument("--batch", type=int, default=1024)
    ap.add_argument("--mode", type=int, default=3,
                    help="event kernel: 0 levels, 1 walk, 2 LDS-resident, 3 chain (default)")
    ap.add_argument("--order", type=int, default=0, help="0: Eq. (1) order (default); 1: Algorithm 1's listing order")
    ap.add_argument("--fifo", type=float, default=None,
                    help="use the first-in-first-out pairing source with this many averagings per gradient step")
    ap.add_argument("--out", default=os.path.join(ROOT, "gpurun_out", "full_stream.json"))
    args = ap.parse_args()
    results = []
    if os.path.exists(args.out):
        results = json.load(open(args.out))
    ok = True
    for name in args.configs:
        fifo = None if args.fifo is None else dict(comm_per_grad=args.fifo, comm_time=0.02, jitter=0.2)
        rec = run(name, args.events, args.check_every, args.batch, args.mode, args.order, fifo)
        results = [r for r in results if (r["config"], r.get("mode", 3), r.get("order", 0), bool(r.get("fifo"))) !=
                   (name, args.mode, args.order, fifo is not None)] + [rec]
        os.makedirs(os.path.dirname(args.out), exist_ok=True)
        json.dump(results, open(args.out, "w"), indent=1)
        ok = ok and rec["pass"]
    sys.exit(0 if ok else 1)


if __name__ == "__main__":
    main()
