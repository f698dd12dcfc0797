#!/usr/bin/env python3
"""Benchmark of the A2CiD2 hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic events: the scheduler draws
and level-packs `--batch` events, the planner validates them and computes the mixing
coefficients, the event kernel applies them to x and xt, and the observables kernel reads the
state once.  Inputs (state, c_i, gradient-noise pool) are resident in HBM before timing starts;
generating the per-event noise stands in for the gradient computation and is outside the path.

Prints ONE JSON line.  The headline figures (value, roofline) belong to the walk kernel, which
makes one full pass over the touched rows per event, so that its traffic IS the algorithmic byte
count of the method: 32 d per gossip event, 16 d + 4 d per gradient input per gradient event
(+ 8 n d per observables call in `value`).  The kernels that keep workers on the chip between
events -- the chain kernel, the LDS-resident kernel and the register-file kernel, between which the library chooses
by shape -- move fewer bytes for the same events; they are timed on the same steps and reported as separate lines
(`chain_variant`, `resident_variant`, `regfile_variant`: events/s up, HBM GB/s down, with the bytes they move by
construction and the same work priced at one pass per event).  Also: the copy ceiling of the
machine, and the CPU oracle timed on a bounded sample on this machine's host cores.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0     # MI355X published HBM3E bandwidth

# Bytes per launch that crossed the L2 <-> memory-fabric boundary, from two rocprofv3 --pmc runs of this same
# command (FETCH_SIZE, then WRITE_SIZE), each scaled by what the same counter reads for the library's copy probe of
# known size.  NOT a reading of the run that prints the line: `traffic_source` names the committed summary the
# figure comes from.  Only valid for the workload, batch size, kernel and launch shape it names.  The counters sit
# between the L2 and the fabric: bytes served by the 256 MB last-level cache behind it count as traffic here.
MEASURED_TRAFFIC = {
    ("C4", 1024, "walk_kernel"): (7.9190e11, "profiles/bench_C4_hbm_counters.md"),
    ("C4", 1024, "chain_kernel"): (3.2498e11, "profiles/bench_C4_hbm_counters.md"),
    ("C4", 1024, "resident_kernel"): (4.2486e10, "profiles/bench_C4_hbm_counters.md"),
    ("C4", 1024, "regfile_kernel"): (4.2788e10, "profiles/bench_C4_hbm_counters.md"),
    ("C3", 1024, "walk_kernel"): (3.3678e11, "profiles/bench_C3_hbm_counters.md"),
    ("C3", 1024, "chain_kernel"): (7.2111e10, "profiles/bench_C3_hbm_counters.md"),
    ("C3", 1024, "resident_kernel"): (2.6894e10, "profiles/bench_C3_hbm_counters.md"),
    ("C3", 1024, "regfile_kernel"): (2.6515e10, "profiles/bench_C3_hbm_counters.md"),
    ("C5", 1024, "walk_kernel"): (8.2851e11, "profiles/bench_C5_hbm_counters.md"),
    ("C5", 1024, "chain_kernel"): (3.7700e11, "profiles/bench_C5_hbm_counters.md"),
    ("C5", 1024, "resident_kernel"): (3.7917e10, "profiles/bench_C5_hbm_counters.md"),
    ("C5", 1024, "regfile_kernel"): (3.8749e10, "profiles/bench_C5_hbm_counters.md"),
}

# The resident and register-file kernels are bound by instruction issue, not by memory: their roofline is the chip's
# fp32 vector rate.
# Arithmetic of the method per column (one fused multiply-add = 2 flop): a gossip event mixes two workers (a subtraction
# and two fused multiply-adds each), forms m (a subtraction) and applies four fused multiply-adds: 19 flop; a gradient
# event mixes one worker (5), forms g = s (x - c) + xi (3) and applies two fused multiply-adds (4): 12 flop.
# Peak: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz x 2 flop = 78.6 TFLOP/s with one fp32 operation per lane and cycle, twice
# that (the published 157.3 TFLOP/s) only with packed two-wide fp32 instructions, which this build does not emit.
FLOP_PER_COLUMN = {"gossip": 19.0, "gradient": 12.0}
FP32_VECTOR_PEAK_TFLOPS = 157.3
MODE_NAMES = {0: "level_kernel", 1: "walk_kernel", 2: "resident_kernel", 3: "chain_kernel", 4: "regfile_kernel"}
MODE_WHAT = {0: "level_kernel: one launch per level, one full pass over the touched rows per event",
             1: "walk_kernel: one launch per batch, one full pass over the touched rows per event",
             2: "resident_kernel (the library's choice for 65 to 160 workers): every touched row stays in LDS for the "
                "whole batch (state read and written once per batch)",
             3: "chain_kernel (the library's choice for more than 160 workers): events re-ordered so "
                "that a worker's columns are found in registers or parked in LDS as often as possible",
             4: "regfile_kernel (the library's choice for up to 64 workers): a wave keeps its 64 columns of every worker's "
                "x and xt in vector registers for the whole batch (state read and written once per batch, no LDS, no "
                "barrier)"}


def cpu_baseline(cfg, seconds_budget=20.0):
    """The oracle as it stands, one host core, on a d-slice of the same workload (work is linear in d)."""
    import numpy as np
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    import parity_util as pu
    from oracle import core
    d_slice, n_events = min(250_000, cfg.d), 400
    edges, node_rate, edge_rate, eta, alpha, alpha_t = pu.oracle_params(cfg)
    ev = core.generate_events(cfg.n, [e[0] for e in edges], [e[1] for e in edges], node_rate,
                              np.full(len(edges), edge_rate), cfg.seed, n_events)
    rng = np.random.default_rng(0)
    x0 = rng.normal(0.0, cfg.init_sigma, (cfg.n, d_slice))
    is_grad = ev.kind == 0
    m = len(ev)
    c = c_row = xi = xi_row = None
    if cfg.use_c:
        c = rng.normal(size=(cfg.n, d_slice)); c_row = np.where(is_grad, ev.i, -1)
    if cfg.xi_sigma > 0:
        ids = np.nonzero(is_grad)[0]
        xi = rng.normal(0.0, cfg.xi_sigma, (len(ids), d_slice))
        xi_row = np.full(m, -1, np.int64); xi_row[ids] = np.arange(len(ids))
    st = core.State(x0, None, eta, alpha, alpha_t)
    n_goss, n_grad = int((~is_grad).sum()), int(is_grad.sum())
    per_col = 32.0 * n_goss + (16.0 + (4.0 if xi is not None else 0.0) + (4.0 if c is not None else 0.0)) * n_grad
    t0 = time.perf_counter()
    reps = 0
    while True:
        st.t[:] = 0.0
        st.apply(ev, cfg.gamma, cfg.gscale, xi, xi_row, c, c_row)
        st.stats(float(ev.t[-1]))
        reps += 1
        el = time.perf_counter() - t0
        if el > seconds_budget * 0.5 or reps >= 50:
            break
    per_col += 8.0 * cfg.n
    gbs = per_col * d_slice * reps / el / 1e9
    ev_s_full_d = m * reps / el * d_slice / cfg.d
    return {"value": gbs, "unit": "GB/s", "cores": 1, "kind": "oracle",
            "events_per_s_at_full_d": ev_s_full_d,
            "sample": f"first {m} events of {cfg.name} + one observables pass on a {d_slice}-column slice of "
                      f"all {cfg.n} workers, fp64 state, repeated {reps}x ({el:.1f} s); bytes counted as one fp32 "
                      f"pass per event (compare with one_pass_equivalent_GBs, or events_per_s_at_full_d with "
                      f"events_per_s); host has {os.cpu_count()} cores"}


def short_run(name, batch, steps=6, warmup=2):
    """A few steps of one configuration with the walk, chain, LDS-resident and register-file kernels."""
    import torch
    from paper_2306_08289_amd import workloads as wl
    cfg = wl.CONFIGS[name]
    w = wl.Workload(cfg, device="cuda:0", batch_events=batch, xi_slots=32, reuse_xi=True)
    stats_bytes = 8.0 * cfg.n * cfg.d
    res = {"workload": name, "n": cfg.n, "topology": cfg.topology, "d": cfg.d, "events_per_step": batch,
           "state_bytes": 8.0 * cfg.n * cfg.d,
           "note": "state fits the 256 MB last-level cache: not an HBM figure" if 8.0 * cfg.n * cfg.d < 3e8 else ""}
    for mode, key in ((1, "walk"), (3, "chain"), (2, "resident"), (4, "regfile")):
        w.engine.set_tuning(1, 0, 256, mode)
        for _ in range(warmup):
            w.step(); w.engine.stats(w.t_last)
        torch.cuda.synchronize()
        w.engine.counters(reset=True)
        t0 = time.perf_counter()
        for _ in range(steps):
            w.step(); w.engine.stats(w.t_last)
        torch.cuda.synchronize()
        el = time.perf_counter() - t0
        c = w.engine.counters()
        ev = c["gossip"] + c["gradient"]
        res[key] = {"events_per_s": ev / el, "gossip_events_per_s": c["gossip"] / el,
                    "hbm_GBs": (c["moved_bytes"] + stats_bytes * steps) / el / 1e9,
                    "frac_of_hbm_peak": (c["moved_bytes"] + stats_bytes * steps) / el / 1e9 / HBM_PEAK_GBS,
                    "one_pass_equivalent_GBs": (c["bytes"] + stats_bytes * steps) / el / 1e9}
    w.close()
    del w
    torch.cuda.empty_cache()
    res["cpu_oracle"] = cpu_baseline(cfg, seconds_budget=6.0)
    return res


def reuse_sweep(name, batch):
    """Walk kernel against the distance at which a row comes back: gossip-only batches that cycle over k disjoint
    pairs (0,1), (2,3), ... of the configuration's workers, so that every row is read again k operations after it was
    written.  Needs a graph that has these edges (the complete graph of C5).  With about 2000 resident workgroups of
    16 KB each an operation's footprint is 32 MB: the curve shows which reuse distances the on-chip caches (L2, then
    the 256 MB last-level cache) still serve, and what is left when none does."""
    import numpy as np
    import torch
    from paper_2306_08289_amd import binding, workloads as wl
    cfg = wl.CONFIGS[name]
    w = wl.Workload(cfg, device="cuda:0", batch_events=batch, xi_slots=1, reuse_xi=True)
    eng = w.engine
    eng.set_tuning(1, 0, 256, 1)
    now = [0.0]

    def cyclic_batch(k):
        ops = np.zeros(batch, binding.OP_DTYPE)
        pair = np.arange(batch) % k
        ops["kind"], ops["i"], ops["j"] = binding.KIND_GOSSIP, 2 * pair, 2 * pair + 1
        ops["t"] = now[0] + 1e-3 * (np.arange(batch) // k + 1)
        now[0] = float(ops["t"][-1])
        off = np.arange(0, batch + 1, k, dtype=np.int64)
        return binding.Batch(ops, off if off[-1] == batch else np.append(off, batch))

    rows = []
    k = 1
    while 2 * k <= cfg.n:
        for _ in range(2):
            eng.apply_events(cyclic_batch(k))
        torch.cuda.synchronize()
        eng.counters(reset=True)
        eng.profile(True)
        for _ in range(4):
            eng.apply_events(cyclic_batch(k))
        launches, ms = eng.profile_read()
        eng.profile(False)
        moved = eng.counters()["moved_bytes"]
        rows.append({"reuse_distance_ops": k, "workers_in_cycle": 2 * k, "GBs": moved / (ms * 1e-3) / 1e9,
                     "avg_launch_ms": ms / launches, "alg_bytes_per_launch": moved / launches})
        k *= 2
    w.close()
    return rows


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="C4", help="C1..C5, C4-baseline")
    ap.add_argument("--batch", type=int, default=1024, help="events per step")
    ap.add_argument("--d", type=int, default=None, help="override the parameter count (debugging)")
    ap.add_argument("--unroll", type=int, default=None)
    ap.add_argument("--nontemporal", type=int, default=None)
    ap.add_argument("--threads", type=int, default=None)
    ap.add_argument("--walk", type=int, default=None,
                    help="event kernel of the headline line: 1 = walk, one full pass per event (default: the kernel "
                         "whose traffic is the algorithmic byte count), 3 = chain, 0 = one launch per level, "
                         "2 = LDS-resident (the library's choice for 65 to 160 workers), 4 = register file (the "
                         "library's choice for up to 64 workers)")
    ap.add_argument("--slots", type=int, default=None, help="chain kernel: LDS slots for parked workers (default 5)")
    ap.add_argument("--walk-occupancy", type=int, default=None, help="walk kernel: at most this many workgroups per CU")
    ap.add_argument("--group", type=int, default=None, help="resident kernel: waves per workgroup (default: chosen per batch)")
    ap.add_argument("--cols", type=int, default=None, help="resident kernel: columns per lane")
    ap.add_argument("--no-resident-leg", action="store_true", help="skip the separate LDS-resident measurement")
    ap.add_argument("--no-regfile-leg", action="store_true", help="skip the separate register-file measurement")
    ap.add_argument("--no-chain-leg", action="store_true", help="skip the separate chain-kernel measurement")
    ap.add_argument("--ld-pad", type=int, default=0, help="extra row pitch in units of 4 floats (layout experiments)")
    ap.add_argument("--all-configs", action="store_true",
                    help="append a short measurement of every configuration (C1..C5) to the JSON line")
    ap.add_argument("--no-stats", action="store_true", help="leave the observables pass out of the step")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-inplace-probe", action="store_true", help="skip the in-place streaming ceilings")
    ap.add_argument("--reuse-sweep", action="store_true",
                    help="instead of the benchmark: the walk kernel's rate against the reuse distance of a row "
                         "(synthetic gossip-only batches on --workload, which needs the complete graph: C5)")
    ap.add_argument("--no-profile", action="store_true", help="do not bracket each kernel launch with HIP events")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU (workers are rows of one device buffer; "
                 "no collectives exist) -- use --gpus 1")

    import torch
    from paper_2306_08289_amd import workloads as wl, a2cid_stream_probe

    if args.reuse_sweep:
        torch.cuda.set_device(0)
        print(json.dumps({"reuse_sweep": {"workload": args.workload, "kernel": MODE_WHAT[1], "events_per_launch": args.batch,
                                          "rows": reuse_sweep(args.workload, args.batch)}}))
        return
    cfg = wl.CONFIGS[args.workload]
    if args.d:
        cfg = wl.scaled(cfg, d=args.d)
    torch.cuda.set_device(0)
    w = wl.Workload(cfg, device="cuda:0", batch_events=args.batch, xi_slots=32, reuse_xi=True, ld_pad=args.ld_pad)
    mode = 1 if args.walk is None else args.walk
    auto_mode = 4 if cfg.n <= 64 else 2 if cfg.n <= 160 else 1 if cfg.d <= 4096 else 3      # a2cid_set_tuning, mode -1
    if args.slots is not None:
        w.engine.set_chain_slots(args.slots)
    w.engine.set_tuning(args.unroll or 1, args.nontemporal or 0, args.threads or 256, mode)
    if args.walk_occupancy is not None:
        w.engine.set_walk_occupancy(args.walk_occupancy)
    if args.group is not None or args.cols is not None:
        w.engine.set_resident_group(args.group or 0, args.cols or 1)
    stats_bytes = 0.0 if args.no_stats else 8.0 * cfg.n * cfg.d

    def step():
        b = w.step()
        if not args.no_stats:
            w.engine.stats(w.t_last)
        return b

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # streaming ceiling of this machine: a plain copy of 1/4 of the state (>= 1.6 GB each way at full size)
    rows = max(1, cfg.n // 4)
    src, dst = w.x[:rows].reshape(-1), w.xt[cfg.n - rows:].reshape(-1)
    keep = dst.clone()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a2cid_stream_probe(src, dst)
    e0.record()
    for _ in range(5):
        a2cid_stream_probe(src, dst)
    e1.record()
    torch.cuda.synchronize()
    copy_gbs = 5 * 8.0 * src.numel() / (e0.elapsed_time(e1) * 1e-3) / 1e9
    dst.copy_(keep)
    del keep
    torch.cuda.synchronize()
    # the stored counter readings belong to the default launch shape of their kernel
    default_shape = (not args.d and args.unroll in (None, 1) and args.threads in (None, 256) and
                     args.nontemporal in (None, 0) and args.slots in (None, 5) and not args.ld_pad)

    def measure(steps):
        """Times `steps` steps with the kernel mode currently set; returns wall time, counters and, with profiling
        on, the summed duration of the event-kernel launches (HIP events on the engine's stream)."""
        w.engine.counters(reset=True)
        if not args.no_profile:
            w.engine.profile(True)
        t0 = time.perf_counter()
        for _ in range(steps):
            step()
        torch.cuda.synchronize()
        el = time.perf_counter() - t0
        cnt = w.engine.counters()
        launches, kernel_ms = (0, 0.0)
        if not args.no_profile:
            launches, kernel_ms = w.engine.profile_read()
            w.engine.profile(False)
        return el, cnt, launches, kernel_ms

    def kernel_line(kernel_name, cnt, launches, kernel_ms):
        """Roofline figures of the event kernel of one leg: bytes it moves by construction over its launch time."""
        if not launches:
            return None
        achieved = cnt["moved_bytes"] / (kernel_ms * 1e-3) / 1e9
        traffic, source = MEASURED_TRAFFIC.get((args.workload, args.batch, kernel_name), (None, None)) \
            if default_shape else (None, None)
        head = {"bound": "hbm", "kernel": kernel_name, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": achieved / HBM_PEAK_GBS}
        if kernel_name in ("resident_kernel", "regfile_kernel"):
            # instruction issue (and, for the resident kernel, the level barriers) bound these kernels (SQ counters:
            # profiles/): their HBM figures follow as hbm_GBs / frac_of_hbm_peak
            flop = cfg.d * (FLOP_PER_COLUMN["gossip"] * cnt["gossip"] + FLOP_PER_COLUMN["gradient"] * cnt["gradient"])
            tflops = flop / (kernel_ms * 1e-3) / 1e12
            head = {"bound": "alu", "kernel": kernel_name, "achieved": tflops, "peak": FP32_VECTOR_PEAK_TFLOPS,
                    "unit": "TFLOP/s", "frac": tflops / FP32_VECTOR_PEAK_TFLOPS,
                    "frac_of_unpacked_fp32_peak": tflops / (FP32_VECTOR_PEAK_TFLOPS / 2),
                    "alg_flop_per_launch": flop / launches,
                    "hbm_GBs": achieved, "frac_of_hbm_peak": achieved / HBM_PEAK_GBS}
        return {**head,
                "traffic": traffic,
                "traffic_source": None if traffic is None else
                f"{source}: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of an earlier run of this command, scaled by the "
                "copy probe; bytes between L2 and fabric, per launch; not measured by the run that printed this line",
                "launches": launches, "avg_launch_ms": kernel_ms / launches,
                "alg_bytes_per_launch": cnt["moved_bytes"] / launches,
                "one_pass_bytes_per_launch": cnt["bytes"] / launches,
                "one_pass_equivalent_GBs": cnt["bytes"] / (kernel_ms * 1e-3) / 1e9}

    elapsed, cnt, launches, kernel_ms = measure(args.steps)
    stats_launches, stats_ms = (0, 0.0) if (args.no_profile or args.no_stats) else w.engine.profile_read_stats()

    # in-place streaming ceilings of this machine on the whole state, with the walk kernel's access shape and a reuse
    # distance (n / rows_per_op passes of every resident workgroup) far beyond the caches
    def inplace(rows_per_op, n_ops):
        w.engine.inplace_probe(rows_per_op, n_ops)                 # warm-up
        p0, p1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        p0.record()
        moved = sum(w.engine.inplace_probe(rows_per_op, n_ops) for _ in range(3))
        p1.record()
        torch.cuda.synchronize()
        ms = p0.elapsed_time(p1)
        return {"value": moved / (ms * 1e-3) / 1e9, "unit": "GB/s", "bytes_per_launch": moved / 3,
                "avg_launch_ms": ms / 3, "passes_per_launch": n_ops}
    inplace_ceiling = None
    if not args.no_inplace_probe and cfg.d >= 4:
        per_pass = 64.0 * (cfg.d // 4)
        inplace_ceiling = {
            "what": "in-place pass over the whole state (x and xt of all workers in turn) with the walk kernel's tile and "
                    "access shape, values multiplied by 1; a row is touched again only after n / rows passes of every "
                    "workgroup, so nothing is served from a cache when the state is far larger than 256 MB",
            "gossip_shape": inplace(2, max(8, min(256, int(2.5e10 / per_pass)))),
            "mixing_shape": inplace(1, max(8, min(512, int(2.5e10 / per_pass))))}
    # bytes: what the launched kernels move by construction; for the headline (walk) kernel that is one full pass
    # per event: 32 d per gossip event, 16 d + 4 d per input per gradient event
    total_bytes = cnt["moved_bytes"] + stats_bytes * args.steps
    one_pass_bytes = cnt["bytes"] + stats_bytes * args.steps
    events = cnt["gossip"] + cnt["gradient"]
    value = total_bytes / elapsed / 1e9
    roofline = kernel_line(MODE_NAMES[mode], cnt, launches, kernel_ms)
    out = {
        "metric": "achieved HBM GB/s and gossip events/s, 64 workers \u00d7 25.6M fp32 params"
                  if cfg.n == 64 and cfg.d == 25_600_000 else f"achieved HBM GB/s and gossip events/s, {cfg.name}",
        "value": value, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": elapsed / args.steps * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: n={cfg.n} {cfg.topology} graph, d={cfg.d} fp32, "
                               f"{args.batch} events per step" + ("" if args.no_stats else " + one observables pass"),
                   "kernel": MODE_WHAT[mode],
                   "eta": w.eta, "alpha": w.alpha, "alpha_tilde": w.alpha_tilde, "gamma": cfg.gamma,
                   "edge_rate": w.edge_rate, "unroll": args.unroll, "nontemporal": args.nontemporal,
                   "threads": args.threads, "walk": args.walk, "slots": args.slots},
        "events_per_s": events / elapsed, "gossip_events_per_s": cnt["gossip"] / elapsed,
        "gradient_events_per_s": cnt["gradient"] / elapsed,
        "frac_of_hbm_peak": value / HBM_PEAK_GBS,
        "one_pass_equivalent_GBs": one_pass_bytes / elapsed / 1e9,
        "copy_ceiling": {"value": copy_gbs, "unit": "GB/s",
                         "what": f"plain out-of-place, non-temporal device copy of {8.0 * src.numel() / 1e9:.2f} GB "
                                 "(read + write) on this machine; also the scale of the HBM byte counters"},
        "inplace_ceiling": inplace_ceiling,
        "roofline": roofline,
        "stats_kernel": None if not stats_launches else {
            "bound": "hbm", "kernel": "stats_kernel", "achieved": stats_bytes * stats_launches / (stats_ms * 1e-3) / 1e9,
            "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": stats_bytes * stats_launches / (stats_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "launches": stats_launches, "avg_launch_ms": stats_ms / stats_launches,
            "alg_bytes_per_launch": stats_bytes},
    }
    # separate lines: the kernels that keep workers on the chip between events move fewer bytes than one pass per
    # event, so their events/s go up while their HBM GB/s go down; they are never mixed into the headline figure
    variants = []
    if not args.no_chain_leg and mode != 3:
        variants.append((3, "chain_variant"))
    if not args.no_resident_leg and mode != 2 and cfg.n <= 160:
        variants.append((2, "resident_variant"))
    if not args.no_regfile_leg and mode != 4 and cfg.n <= 64:
        variants.append((4, "regfile_variant"))
    for v_mode, key in variants:
        w.engine.set_tuning(1, 0, 256, v_mode)
        for _ in range(2):
            step()
        torch.cuda.synchronize()
        v_steps = max(3, args.steps // 2)
        v_el, vc, v_launches, v_ms = measure(v_steps)
        if not (args.no_profile or args.no_stats):
            w.engine.profile_read_stats()
        v_events = vc["gossip"] + vc["gradient"]
        out[key] = {
            "what": "same steps with " + MODE_WHAT[v_mode],
            "events_per_s": v_events / v_el, "gossip_events_per_s": vc["gossip"] / v_el,
            "ms_per_step": v_el / v_steps * 1e3, "steps": v_steps,
            "hbm_GBs": (vc["moved_bytes"] + stats_bytes * v_steps) / v_el / 1e9,
            "frac_of_hbm_peak": (vc["moved_bytes"] + stats_bytes * v_steps) / v_el / 1e9 / HBM_PEAK_GBS,
            "one_pass_equivalent_GBs": (vc["bytes"] + stats_bytes * v_steps) / v_el / 1e9,
            "hbm_bytes_per_step_by_construction": vc["moved_bytes"] / v_steps + stats_bytes,
            "one_pass_bytes_per_step": vc["bytes"] / v_steps + stats_bytes,
            "kernel": kernel_line(MODE_NAMES[v_mode], vc, v_launches, v_ms),
            "speedup_vs_headline": (v_events / v_el) / (events / elapsed)}
    # the metric's second figure: events per second of the fastest kernel on this workload (steps as above, one
    # observables pass each), with the kernel named
    legs = [(out["events_per_s"], out["gossip_events_per_s"], MODE_NAMES[mode])]
    legs += [(out[key]["events_per_s"], out[key]["gossip_events_per_s"], MODE_NAMES[v_mode]) for v_mode, key in variants]
    best = max(legs)
    out["fastest_kernel"] = {"kernel": best[2], "events_per_s": best[0], "gossip_events_per_s": best[1],
                             "what": "the highest events/s among the legs of this run; the library chooses this kernel "
                                     "by itself for this shape" if best[2] == MODE_NAMES[auto_mode] else
                                     "the highest events/s among the legs of this run"}
    w.close()
    del w
    torch.cuda.empty_cache()
    if args.all_configs:
        out["all_configs"] = [short_run(name, args.batch) for name in ("C1", "C2", "C3", "C4", "C4-baseline", "C5")]
        # the two cache-resident configurations again with batches long enough to amortise launch and host cost
        out["all_configs"] += [short_run(name, 16384, steps=4, warmup=1) for name in ("C1", "C2")]
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
