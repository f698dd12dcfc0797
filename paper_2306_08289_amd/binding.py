"""ctypes binding of liba2cid.so: argument marshalling only, every step runs in the library.

The module-level functions carry the names of the C entry points (include/a2cid.h).  The two
small classes `Engine` and `Scheduler` only keep handles and buffers alive and convert between
numpy / torch objects and the plain pointers of the C ABI.
"""
import ctypes as C
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "liba2cid.so")

OK, EINVAL, EGRAPH, EORDER, EMATCHING, EALIGN, EHIP, ENOMEM = 0, -1, -2, -3, -4, -5, -6, -7
KIND_GRADIENT, KIND_GOSSIP = 0, 1
STATS_STATIC_MAX_WORKERS = 256        # A2CID_STATS_STATIC_MAX_WORKERS
ERROR_NAMES = {EINVAL: "A2CID_EINVAL", EGRAPH: "A2CID_EGRAPH", EORDER: "A2CID_EORDER",
               EMATCHING: "A2CID_EMATCHING", EALIGN: "A2CID_EALIGN", EHIP: "A2CID_EHIP",
               ENOMEM: "A2CID_ENOMEM"}


class A2cidError(RuntimeError):
    def __init__(self, code, message):
        super().__init__(f"{ERROR_NAMES.get(code, code)}: {message}")
        self.code = code


class a2cid_graph(C.Structure):
    _fields_ = [("n_edges", C.c_int32), ("u", C.POINTER(C.c_int32)), ("v", C.POINTER(C.c_int32)),
                ("rate", C.POINTER(C.c_double))]


class a2cid_buffers(C.Structure):
    _fields_ = [("x", C.c_void_p), ("xt", C.c_void_p), ("ld", C.c_int64), ("hip_stream", C.c_void_p)]


class a2cid_op(C.Structure):
    _fields_ = [("t", C.c_double), ("kind", C.c_int32), ("i", C.c_int32), ("j", C.c_int32),
                ("gamma", C.c_float), ("gscale", C.c_float), ("clock_rate", C.c_float),
                ("xi", C.c_void_p), ("c", C.c_void_p), ("h", C.c_void_p), ("id", C.c_int64)]


OP_DTYPE = np.dtype([("t", "<f8"), ("kind", "<i4"), ("i", "<i4"), ("j", "<i4"), ("gamma", "<f4"),
                     ("gscale", "<f4"), ("clock_rate", "<f4"), ("xi", "<u8"), ("c", "<u8"), ("h", "<u8"), ("id", "<i8")])
assert OP_DTYPE.itemsize == C.sizeof(a2cid_op) == 64


class a2cid_event_batch(C.Structure):
    _fields_ = [("n_ops", C.c_int64), ("ops", C.c_void_p), ("n_levels", C.c_int32),
                ("level_off", C.POINTER(C.c_int64)), ("t_sync", C.c_double)]


class a2cid_stats_out(C.Structure):
    _fields_ = [("consensus_x", C.c_double), ("consensus_xt", C.c_double),
                ("sum_x", C.POINTER(C.c_double)), ("sum_xt", C.POINTER(C.c_double))]


COEF_DTYPE = np.dtype([("b_pre_i", "<f4"), ("b_pre_j", "<f4"), ("b_post_i", "<f4"), ("b_post_j", "<f4")])

# every symbol include/a2cid.h declares: name -> (restype, argtypes)
_P = C.POINTER
SIGNATURES = {
    "a2cid_graph_params": (C.c_int, [_P(a2cid_graph), C.c_int32, _P(C.c_double), _P(C.c_double),
                                     _P(C.c_double), _P(C.c_double)]),
    "a2cid_create": (C.c_int, [_P(C.c_void_p), C.c_int32, C.c_int64, _P(a2cid_graph), C.c_double, C.c_double,
                               C.c_double, _P(a2cid_buffers)]),
    "a2cid_apply_events": (C.c_int, [C.c_void_p, _P(a2cid_event_batch)]),
    "a2cid_stats": (C.c_int, [C.c_void_p, C.c_double, _P(a2cid_stats_out)]),
    "a2cid_stats_static": (C.c_int, [C.c_void_p, C.c_double, C.c_void_p]),
    "a2cid_flush": (C.c_int, [C.c_void_p, C.c_double]),
    "a2cid_set_order": (C.c_int, [C.c_void_p, C.c_int32]),
    "a2cid_average": (C.c_int, [C.c_void_p, C.c_double]),
    "a2cid_get_times": (C.c_int, [C.c_void_p, _P(C.c_double)]),
    "a2cid_set_times": (C.c_int, [C.c_void_p, _P(C.c_double)]),
    "a2cid_get_clock_rates": (C.c_int, [C.c_void_p, _P(C.c_double)]),
    "a2cid_set_clock_rates": (C.c_int, [C.c_void_p, _P(C.c_double)]),
    "a2cid_plan_batch_clocks": (C.c_int, [C.c_int32, _P(a2cid_graph), C.c_double, _P(C.c_double), _P(C.c_double),
                                          _P(a2cid_event_batch), C.c_void_p]),
    "a2cid_synchronize": (C.c_int, [C.c_void_p]),
    "a2cid_destroy": (None, [C.c_void_p]),
    "a2cid_plan_chain": (C.c_int, [C.c_int32, _P(a2cid_event_batch), C.c_int32, C.c_void_p, C.c_int64,
                                   _P(C.c_int64), _P(C.c_double)]),
    "a2cid_plan_resident": (C.c_int, [C.c_int32, _P(a2cid_event_batch), C.c_void_p, _P(C.c_int32), _P(C.c_int32), C.c_int64,
                                      C.c_void_p, C.c_void_p, _P(C.c_int32), C.c_void_p, _P(C.c_int32), _P(C.c_int64)]),
    "a2cid_plan_registers": (C.c_int, [C.c_int32, _P(a2cid_event_batch), C.c_void_p, C.c_int64, C.c_int64, C.c_int32,
                                       C.c_void_p, C.c_void_p, _P(C.c_int64), C.c_void_p, _P(C.c_int32), _P(C.c_uint64),
                                       _P(C.c_int64)]),
    "a2cid_check_registers": (C.c_int, [C.c_int32, C.c_int32, C.c_void_p, C.c_int64]),
    "a2cid_set_chain_slots": (C.c_int, [C.c_void_p, C.c_int32]),
    "a2cid_plan_batch": (C.c_int, [C.c_int32, _P(a2cid_graph), C.c_double, _P(C.c_double),
                                   _P(a2cid_event_batch), C.c_void_p]),
    "a2cid_sched_create": (C.c_int, [_P(C.c_void_p), C.c_int32, _P(a2cid_graph), _P(C.c_double), C.c_uint64]),
    "a2cid_sched_create_fifo": (C.c_int, [_P(C.c_void_p), C.c_int32, _P(a2cid_graph), _P(C.c_double), C.c_double,
                                          C.c_double, C.c_double, C.c_int32, C.c_uint64]),
    "a2cid_sched_next": (C.c_int, [C.c_void_p, C.c_int64, _P(a2cid_event_batch)]),
    "a2cid_sched_skip": (C.c_int, [C.c_void_p, C.c_int64]),
    "a2cid_sched_counts": (C.c_int, [C.c_void_p, _P(C.c_int64)]),
    "a2cid_sched_destroy": (None, [C.c_void_p]),
    "a2cid_set_tuning": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32]),
    "a2cid_set_stats_tuning": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32]),
    "a2cid_check_device_span": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int64]),
    "a2cid_stream_probe": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p]),
    "a2cid_counters": (C.c_int, [C.c_void_p, _P(C.c_int64), _P(C.c_int64), _P(C.c_int64), _P(C.c_double),
                                 _P(C.c_double), C.c_int32]),
    "a2cid_set_resident_group": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32]),
    "a2cid_set_walk_occupancy": (C.c_int, [C.c_void_p, C.c_int32]),
    "a2cid_profile": (C.c_int, [C.c_void_p, C.c_int32]),
    "a2cid_profile_read": (C.c_int, [C.c_void_p, _P(C.c_int64), _P(C.c_double)]),
    "a2cid_profile_read_stats": (C.c_int, [C.c_void_p, _P(C.c_int64), _P(C.c_double)]),
    "a2cid_inplace_probe": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, _P(C.c_double)]),
    "a2cid_last_error": (C.c_char_p, []),
    "a2cid_version": (C.c_char_p, []),
}

_lib = None


def load():
    """Loads liba2cid.so.  There is no fallback: a missing library is an error."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2306_08289_amd.build` "
                              "(or __graft_entry__.build()); there is no CPU fallback")
        lib = C.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype = res
            fn.argtypes = args
        _lib = lib
    return _lib


def _check(rc):
    if rc != OK:
        raise A2cidError(rc, load().a2cid_last_error().decode())


def _dptr(arr):
    return arr.ctypes.data_as(_P(C.c_double))


def a2cid_stream_probe(src, dst, stream=None):
    """Enqueues the copy probe dst <- src on two equally sized contiguous fp32 CUDA tensors."""
    import torch
    assert src.is_cuda and dst.is_cuda and src.dtype == dst.dtype == torch.float32
    assert src.is_contiguous() and dst.is_contiguous() and src.numel() == dst.numel()
    if stream is None:
        stream = torch.cuda.current_stream(src.device)
    _check(load().a2cid_stream_probe(src.data_ptr(), dst.data_ptr(), src.numel(), stream.cuda_stream))


class _GraphArg:
    """Keeps the numpy arrays behind an a2cid_graph alive."""

    def __init__(self, u, v, rate):
        self.u = np.ascontiguousarray(u, np.int32)
        self.v = np.ascontiguousarray(v, np.int32)
        self.rate = np.ascontiguousarray(np.broadcast_to(rate, self.u.shape), np.float64)
        self.struct = a2cid_graph(len(self.u), self.u.ctypes.data_as(_P(C.c_int32)),
                                  self.v.ctypes.data_as(_P(C.c_int32)), _dptr(self.rate))


class Batch:
    """Host-side batch: a structured numpy array of a2cid_op records plus the level table."""

    def __init__(self, ops, level_off, t_sync=float("nan")):
        self.ops = np.ascontiguousarray(ops, OP_DTYPE)
        self.level_off = np.ascontiguousarray(level_off, np.int64)
        self.t_sync = float(t_sync)

    @property
    def n_levels(self):
        return len(self.level_off) - 1

    def struct(self):
        return a2cid_event_batch(len(self.ops), self.ops.ctypes.data, self.n_levels,
                                 self.level_off.ctypes.data_as(_P(C.c_int64)), self.t_sync)


def a2cid_graph_params(n, u, v, rate):
    g = _GraphArg(u, v, rate)
    out = [C.c_double() for _ in range(4)]
    _check(load().a2cid_graph_params(C.byref(g.struct), n, *[C.byref(o) for o in out]))
    return {"chi1": out[0].value, "chi2": out[1].value, "eta": out[2].value, "alpha": 0.5,
            "alpha_tilde": out[3].value}


def a2cid_plan_batch(n, u, v, rate, eta, t, batch, clock_rates=None):
    """Returns (t_after, coefficients), or with clock_rates (the speeds of the workers' own clocks) (t_after,
    coefficients, clock_rates_after); the arguments are not modified."""
    g = _GraphArg(u, v, rate)
    t = np.array(t, np.float64)
    coef = np.zeros(len(batch.ops), COEF_DTYPE)
    bs = batch.struct()
    if clock_rates is None:
        _check(load().a2cid_plan_batch(n, C.byref(g.struct), float(eta), _dptr(t), C.byref(bs), coef.ctypes.data))
        return t, coef
    cr = np.array(clock_rates, np.float64)
    _check(load().a2cid_plan_batch_clocks(n, C.byref(g.struct), float(eta), _dptr(t), _dptr(cr), C.byref(bs),
                                          coef.ctypes.data))
    return t, coef, cr


STEP_DTYPE = np.dtype([("op", "<i4"), ("row_i", "<i4"), ("row_j", "<i4"), ("src_i", "u1"), ("src_j", "u1"),
                       ("dst_i", "u1"), ("dst_j", "u1")])
LOC_MEMORY, LOC_CARRY, LOC_SLOT0 = 0, 1, 2


def a2cid_plan_chain(n, batch, lds_slots=5):
    """Returns (steps, bytes_per_column): the chain kernel's programme for the batch as a STEP_DTYPE array."""
    m = len(batch.ops)
    steps = np.zeros(3 * m + int(lds_slots), STEP_DTYPE)
    count, per_col = C.c_int64(), C.c_double()
    bs = batch.struct()
    _check(load().a2cid_plan_chain(int(n), C.byref(bs), int(lds_slots), steps.ctypes.data, len(steps),
                                   C.byref(count), C.byref(per_col)))
    return steps[:count.value], per_col.value


SLOT_DTYPE = np.dtype([("x", "<u4"), ("y", "<u4"), ("z", "<u4"), ("w", "<u4")])
RES_JUMP, RES_END, RES_NONE = 0x10000, 0x20000, 0xffffffff


def a2cid_plan_resident(n, batch, coef, first_op=0, waves=0, cols=1):
    """One launch of the resident kernel from operation first_op on.  Returns a dict: waves, cols (as used), slots
    (waves x slots-per-wave SLOT_DTYPE array), rows (LDS row -> worker), gradient_ops (ordinal -> index in the batch),
    next_op."""
    slots = np.zeros(8192, SLOT_DTYPE)
    rows = np.zeros(int(n), np.int32)
    gops = np.zeros(max(1, len(batch.ops)), np.int64)
    w, c = C.c_int32(int(waves)), C.c_int32(int(cols))
    n_rows, n_g, nxt = C.c_int32(), C.c_int32(), C.c_int64()
    bs = batch.struct()
    coef = np.ascontiguousarray(coef, COEF_DTYPE)
    _check(load().a2cid_plan_resident(int(n), C.byref(bs), coef.ctypes.data, C.byref(w), C.byref(c), int(first_op),
                                      slots.ctypes.data, rows.ctypes.data, C.byref(n_rows), gops.ctypes.data,
                                      C.byref(n_g), C.byref(nxt)))
    per_wave = 256 if w.value >= 16 else 512
    return {"waves": w.value, "cols": c.value, "slots": slots[:w.value * per_wave].reshape(w.value, per_wave).copy(),
            "rows": rows[:n_rows.value].copy(), "gradient_ops": gops[:n_g.value].copy(), "next_op": nxt.value}


REG_GOSSIP, REG_GRADIENT, REG_MIX, REG_CONTROL = 0, 1, 2, 3      # kind of a register-file slot: x >> 8
REG_SWITCH, REG_END, REG_REQUEST = 1, 2, 3                      # y of a control slot
REG_BLOCK, REG_CHUNK = 8, 8


def a2cid_plan_registers(n, batch, coef, first_op=0, max_slots=8192, full=False, zero_one=0x1000):
    """One launch of the register-file kernel from operation first_op on.  Returns a dict: slots (SLOT_DTYPE array),
    gradient_ops (ordinal -> index in the batch), touched (bit mask of workers), next_op."""
    slots = np.zeros(max(int(max_slots), 1), SLOT_DTYPE)
    gops = np.zeros(max(1, len(batch.ops)), np.int64)
    n_slots, n_g, touched, nxt = C.c_int64(), C.c_int32(), C.c_uint64(), C.c_int64()
    bs = batch.struct()
    coef = np.ascontiguousarray(coef, COEF_DTYPE)
    _check(load().a2cid_plan_registers(int(n), C.byref(bs), coef.ctypes.data, int(first_op), int(max_slots),
                                       int(bool(full)), C.c_void_p(int(zero_one)), slots.ctypes.data, C.byref(n_slots),
                                       gops.ctypes.data, C.byref(n_g), C.byref(touched), C.byref(nxt)))
    return {"slots": slots[:n_slots.value].copy(), "gradient_ops": gops[:n_g.value].copy(), "touched": touched.value,
            "next_op": nxt.value}


def a2cid_check_registers(n, slots, full=False):
    """Raises A2cidError unless slots is a programme the register-file kernel may run for n workers."""
    slots = np.ascontiguousarray(slots, SLOT_DTYPE)
    _check(load().a2cid_check_registers(int(n), int(bool(full)), slots.ctypes.data, len(slots)))


class Scheduler:
    """a2cid_sched_*: seeded Poisson clocks -> serial stream -> level-packed batches."""

    def __init__(self, n, u, v, edge_rate, node_rate, seed, fifo=None):
        """fifo = None: Poisson clocks per node and edge; fifo = dict(comm_per_grad, comm_time, jitter[, normalize]): the
        first-in-first-out pairing source (edge rates are then ignored)."""
        self._g = _GraphArg(u, v, edge_rate)
        self.n = n
        self.n_clocks = n + len(self._g.u)
        nr = np.ascontiguousarray(np.broadcast_to(node_rate, (n,)), np.float64)
        self._h = C.c_void_p()
        if fifo is None:
            _check(load().a2cid_sched_create(C.byref(self._h), n, C.byref(self._g.struct), _dptr(nr), int(seed)))
        else:
            _check(load().a2cid_sched_create_fifo(C.byref(self._h), n, C.byref(self._g.struct), _dptr(nr),
                                                  float(fifo["comm_per_grad"]), float(fifo["comm_time"]),
                                                  float(fifo["jitter"]), {False: 0, True: 1, "worker": 2}[fifo.get("normalize", False)],
                                                  int(seed)))

    def next(self, max_events):
        """Next batch as a `Batch` (copied out of the scheduler's storage)."""
        bs = a2cid_event_batch()
        _check(load().a2cid_sched_next(self._h, int(max_events), C.byref(bs)))
        if bs.n_ops:
            ops = np.ctypeslib.as_array(C.cast(bs.ops, _P(C.c_uint8)), (bs.n_ops * OP_DTYPE.itemsize,))
            ops = ops.view(OP_DTYPE).copy()
        else:
            ops = np.zeros(0, OP_DTYPE)
        level_off = np.ctypeslib.as_array(bs.level_off, (bs.n_levels + 1,)).copy()
        return Batch(ops, level_off, bs.t_sync)

    def skip(self, n_events):
        _check(load().a2cid_sched_skip(self._h, int(n_events)))

    def counts(self):
        out = np.zeros(self.n_clocks, np.int64)
        _check(load().a2cid_sched_counts(self._h, out.ctypes.data_as(_P(C.c_int64))))
        return out

    def close(self):
        if self._h:
            load().a2cid_sched_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Engine:
    """a2cid_create / apply_events / stats / flush on two torch device tensors (memory and stream only)."""

    def __init__(self, x, xt, d, u, v, edge_rate, eta, alpha, alpha_tilde, stream=None):
        import torch
        assert x.is_cuda and xt.is_cuda and x.dtype == torch.float32 and xt.dtype == torch.float32
        assert x.dim() == 2 and x.shape == xt.shape and x.stride(1) == 1 and xt.stride() == x.stride()
        self.x, self.xt = x, xt            # keep the tensors alive
        self.n, self.d, self.ld = x.shape[0], int(d), x.stride(0)
        self._g = _GraphArg(u, v, edge_rate)
        if stream is None:
            stream = torch.cuda.current_stream(x.device)
        self.stream = stream
        buf = a2cid_buffers(x.data_ptr(), xt.data_ptr(), self.ld, stream.cuda_stream)
        self._h = C.c_void_p()
        with torch.cuda.device(x.device):
            _check(load().a2cid_create(C.byref(self._h), self.n, self.d, C.byref(self._g.struct), float(eta),
                                       float(alpha), float(alpha_tilde), C.byref(buf)))

    def _device(self):
        """The library requires the device of creation to be current on every call that touches the GPU."""
        import torch
        return torch.cuda.device(self.x.device)

    def apply_events(self, batch):
        bs = batch.struct()
        with self._device():
            _check(load().a2cid_apply_events(self._h, C.byref(bs)))

    def stats(self, t_now):
        sx = np.zeros(self.n); sxt = np.zeros(self.n)
        out = a2cid_stats_out(0.0, 0.0, _dptr(sx), _dptr(sxt))
        with self._device():
            _check(load().a2cid_stats(self._h, float(t_now), C.byref(out)))
        return {"consensus_x": out.consensus_x, "consensus_xt": out.consensus_xt, "sum_x": sx, "sum_xt": sxt}

    def stats_static(self, t_now, out):
        """a2cid_stats_static: the observables into `out`, a contiguous fp64 CUDA tensor of 2 n + 2 elements
        (sums of x, sums of xt, consensus distances); asynchronous, nothing is allocated."""
        import torch
        assert out.is_cuda and out.dtype == torch.float64 and out.is_contiguous() and out.numel() == 2 * self.n + 2
        with self._device():
            _check(load().a2cid_stats_static(self._h, float(t_now), C.c_void_p(out.data_ptr())))

    def set_order(self, order):
        _check(load().a2cid_set_order(self._h, int(order)))

    def flush(self, t_now):
        with self._device():
            _check(load().a2cid_flush(self._h, float(t_now)))

    def average(self, t_now):
        with self._device():
            _check(load().a2cid_average(self._h, float(t_now)))

    def times(self):
        t = np.zeros(self.n)
        _check(load().a2cid_get_times(self._h, _dptr(t)))
        return t

    def clock_rates(self):
        r = np.zeros(self.n, np.float64)
        _check(load().a2cid_get_clock_rates(self._h, _dptr(r)))
        return r

    def set_clock_rates(self, rate):
        r = np.ascontiguousarray(np.broadcast_to(rate, (self.n,)), np.float64)
        _check(load().a2cid_set_clock_rates(self._h, _dptr(r)))

    def set_times(self, t):
        t = np.ascontiguousarray(t, np.float64)
        assert t.shape == (self.n,)
        _check(load().a2cid_set_times(self._h, _dptr(t)))

    def synchronize(self):
        _check(load().a2cid_synchronize(self._h))

    def check_device_span(self, address, nbytes):
        """Raises A2cidError unless [address, address + nbytes) is device memory the kernels may touch."""
        _check(load().a2cid_check_device_span(self._h, C.c_void_p(int(address)), int(nbytes)))

    def set_tuning(self, unroll=1, nontemporal=0, threads=256, mode=-1):
        _check(load().a2cid_set_tuning(self._h, int(unroll), int(bool(nontemporal)), int(threads), int(mode)))

    def set_chain_slots(self, slots=5):
        _check(load().a2cid_set_chain_slots(self._h, int(slots)))

    def set_walk_occupancy(self, workgroups_per_cu=0):
        _check(load().a2cid_set_walk_occupancy(self._h, int(workgroups_per_cu)))

    def set_resident_group(self, group=0, cols=1):
        _check(load().a2cid_set_resident_group(self._h, int(group), int(cols)))

    def set_stats_tuning(self, pieces=2, rows=2, blocks=2048, nontemporal=1):
        _check(load().a2cid_set_stats_tuning(self._h, int(pieces), int(rows), int(blocks), int(bool(nontemporal))))

    def counters(self, reset=False):
        g, gr, la = C.c_int64(), C.c_int64(), C.c_int64()
        by, rb = C.c_double(), C.c_double()
        _check(load().a2cid_counters(self._h, C.byref(g), C.byref(gr), C.byref(la), C.byref(by), C.byref(rb),
                                     int(reset)))
        return {"gossip": g.value, "gradient": gr.value, "launches": la.value, "bytes": by.value,
                "moved_bytes": rb.value}

    def profile(self, enable):
        _check(load().a2cid_profile(self._h, int(bool(enable))))

    def profile_read(self):
        nl, ms = C.c_int64(), C.c_double()
        _check(load().a2cid_profile_read(self._h, C.byref(nl), C.byref(ms)))
        return nl.value, ms.value

    def profile_read_stats(self):
        nl, ms = C.c_int64(), C.c_double()
        _check(load().a2cid_profile_read_stats(self._h, C.byref(nl), C.byref(ms)))
        return nl.value, ms.value

    def inplace_probe(self, rows_per_op, n_ops):
        """Enqueues the in-place streaming probe on the state; returns the bytes the launch moves."""
        moved = C.c_double()
        with self._device():
            _check(load().a2cid_inplace_probe(self._h, int(rows_per_op), int(n_ops), C.byref(moved)))
        return moved.value

    def close(self):
        if self._h:
            load().a2cid_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
