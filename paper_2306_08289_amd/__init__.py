"""MI355X-native engine for the continuous-momentum gossip dynamic of A2CiD2 (arXiv 2306.08289).

Everything runs in liba2cid.so (HIP kernels for gfx950 + a C++ host planner / scheduler);
this package is only the ctypes binding.  There is no CPU fallback: using the engine without the
built library raises ImportError.
"""
from .binding import (A2cidError, Batch, Engine, Scheduler, OP_DTYPE, COEF_DTYPE, KIND_GOSSIP,  # noqa: F401
                      KIND_GRADIENT, a2cid_graph_params, a2cid_plan_batch, a2cid_stream_probe, load)
