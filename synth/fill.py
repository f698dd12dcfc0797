"""Loader for the device side of the input generator (libsynth_fill.so)."""
import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libsynth_fill.so")
_lib = None


def load():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run `python -m synth.build`")
        _lib = C.CDLL(LIB_PATH)
        _lib.synth_fill_normal.restype = C.c_int
        _lib.synth_fill_normal.argtypes = [C.c_void_p, C.c_int64, C.c_uint64, C.c_uint32, C.c_uint64,
                                           C.c_float, C.c_float, C.c_void_p]
    return _lib


def fill_normal(tensor_row, seed, domain, row, sigma=1.0, mean=0.0, stream=None):
    """Fills a contiguous 1-D fp32 CUDA tensor with generator row `row` (columns 0..len-1)."""
    import torch
    assert tensor_row.is_cuda and tensor_row.dtype == torch.float32 and tensor_row.dim() == 1
    assert tensor_row.stride(0) == 1
    if stream is None:
        stream = torch.cuda.current_stream(tensor_row.device)
    rc = load().synth_fill_normal(tensor_row.data_ptr(), tensor_row.numel(), int(seed), int(domain), int(row),
                                  float(sigma), float(mean), stream.cuda_stream)
    if rc != 0:
        raise RuntimeError(f"synth_fill_normal failed with HIP error {rc}")
