"""Measurement helper (not part of the library's API): times a plain streaming read of a device buffer with
libfls_probe.so, the empirical HBM ceiling bench.py reports beside the SpMM kernel's achieved bandwidth."""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfls_probe.so")
_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with paper_2309_10285_amd._build.build()")
        L = ctypes.CDLL(LIB_PATH)
        L.fls_probe_stream_read.argtypes = [ctypes.c_void_p, ctypes.c_uint64, ctypes.c_int, ctypes.c_int,
                                            ctypes.c_void_p, ctypes.c_void_p]
        L.fls_probe_stream_read.restype = ctypes.c_int
        _lib = L
    return _lib


def stream_read_gbps(buffers, grid, unroll=8, steps=200, warmup=20):
    """GB/s of a plain read of the given uint8 CUDA tensors (all of one size, rotated so that no read finds
    its data in the Infinity Cache), `grid` persistent workgroups of eight waves.  Timed with events on the
    current stream, like the kernel it is compared with."""
    import torch

    f = lib().fls_probe_stream_read
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    sink = torch.zeros(64, dtype=torch.int32, device="cuda")
    nbytes = buffers[0].numel()
    args = [(ctypes.c_void_p(b.data_ptr()), nbytes, grid, unroll, ctypes.c_void_p(sink.data_ptr()), stream) for b in buffers]
    for i in range(warmup):
        assert f(*args[i % len(args)]) == 0
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(steps):
        f(*args[i % len(args)])
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / steps
    return nbytes / ms / 1e6, ms * 1e3
