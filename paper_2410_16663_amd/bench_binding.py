"""ctypes view of include/fa_bench.h -- the benchmark's measurement aids (argument marshalling only).

Two small libraries of their own, libfa_bench.so (HIP: the matrix-only ceiling probe) and libfa_bench_cpu.so
(plain C: the host streaming-read yardstick); the product libraries neither link nor load them.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
GPU_LIB_PATH = os.path.join(_HERE, "libfa_bench.so")
CPU_LIB_PATH = os.path.join(_HERE, "libfa_bench_cpu.so")
GPU_EXPORTS = ("fa_mfma_probe",)
CPU_EXPORTS = ("fa_cpu_stream_read",)

_gpu = None
_cpu = None


def load_gpu() -> ctypes.CDLL:
    global _gpu
    if _gpu is None:
        if not os.path.exists(GPU_LIB_PATH):
            raise FileNotFoundError(f"{GPU_LIB_PATH} is missing: build it with `python -m paper_2410_16663_amd.build`")
        from . import binding
        binding.load()    # one HIP runtime per process: the attention library's loader sees to that first
        lib = ctypes.CDLL(GPU_LIB_PATH)
        vp = ctypes.c_void_p
        lib.fa_mfma_probe.restype = ctypes.c_int
        lib.fa_mfma_probe.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, vp, ctypes.POINTER(ctypes.c_longlong), vp]
        _gpu = lib
    return _gpu


def load_cpu() -> ctypes.CDLL:
    global _cpu
    if _cpu is None:
        if not os.path.exists(CPU_LIB_PATH):
            raise FileNotFoundError(f"{CPU_LIB_PATH} is missing: build it with `python -m paper_2410_16663_amd.build`")
        lib = ctypes.CDLL(CPU_LIB_PATH)
        lib.fa_cpu_stream_read.restype = ctypes.c_int
        lib.fa_cpu_stream_read.argtypes = [ctypes.c_void_p, ctypes.c_longlong, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                           ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_ulonglong)]
        _cpu = lib
    return _cpu


def _dev_addr(x) -> int:
    if x is None:
        return 0
    return x if isinstance(x, int) else int(x.data_ptr())


def fa_mfma_probe(dtype, operands, iters, scratch, stream=0) -> int:
    """fa_mfma_probe of include/fa_bench.h: enqueue the matrix-only kernel, return the flop it performs."""
    flops = ctypes.c_longlong()
    rc = load_gpu().fa_mfma_probe(int(dtype), int(operands), int(iters), _dev_addr(scratch), ctypes.byref(flops),
                                  _dev_addr(stream))
    if rc != 0:
        raise RuntimeError(f"fa_mfma_probe failed with code {rc}")
    return flops.value


def fa_cpu_stream_read(buf, nbytes, nthreads=0, reps=1, force_scalar=False):
    """fa_cpu_stream_read of include/fa_bench.h: (GB/s, checksum) of `reps` threaded passes over a numpy buffer."""
    gbs = ctypes.c_double()
    chk = ctypes.c_ulonglong()
    rc = load_cpu().fa_cpu_stream_read(int(buf.ctypes.data), int(nbytes), int(nthreads), int(reps), int(bool(force_scalar)),
                                       ctypes.byref(gbs), ctypes.byref(chk))
    if rc != 0:
        raise RuntimeError(f"fa_cpu_stream_read failed with code {rc}")
    return gbs.value, chk.value
