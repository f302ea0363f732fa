"""ctypes view of the host-side C ABI declared in include/fa_cpu.h -- argument marshalling only.

The layer split of the CPU-GPU cooperative strategy and the decoding-step attention on the CPU run inside
libfa_cpu.so.  numpy arrays (uint16 bit patterns) or raw host addresses are accepted.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfa_cpu.so")

FA_CPU_OK = 0
FA_CPU_ERR_NULL = -1
FA_CPU_ERR_SHAPE = -2
FA_CPU_ERR_HEADDIM = -3
FA_CPU_ERR_DTYPE = -4
FA_CPU_ERR_SCALE = -5
FA_CPU_ERR_NOMEM = -8

# every symbol include/fa_cpu.h declares
EXPORTS = ("fa_coop_plan_bytes", "fa_coop_plan_fp16", "fa_cpu_decode", "fa_cpu_has_avx512", "fa_cpu_set_scalar")

_lib = None


class FaCpuError(RuntimeError):
    def __init__(self, code: int):
        self.code = code
        super().__init__(f"fa_cpu error {code}")


def load() -> ctypes.CDLL:
    """Load libfa_cpu.so (built by paper_2410_16663_amd.build.build_cpu); raises if it is not there."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is missing: build it with `python -m paper_2410_16663_amd.build`")
        lib = ctypes.CDLL(LIB_PATH)
        ip = ctypes.POINTER(ctypes.c_int)
        vp = ctypes.c_void_p
        lib.fa_coop_plan_bytes.restype = ctypes.c_int
        lib.fa_coop_plan_bytes.argtypes = [ctypes.c_double] * 5 + [ctypes.c_int, ctypes.c_int, ip, ip]
        lib.fa_coop_plan_fp16.restype = ctypes.c_int
        lib.fa_coop_plan_fp16.argtypes = [ctypes.c_double, ctypes.c_int, ctypes.c_int] + [ctypes.c_longlong] * 6 + [ip, ip]
        lib.fa_cpu_decode.restype = ctypes.c_int
        lib.fa_cpu_decode.argtypes = [vp, vp, vp, vp, vp] + [ctypes.c_int] * 4 + [ctypes.c_float, ctypes.c_int,
                                                                                  ctypes.c_int]
        lib.fa_cpu_has_avx512.restype = ctypes.c_int
        lib.fa_cpu_has_avx512.argtypes = []
        lib.fa_cpu_set_scalar.restype = ctypes.c_int
        lib.fa_cpu_set_scalar.argtypes = [ctypes.c_int]
        _lib = lib
    return _lib


def _addr(x) -> int:
    if x is None:
        return 0
    if isinstance(x, int):
        return x
    if hasattr(x, "ctypes"):
        return int(x.ctypes.data)
    raise TypeError("pass a host address (int) or a numpy array")


def fa_coop_plan_bytes(m_gpu, m_w, m_mid, m_vocab, m_kv, n, L):
    """fa_coop_plan_bytes of include/fa_cpu.h: returns (L_GPU, L_CPU)."""
    a, b = ctypes.c_int(), ctypes.c_int()
    rc = load().fa_coop_plan_bytes(float(m_gpu), float(m_w), float(m_mid), float(m_vocab), float(m_kv), int(n), int(L),
                                   ctypes.byref(a), ctypes.byref(b))
    if rc != FA_CPU_OK:
        raise FaCpuError(rc)
    return a.value, b.value


def fa_coop_plan_fp16(m_gpu, n, L, H1, H2, V, B, S, O):
    """fa_coop_plan_fp16 of include/fa_cpu.h: returns (L_GPU, L_CPU)."""
    a, b = ctypes.c_int(), ctypes.c_int()
    rc = load().fa_coop_plan_fp16(float(m_gpu), int(n), int(L), int(H1), int(H2), int(V), int(B), int(S), int(O),
                                  ctypes.byref(a), ctypes.byref(b))
    if rc != FA_CPU_OK:
        raise FaCpuError(rc)
    return a.value, b.value


def fa_cpu_decode_raw(q, k, v, o, lse, B, H, Nk, D, scale, dtype, nthreads=0) -> int:
    """Call fa_cpu_decode and return its status code unchanged."""
    return load().fa_cpu_decode(_addr(q), _addr(k), _addr(v), _addr(o), _addr(lse), int(B), int(H), int(Nk), int(D),
                                float(scale), int(dtype), int(nthreads))


def fa_cpu_decode(q, k, v, o, lse, B, H, Nk, D, scale, dtype, nthreads=0) -> None:
    """fa_cpu_decode of include/fa_cpu.h; raises FaCpuError on a negative status."""
    rc = fa_cpu_decode_raw(q, k, v, o, lse, B, H, Nk, D, scale, dtype, nthreads)
    if rc != FA_CPU_OK:
        raise FaCpuError(rc)


def fa_cpu_has_avx512() -> bool:
    return bool(load().fa_cpu_has_avx512())


def fa_cpu_set_scalar(on: bool) -> bool:
    return bool(load().fa_cpu_set_scalar(int(bool(on))))
