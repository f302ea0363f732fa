"""ctypes view of the C ABI declared in include/fa.h -- argument marshalling only.

Every step of the attention forward runs inside libfa.so's HIP kernels.  There is no
fallback: if the library is missing, loading raises.  torch is optional here; device
buffers may be passed as raw integer addresses or as anything with ``data_ptr()``.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfa.so")

FA_OK = 0
FA_ERR_NULL = -1
FA_ERR_SHAPE = -2
FA_ERR_HEADDIM = -3
FA_ERR_DTYPE = -4
FA_ERR_SCALE = -5
FA_ERR_ALIGN = -6
FA_ERR_LAUNCH = -7
FA_ERR_WORKSPACE = -8
FA_ERR_NSPLIT = -9
FA_ERR_MASK = -10
FA_ERR_OPTION = -11
FA_AUTO = -1
FA_OPT_FWD_MODE = 0
FA_OPT_DECODE_KERNEL = 1
FA_OPT_LINEAR_TILE = 2
FA_OPT_LINEAR_PANEL = 3
FA_OPT_LINEAR_OVERLAP = 4
FA_TILE_SKIP = 0
FA_TILE_FULL = 1
FA_TILE_PARTIAL = 2
FA_DTYPE_F16 = 0
FA_DTYPE_BF16 = 1
FA_MODE_SPLIT = 0
FA_MODE_WIDE = 1
FA_MODE_WIDE64 = 4
FA_MODE_WIDE_FOLD = 2
FA_MODE_STREAM = 3

# every symbol include/fa.h declares
EXPORTS = ("fa_fwd", "fa_fwd_plan", "fa_fwd_splitkv", "fa_fwd_splitkv_static", "fa_fwd_splitkv_plan", "fa_fwd_masked", "fa_attn_linear_block",
           "fa_attn_linear", "fa_mask_tile_class",
           "fa_mask_tile_walk", "fa_mask_interior_run", "fa_set_option", "fa_strerror", "fa_version", "fa_last_hip_error",
           "fa_decode_masked")

_lib = None


class FaPlan(ctypes.Structure):
    """fa_plan_t of include/fa.h."""
    _fields_ = [("mode", ctypes.c_int), ("block_m", ctypes.c_int), ("block_n", ctypes.c_int),
                ("threads", ctypes.c_int), ("grid", ctypes.c_int), ("lds_bytes", ctypes.c_int),
                ("work_items", ctypes.c_longlong), ("tiles_visited", ctypes.c_longlong),
                ("tiles_total", ctypes.c_longlong)]


class FaSplitKvPlan(ctypes.Structure):
    """fa_splitkv_plan_t of include/fa.h."""
    _fields_ = [("nsplit", ctypes.c_int), ("grid_x", ctypes.c_int), ("grid_y", ctypes.c_int),
                ("combine_grid", ctypes.c_int), ("work_items", ctypes.c_longlong),
                ("workspace_bytes", ctypes.c_longlong), ("streaming", ctypes.c_int)]


class FaMask(ctypes.Structure):
    """fa_mask_t of include/fa.h (kv_len is a device address or 0)."""
    _fields_ = [("window_left", ctypes.c_int), ("window_right", ctypes.c_int), ("prefix", ctypes.c_int),
                ("diag_from_kv_len", ctypes.c_int), ("kv_len", ctypes.c_void_p)]


class FaError(RuntimeError):
    def __init__(self, code: int):
        self.code = code
        super().__init__(f"fa error {code}: {fa_strerror(code)}")


def _share_torchs_hip_runtime() -> None:
    """One HIP runtime per process.  A PyTorch wheel ships its own libamdhip64.so and loads it by that file
    name; libfa.so asks the loader for ``libamdhip64.so.7``.  When torch is imported first the loader hands
    libfa.so torch's copy (same SONAME).  The other way round it would load the system's copy for libfa.so and,
    later, torch's for torch: two runtimes with separate device state, and the first kernel launch through
    libfa.so fails.  So if torch is installed but not imported yet, its copy is loaded here, globally, before
    libfa.so: both then resolve to it (torch is located, not imported)."""
    import importlib.util
    import sys
    if "torch" in sys.modules:
        return
    try:
        spec = importlib.util.find_spec("torch")
    except (ImportError, ValueError):
        return
    if spec is None or not spec.origin:
        return
    cand = os.path.join(os.path.dirname(spec.origin), "lib", "libamdhip64.so")
    if os.path.exists(cand):
        ctypes.CDLL(cand, mode=ctypes.RTLD_GLOBAL)


def load() -> ctypes.CDLL:
    """Load libfa.so (built by paper_2410_16663_amd.build); raises if it is not there."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2410_16663_amd.build` "
                "(there is no non-HIP fallback)")
        _share_torchs_hip_runtime()
        lib = ctypes.CDLL(LIB_PATH)
        vp = ctypes.c_void_p
        lib.fa_fwd.restype = ctypes.c_int
        lib.fa_fwd.argtypes = [vp, vp, vp, vp, vp] + [ctypes.c_int] * 5 + [
            ctypes.c_float, ctypes.c_int, ctypes.c_int, vp]
        lib.fa_fwd_plan.restype = ctypes.c_int
        lib.fa_fwd_plan.argtypes = [ctypes.c_int] * 7 + [ctypes.POINTER(FaPlan)]
        lib.fa_fwd_splitkv.restype = ctypes.c_int
        lib.fa_fwd_splitkv.argtypes = [vp, vp, vp, vp, vp] + [ctypes.c_int] * 5 + [
            ctypes.c_float, ctypes.c_int, ctypes.c_int, ctypes.c_int, vp, ctypes.c_longlong, vp]
        lib.fa_fwd_splitkv_static.restype = ctypes.c_int
        lib.fa_fwd_splitkv_static.argtypes = [vp, vp, vp, vp, vp] + [ctypes.c_int] * 5 + [
            ctypes.c_float, ctypes.c_int, ctypes.c_int, ctypes.c_int, vp]
        lib.fa_fwd_splitkv_plan.restype = ctypes.c_int
        lib.fa_fwd_splitkv_plan.argtypes = [ctypes.c_int] * 8 + [ctypes.POINTER(FaSplitKvPlan)]
        lib.fa_attn_linear_block.restype = ctypes.c_int
        lib.fa_attn_linear_block.argtypes = [vp] * 7 + [ctypes.c_int] * 6 + [ctypes.c_float] + [ctypes.c_int] * 4 + [vp]
        lib.fa_attn_linear.restype = ctypes.c_int
        lib.fa_attn_linear.argtypes = [vp] * 7 + [ctypes.c_int] * 6 + [ctypes.c_float] + [ctypes.c_int] * 3 + [vp]
        ip = ctypes.POINTER(ctypes.c_int)
        lib.fa_fwd_masked.restype = ctypes.c_int
        lib.fa_fwd_masked.argtypes = [vp, vp, vp, vp, vp] + [ctypes.c_int] * 5 + [
            ctypes.c_float, ctypes.POINTER(FaMask), ctypes.c_int, vp]
        lib.fa_decode_masked.restype = ctypes.c_int
        lib.fa_decode_masked.argtypes = [vp, vp, vp, vp, vp] + [ctypes.c_int] * 4 + [
            ctypes.c_float, ctypes.POINTER(FaMask), ctypes.c_int, ctypes.c_int, vp, ctypes.c_longlong, vp]
        lib.fa_mask_tile_class.restype = ctypes.c_int
        lib.fa_mask_tile_class.argtypes = [ctypes.POINTER(FaMask)] + [ctypes.c_int] * 6
        lib.fa_mask_tile_walk.restype = ctypes.c_int
        lib.fa_mask_tile_walk.argtypes = [ctypes.POINTER(FaMask)] + [ctypes.c_int] * 5 + [ip, ctypes.c_int, ip]
        lib.fa_mask_interior_run.restype = ctypes.c_int
        lib.fa_mask_interior_run.argtypes = [ctypes.POINTER(FaMask)] + [ctypes.c_int] * 7 + [ip, ip]
        lib.fa_set_option.restype = ctypes.c_int
        lib.fa_set_option.argtypes = [ctypes.c_int, ctypes.c_int]
        lib.fa_strerror.restype = ctypes.c_char_p
        lib.fa_strerror.argtypes = [ctypes.c_int]
        lib.fa_version.restype = ctypes.c_int
        lib.fa_version.argtypes = []
        lib.fa_last_hip_error.restype = ctypes.c_int
        lib.fa_last_hip_error.argtypes = []
        _lib = lib
    return _lib


def _addr(x) -> int:
    if x is None:
        return 0
    if isinstance(x, int):
        return x
    if hasattr(x, "data_ptr"):
        return int(x.data_ptr())
    raise TypeError("pass a device address (int) or an object with data_ptr()")


def fa_fwd_raw(q, k, v, o, lse, B, H, Nq, Nk, D, scale, causal, dtype, stream=0) -> int:
    """Call fa_fwd and return its status code unchanged."""
    return load().fa_fwd(_addr(q), _addr(k), _addr(v), _addr(o), _addr(lse), int(B), int(H), int(Nq), int(Nk),
                         int(D), float(scale), int(causal), int(dtype), _addr(stream))


def fa_fwd(q, k, v, o, lse, B, H, Nq, Nk, D, scale, causal, dtype, stream=0) -> None:
    """fa_fwd of include/fa.h; raises FaError on a negative status. Asynchronous on ``stream``."""
    rc = fa_fwd_raw(q, k, v, o, lse, B, H, Nq, Nk, D, scale, causal, dtype, stream)
    if rc != FA_OK:
        raise FaError(rc)


def fa_fwd_plan(B, H, Nq, Nk, D, causal, dtype) -> FaPlan:
    """fa_fwd_plan of include/fa.h (host only, no GPU needed); raises FaError on a bad shape."""
    plan = FaPlan()
    rc = load().fa_fwd_plan(int(B), int(H), int(Nq), int(Nk), int(D), int(causal), int(dtype), ctypes.byref(plan))
    if rc != FA_OK:
        raise FaError(rc)
    return plan


def fa_fwd_splitkv_raw(q, k, v, o, lse, B, H, Nq, Nk, D, scale, causal, dtype, nsplit, workspace, workspace_bytes,
                       stream=0) -> int:
    """Call fa_fwd_splitkv and return its status code unchanged."""
    return load().fa_fwd_splitkv(_addr(q), _addr(k), _addr(v), _addr(o), _addr(lse), int(B), int(H), int(Nq),
                                 int(Nk), int(D), float(scale), int(causal), int(dtype), int(nsplit),
                                 _addr(workspace), int(workspace_bytes), _addr(stream))


def fa_fwd_splitkv(q, k, v, o, lse, B, H, Nq, Nk, D, scale, causal, dtype, nsplit, workspace, workspace_bytes,
                   stream=0) -> None:
    """fa_fwd_splitkv of include/fa.h; raises FaError on a negative status. Asynchronous on ``stream``."""
    rc = fa_fwd_splitkv_raw(q, k, v, o, lse, B, H, Nq, Nk, D, scale, causal, dtype, nsplit, workspace,
                            workspace_bytes, stream)
    if rc != FA_OK:
        raise FaError(rc)


def fa_fwd_splitkv_static_raw(q, k, v, o, lse, B, H, Nq, Nk, D, scale, causal, dtype, nsplit, stream=0) -> int:
    """Call fa_fwd_splitkv_static and return its status code unchanged."""
    return load().fa_fwd_splitkv_static(_addr(q), _addr(k), _addr(v), _addr(o), _addr(lse), int(B), int(H), int(Nq),
                                        int(Nk), int(D), float(scale), int(causal), int(dtype), int(nsplit),
                                        _addr(stream))


def fa_fwd_splitkv_static(q, k, v, o, lse, B, H, Nq, Nk, D, scale, causal, dtype, nsplit, stream=0) -> None:
    """fa_fwd_splitkv_static of include/fa.h; raises FaError on a negative status. Asynchronous on ``stream``."""
    rc = fa_fwd_splitkv_static_raw(q, k, v, o, lse, B, H, Nq, Nk, D, scale, causal, dtype, nsplit, stream)
    if rc != FA_OK:
        raise FaError(rc)


def fa_fwd_splitkv_plan(B, H, Nq, Nk, D, causal, dtype, nsplit=0) -> FaSplitKvPlan:
    """fa_fwd_splitkv_plan of include/fa.h (host only); raises FaError on a bad shape or nsplit."""
    plan = FaSplitKvPlan()
    rc = load().fa_fwd_splitkv_plan(int(B), int(H), int(Nq), int(Nk), int(D), int(causal), int(dtype), int(nsplit),
                                    ctypes.byref(plan))
    if rc != FA_OK:
        raise FaError(rc)
    return plan


def fa_attn_linear_block_raw(q, k, v, w, o, lse, y, B, H, Nq, Nk, D, N, scale, causal, dtype, row_first, row_count,
                             stream=0) -> int:
    """Call fa_attn_linear_block and return its status code unchanged."""
    return load().fa_attn_linear_block(_addr(q), _addr(k), _addr(v), _addr(w), _addr(o), _addr(lse), _addr(y), int(B),
                                       int(H), int(Nq), int(Nk), int(D), int(N), float(scale), int(causal),
                                       int(dtype), int(row_first), int(row_count), _addr(stream))


def fa_attn_linear_block(q, k, v, w, o, lse, y, B, H, Nq, Nk, D, N, scale, causal, dtype, row_first, row_count,
                         stream=0) -> None:
    """fa_attn_linear_block of include/fa.h; raises FaError on a negative status. Asynchronous on ``stream``."""
    rc = fa_attn_linear_block_raw(q, k, v, w, o, lse, y, B, H, Nq, Nk, D, N, scale, causal, dtype, row_first,
                                  row_count, stream)
    if rc != FA_OK:
        raise FaError(rc)


def fa_attn_linear(q, k, v, w, o, lse, y, B, H, Nq, Nk, D, N, scale, causal, dtype, rows_per_block=0, stream=0) -> None:
    """fa_attn_linear of include/fa.h; raises FaError on a negative status. Asynchronous on ``stream``."""
    rc = load().fa_attn_linear(_addr(q), _addr(k), _addr(v), _addr(w), _addr(o), _addr(lse), _addr(y), int(B), int(H),
                               int(Nq), int(Nk), int(D), int(N), float(scale), int(causal), int(dtype),
                               int(rows_per_block), _addr(stream))
    if rc != FA_OK:
        raise FaError(rc)


def _mask(left, right, prefix, kv_len, diag_from_kv_len=0):
    return FaMask(int(left), int(right), int(prefix), int(diag_from_kv_len), _addr(kv_len) or None)


def fa_fwd_masked_raw(q, k, v, o, lse, B, H, Nq, Nk, D, scale, left, right, prefix, kv_len, dtype, stream=0,
                      diag_from_kv_len=0) -> int:
    """Call fa_fwd_masked (mask fields passed one by one) and return its status code unchanged."""
    m = _mask(left, right, prefix, kv_len, diag_from_kv_len)
    return load().fa_fwd_masked(_addr(q), _addr(k), _addr(v), _addr(o), _addr(lse), int(B), int(H), int(Nq),
                                int(Nk), int(D), float(scale), ctypes.byref(m), int(dtype), _addr(stream))


def fa_fwd_masked(q, k, v, o, lse, B, H, Nq, Nk, D, scale, left, right, prefix, kv_len, dtype, stream=0,
                  diag_from_kv_len=0) -> None:
    """fa_fwd_masked of include/fa.h; raises FaError on a negative status. Asynchronous on ``stream``."""
    rc = fa_fwd_masked_raw(q, k, v, o, lse, B, H, Nq, Nk, D, scale, left, right, prefix, kv_len, dtype, stream,
                           diag_from_kv_len)
    if rc != FA_OK:
        raise FaError(rc)


def fa_decode_masked_raw(q, k, v, o, lse, B, H, Nk, D, scale, left, right, prefix, kv_len, dtype, nsplit, workspace,
                         workspace_bytes, stream=0, diag_from_kv_len=0) -> int:
    """Call fa_decode_masked (mask fields passed one by one) and return its status code unchanged."""
    m = _mask(left, right, prefix, kv_len, diag_from_kv_len)
    return load().fa_decode_masked(_addr(q), _addr(k), _addr(v), _addr(o), _addr(lse), int(B), int(H), int(Nk), int(D),
                                   float(scale), ctypes.byref(m), int(dtype), int(nsplit), _addr(workspace),
                                   int(workspace_bytes), _addr(stream))


def fa_decode_masked(q, k, v, o, lse, B, H, Nk, D, scale, left, right, prefix, kv_len, dtype, nsplit, workspace,
                     workspace_bytes, stream=0, diag_from_kv_len=0) -> None:
    """fa_decode_masked of include/fa.h; raises FaError on a negative status. Asynchronous on ``stream``."""
    rc = fa_decode_masked_raw(q, k, v, o, lse, B, H, Nk, D, scale, left, right, prefix, kv_len, dtype, nsplit,
                              workspace, workspace_bytes, stream, diag_from_kv_len)
    if rc != FA_OK:
        raise FaError(rc)


def fa_mask_tile_class(left, right, prefix, kv_len, Nq, Nk, row_first, row_last, key_first, diag_from_kv_len=0) -> int:
    """fa_mask_tile_class of include/fa.h (host only; kv_len is one batch entry's key count)."""
    m = _mask(left, right, prefix, None, diag_from_kv_len)
    rc = load().fa_mask_tile_class(ctypes.byref(m), int(kv_len), int(Nq), int(Nk), int(row_first), int(row_last),
                                   int(key_first))
    if rc < 0:
        raise FaError(rc)
    return rc


def fa_mask_tile_walk(left, right, prefix, kv_len, Nq, Nk, row_first, row_last, diag_from_kv_len=0):
    """fa_mask_tile_walk of include/fa.h (host only): the list of tile indices, in the order walked."""
    m = _mask(left, right, prefix, None, diag_from_kv_len)
    count = ctypes.c_int()
    args = (ctypes.byref(m), int(kv_len), int(Nq), int(Nk), int(row_first), int(row_last))
    rc = load().fa_mask_tile_walk(*args, None, 0, ctypes.byref(count))
    if rc != FA_OK:
        raise FaError(rc)
    tiles = (ctypes.c_int * max(count.value, 1))()
    rc = load().fa_mask_tile_walk(*args, tiles, count.value, ctypes.byref(count))
    if rc != FA_OK:
        raise FaError(rc)
    return list(tiles[:count.value])


def fa_mask_interior_run(left, right, prefix, kv_len, Nq, Nk, wg_row_first, wg_row_last, row_first, row_last, diag_from_kv_len=0):
    """fa_mask_interior_run of include/fa.h (host only): (first, count) in positions of the workgroup's walk."""
    m = _mask(left, right, prefix, None, diag_from_kv_len)
    first, count = ctypes.c_int(), ctypes.c_int()
    rc = load().fa_mask_interior_run(ctypes.byref(m), int(kv_len), int(Nq), int(Nk), int(wg_row_first),
                                     int(wg_row_last), int(row_first), int(row_last), ctypes.byref(first),
                                     ctypes.byref(count))
    if rc != FA_OK:
        raise FaError(rc)
    return first.value, count.value


def fa_set_option(option: int, value: int) -> int:
    """fa_set_option of include/fa.h: returns the previous value; raises FaError for an unknown option or value."""
    rc = load().fa_set_option(int(option), int(value))
    if rc == FA_ERR_OPTION:
        raise FaError(rc)
    return rc


def fa_strerror(code: int) -> str:
    return load().fa_strerror(int(code)).decode()


def fa_version() -> int:
    return load().fa_version()


def fa_last_hip_error() -> int:
    return load().fa_last_hip_error()
