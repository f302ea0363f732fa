"""CPU fp64 oracle for exact attention forward -- TEST INFRASTRUCTURE ONLY.

Thin ctypes wrapper around ``fa_oracle.c`` (plain three-loop attention, the
"standard attention" of FastAttention section 5.1).  Only tests, the smoke check
and the benchmark's ``cpu_baseline`` leg may import this package; the GPU library
never does, and this package never imports the GPU library.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fa_oracle.c")
_LIB = os.path.join(_HERE, "libfa_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile fa_oracle.c with gcc (-O2, no fast-math, OpenMP) into libfa_oracle.so."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        cmd = ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra", _SRC, "-o", _LIB, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        u16p = ctypes.POINTER(ctypes.c_uint16)
        f64p = ctypes.POINTER(ctypes.c_double)
        i64p = ctypes.POINTER(ctypes.c_int64)
        lib.fa_oracle_fwd.restype = ctypes.c_int
        lib.fa_oracle_fwd.argtypes = [u16p, u16p, u16p, f64p, f64p] + [ctypes.c_int] * 5 + [
            ctypes.c_double, ctypes.c_int, ctypes.c_int, i64p, ctypes.c_int64, ctypes.c_int]
        lib.fa_oracle_probs.restype = ctypes.c_int
        lib.fa_oracle_probs.argtypes = [u16p, u16p, f64p] + [ctypes.c_int] * 5 + [
            ctypes.c_double, ctypes.c_int, ctypes.c_int, ctypes.c_int64]
        lib.fa_oracle_fwd_masked.restype = ctypes.c_int
        lib.fa_oracle_fwd_masked.argtypes = [u16p, u16p, u16p, f64p, f64p] + [ctypes.c_int] * 5 + [
            ctypes.c_double, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.POINTER(ctypes.c_int32),
            ctypes.c_int, ctypes.c_int, i64p, ctypes.c_int64, ctypes.c_int]
        lib.fa_oracle_attn_linear.restype = ctypes.c_int
        lib.fa_oracle_attn_linear.argtypes = [u16p, u16p, u16p, u16p, f64p] + [ctypes.c_int] * 6 + [
            ctypes.c_double, ctypes.c_int, ctypes.c_int, i64p, ctypes.c_int64, ctypes.c_int]
        lib.fa_oracle_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def _u16(a, shape):
    a = np.ascontiguousarray(a)
    if a.dtype != np.uint16:
        raise TypeError("inputs are uint16 bit patterns of fp16/bf16 values")
    if tuple(a.shape) != tuple(shape):
        raise ValueError(f"expected shape {shape}, got {a.shape}")
    return a


def _ptr(a, ctype):
    return a.ctypes.data_as(ctypes.POINTER(ctype))


def num_threads() -> int:
    return _load().fa_oracle_num_threads()


def attention_fwd(q_bits, k_bits, v_bits, scale, causal, dtype, rows=None, nthreads=0):
    """Oracle forward.

    q_bits [B,H,Nq,D], k_bits/v_bits [B,H,Nk,D]: uint16 bit patterns (dtype 0 = fp16,
    1 = bf16).  Returns (o, lse) in fp64: shapes [B,H,Nq,D], [B,H,Nq] when ``rows`` is
    None, else [len(rows),D], [len(rows)] for the flat row ids (b*H+h)*Nq+i listed.
    """
    lib = _load()
    B, H, Nq, D = q_bits.shape
    Nk = k_bits.shape[2]
    q = _u16(q_bits, (B, H, Nq, D))
    k = _u16(k_bits, (B, H, Nk, D))
    v = _u16(v_bits, (B, H, Nk, D))
    if rows is None:
        o = np.empty((B, H, Nq, D), dtype=np.float64)
        lse = np.empty((B, H, Nq), dtype=np.float64)
        rp, nr = None, 0
    else:
        rows = np.ascontiguousarray(rows, dtype=np.int64)
        o = np.empty((rows.size, D), dtype=np.float64)
        lse = np.empty((rows.size,), dtype=np.float64)
        rp, nr = _ptr(rows, ctypes.c_int64), rows.size
    rc = lib.fa_oracle_fwd(_ptr(q, ctypes.c_uint16), _ptr(k, ctypes.c_uint16), _ptr(v, ctypes.c_uint16),
                           _ptr(o, ctypes.c_double), _ptr(lse, ctypes.c_double), B, H, Nq, Nk, D,
                           float(scale), int(bool(causal)), int(dtype), rp, nr, int(nthreads))
    if rc != 0:
        raise RuntimeError(f"fa_oracle_fwd failed with code {rc}")
    return o, lse


def attention_fwd_masked(q_bits, k_bits, v_bits, scale, dtype, left=-1, right=-1, prefix=0, kv_len=None, rows=None,
                         nthreads=0, diag_from_kv_len=False):
    """Oracle forward under a mask given by a descriptor: key j is visible to row i of batch entry b iff
    ``j < kv_len[b]`` (all keys if ``kv_len`` is None) and (``j < prefix`` or
    ``diag - left <= j <= diag + right``), ``diag = i + Nk - Nq``, or ``i + kv_len[b] - Nq`` with
    ``diag_from_kv_len`` (the queries are the last Nq positions of each entry's own sequence); a negative
    ``left`` / ``right`` is no limit.  Same shapes and return values as :func:`attention_fwd`."""
    lib = _load()
    B, H, Nq, D = q_bits.shape
    Nk = k_bits.shape[2]
    q = _u16(q_bits, (B, H, Nq, D))
    k = _u16(k_bits, (B, H, Nk, D))
    v = _u16(v_bits, (B, H, Nk, D))
    if rows is None:
        o = np.empty((B, H, Nq, D), dtype=np.float64)
        lse = np.empty((B, H, Nq), dtype=np.float64)
        rp, nr = None, 0
    else:
        rows = np.ascontiguousarray(rows, dtype=np.int64)
        o = np.empty((rows.size, D), dtype=np.float64)
        lse = np.empty((rows.size,), dtype=np.float64)
        rp, nr = _ptr(rows, ctypes.c_int64), rows.size
    if kv_len is None:
        lp = None
    else:
        kv_len = np.ascontiguousarray(kv_len, dtype=np.int32)
        if kv_len.shape != (B,):
            raise ValueError("kv_len must have one entry per batch element")
        lp = _ptr(kv_len, ctypes.c_int32)
    rc = lib.fa_oracle_fwd_masked(_ptr(q, ctypes.c_uint16), _ptr(k, ctypes.c_uint16), _ptr(v, ctypes.c_uint16),
                                  _ptr(o, ctypes.c_double), _ptr(lse, ctypes.c_double), B, H, Nq, Nk, D,
                                  float(scale), int(left), int(right), int(prefix), lp, int(bool(diag_from_kv_len)),
                                  int(dtype), rp, nr, int(nthreads))
    if rc != 0:
        raise RuntimeError(f"fa_oracle_fwd_masked failed with code {rc}")
    return o, lse


def attention_linear(q_bits, k_bits, v_bits, w_bits, scale, causal, dtype, rows=None, nthreads=0):
    """Attention followed by the output projection: y[b,i,:] = concat_h(o[b,h,i,:]) @ w, everything in fp64.

    w_bits [H*D, N] uint16 bit patterns.  Returns y [B,Nq,N], or [len(rows),N] for the flat token ids b*Nq+i."""
    lib = _load()
    B, H, Nq, D = q_bits.shape
    Nk = k_bits.shape[2]
    q = _u16(q_bits, (B, H, Nq, D))
    k = _u16(k_bits, (B, H, Nk, D))
    v = _u16(v_bits, (B, H, Nk, D))
    w = np.ascontiguousarray(w_bits)
    if w.dtype != np.uint16 or w.ndim != 2 or w.shape[0] != H * D:
        raise ValueError("w_bits must be uint16 [H*D, N]")
    N = w.shape[1]
    if rows is None:
        y = np.empty((B, Nq, N), dtype=np.float64)
        rp, nr = None, 0
    else:
        rows = np.ascontiguousarray(rows, dtype=np.int64)
        y = np.empty((rows.size, N), dtype=np.float64)
        rp, nr = _ptr(rows, ctypes.c_int64), rows.size
    rc = lib.fa_oracle_attn_linear(_ptr(q, ctypes.c_uint16), _ptr(k, ctypes.c_uint16), _ptr(v, ctypes.c_uint16),
                                   _ptr(w, ctypes.c_uint16), _ptr(y, ctypes.c_double), B, H, Nq, Nk, D, N,
                                   float(scale), int(bool(causal)), int(dtype), rp, nr, int(nthreads))
    if rc != 0:
        raise RuntimeError(f"fa_oracle_attn_linear failed with code {rc}")
    return y


def attention_probs(q_bits, k_bits, scale, causal, dtype, row):
    """Normalised attention probabilities (length Nk, zeros where masked) of one flat row id."""
    lib = _load()
    B, H, Nq, D = q_bits.shape
    Nk = k_bits.shape[2]
    q = _u16(q_bits, (B, H, Nq, D))
    k = _u16(k_bits, (B, H, Nk, D))
    p = np.empty((Nk,), dtype=np.float64)
    rc = lib.fa_oracle_probs(_ptr(q, ctypes.c_uint16), _ptr(k, ctypes.c_uint16), _ptr(p, ctypes.c_double),
                             B, H, Nq, Nk, D, float(scale), int(bool(causal)), int(dtype), int(row))
    if rc != 0:
        raise RuntimeError(f"fa_oracle_probs failed with code {rc}")
    return p
