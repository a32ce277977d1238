"""ctypes loader for the CPU oracle (oracle/attn_ref.cpp).

TEST INFRASTRUCTURE ONLY.  May be imported from tests/, from the smoke check and
from the benchmark's cpu_baseline leg; never from the product package.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "attn_ref.cpp")
_SRCS = [_SRC, os.path.join(_HERE, "gemm_ref.cpp")]
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with the host compiler (no HIP involved)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < max(os.path.getmtime(f) for f in _SRCS)
    if force or stale:
        subprocess.check_call(["g++", "-O2", "-std=c++17", "-fPIC", "-shared", "-pthread",
                               "-o", _LIB, *_SRCS])
    return _LIB


def lib():
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        u16p = ctypes.POINTER(ctypes.c_uint16)
        f64p = ctypes.POINTER(ctypes.c_double)
        L.attn_ref_f64.restype = ctypes.c_int
        L.attn_ref_f64.argtypes = [u16p, u16p, u16p, f64p, f64p,
                                   ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                   ctypes.c_int, ctypes.c_double, ctypes.c_int,
                                   ctypes.POINTER(ctypes.c_longlong), ctypes.c_longlong,
                                   ctypes.c_int, ctypes.POINTER(ctypes.c_int)]
        L.attn_ref_probs_f64.restype = ctypes.c_int
        L.attn_ref_probs_f64.argtypes = [u16p, u16p, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                         ctypes.c_int, ctypes.c_int, ctypes.c_double,
                                         ctypes.c_int, ctypes.c_longlong, f64p]
        L.gemm_lrelu_ref_f64.restype = ctypes.c_int
        L.gemm_lrelu_ref_f64.argtypes = [u16p, u16p, f64p, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                         ctypes.c_double, ctypes.c_int, ctypes.c_int, ctypes.POINTER(ctypes.c_int)]
        L.attn_ref_decode.restype = ctypes.c_double
        L.attn_ref_decode.argtypes = [ctypes.c_uint16, ctypes.c_int]
        _lib = L
    return _lib


def _u16(a):
    a = np.ascontiguousarray(a)
    if a.dtype != np.uint16:
        raise TypeError("inputs must be uint16 bit patterns")
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16))


def attn_ref(q, k, v, causal: bool, scale: float, dtype: int, rows=None, nthreads: int = 0):
    """Run the oracle.  q, k, v: uint16 [B,H,N,d].  Returns (O, lse, threads_used):
    O float64 [B,H,N,d] and lse float64 [B,H,N], or [nrows,d] / [nrows] when a
    row subset (flattened (b*H+h)*N+i indices) is given."""
    q, qp = _u16(q)
    k, kp = _u16(k)
    v, vp = _u16(v)
    if q.ndim != 4 or k.shape != q.shape or v.shape != q.shape:
        raise ValueError("q, k, v must share a [B,H,N,d] shape")
    B, H, N, d = q.shape
    if rows is None:
        out = np.empty((B, H, N, d), dtype=np.float64)
        lse = np.empty((B, H, N), dtype=np.float64)
        rp, nrows = None, 0
    else:
        rows = np.ascontiguousarray(rows, dtype=np.int64)
        out = np.empty((rows.size, d), dtype=np.float64)
        lse = np.empty((rows.size,), dtype=np.float64)
        rp, nrows = rows.ctypes.data_as(ctypes.POINTER(ctypes.c_longlong)), rows.size
    used = ctypes.c_int(0)
    rc = lib().attn_ref_f64(qp, kp, vp, out.ctypes.data_as(ctypes.POINTER(ctypes.c_double)),
                            lse.ctypes.data_as(ctypes.POINTER(ctypes.c_double)),
                            B, H, N, d, int(bool(causal)), float(scale), int(dtype),
                            rp, nrows, int(nthreads), ctypes.byref(used))
    if rc != 0:
        raise ValueError(f"attn_ref_f64 rejected its arguments (rc={rc})")
    return out, lse, used.value


def attn_ref_probs(q, k, causal: bool, scale: float, dtype: int, row: int):
    """Normalised softmax row P[row, :] (float64, length N)."""
    q, qp = _u16(q)
    k, kp = _u16(k)
    B, H, N, d = q.shape
    probs = np.empty((N,), dtype=np.float64)
    rc = lib().attn_ref_probs_f64(qp, kp, B, H, N, d, int(bool(causal)), float(scale), int(dtype),
                                  int(row), probs.ctypes.data_as(ctypes.POINTER(ctypes.c_double)))
    if rc != 0:
        raise ValueError(f"attn_ref_probs_f64 rejected its arguments (rc={rc})")
    return probs


def decode(bits: int, dtype: int) -> float:
    return lib().attn_ref_decode(int(bits), int(dtype))


def gemm_lrelu_ref(a, b, slope: float, dtype: int, nthreads: int = 0):
    """C = leaky_relu(A B) in float64.  a: uint16 [M,K], b: uint16 [K,N].  Returns (C [M,N], threads_used)."""
    a, ap = _u16(a)
    b, bp = _u16(b)
    if a.ndim != 2 or b.ndim != 2 or a.shape[1] != b.shape[0]:
        raise ValueError("a must be [M,K] and b [K,N]")
    M, K = a.shape
    N = b.shape[1]
    out = np.empty((M, N), dtype=np.float64)
    used = ctypes.c_int(0)
    rc = lib().gemm_lrelu_ref_f64(ap, bp, out.ctypes.data_as(ctypes.POINTER(ctypes.c_double)), M, N, K,
                                  float(slope), int(dtype), int(nthreads), ctypes.byref(used))
    if rc != 0:
        raise ValueError(f"gemm_lrelu_ref_f64 rejected its arguments (rc={rc})")
    return out, used.value
