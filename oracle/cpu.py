"""ctypes binding of the C oracle (kmeans_oracle.c) plus the closed-form size accounting of Eq. 1.

TEST INFRASTRUCTURE, NOT THE PRODUCT: argument marshalling for numpy arrays only.
"""
from __future__ import annotations

import ctypes
import math
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "kmeans_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (plain -O2, OpenMP for the loop over vectors)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99", "-Wall", "-Wextra",
             "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        i64, i32, vp = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p
        lib.oracle_threads.restype = ctypes.c_int
        lib.oracle_assign_top2.argtypes = [vp, i64, i32, vp, i64, vp, vp, vp, vp]
        lib.oracle_assign_top2.restype = None
        lib.oracle_update.argtypes = [vp, i64, i32, vp, i64, vp, vp, vp]
        lib.oracle_update.restype = None
        lib.oracle_inertia.argtypes = [vp, i64, i32, vp, vp]
        lib.oracle_inertia.restype = ctypes.c_double
        lib.oracle_decode.argtypes = [vp, i32, vp, i64, vp]
        lib.oracle_decode.restype = None
        lib.oracle_kmeans_fit.argtypes = [vp, i64, i32, i64, i32, vp, vp, vp, vp, vp]
        lib.oracle_kmeans_fit.restype = None
        _lib = lib
    return _lib


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def _u32(a):
    return np.ascontiguousarray(a, dtype=np.uint32)


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def threads() -> int:
    return int(_load().oracle_threads())


def assign_top2(X, C):
    """E-step with runner-up: returns (k1 uint32[N], D1 f64[N], k2 uint32[N], D2 f64[N])."""
    X, C = _f32(X), _f32(C)
    N, d = X.shape
    K = C.shape[0]
    assert C.shape[1] == d
    k1 = np.empty(N, np.uint32)
    k2 = np.empty(N, np.uint32)
    D1 = np.empty(N, np.float64)
    D2 = np.empty(N, np.float64)
    _load().oracle_assign_top2(_p(X), N, d, _p(C), K, _p(k1), _p(D1), _p(k2), _p(D2))
    return k1, D1, k2, D2


def update(X, idx, prev):
    """M-step: returns (centroids f32[K,d], counts uint32[K]); empty clusters keep prev."""
    X, prev, idx = _f32(X), _f32(prev), _u32(idx)
    N, d = X.shape
    K = prev.shape[0]
    assert idx.shape == (N,) and (N == 0 or int(idx.max()) < K)
    out = np.empty_like(prev)
    counts = np.empty(K, np.uint32)
    _load().oracle_update(_p(X), N, d, _p(idx), K, _p(prev), _p(out), _p(counts))
    return out, counts


def inertia(X, C, idx) -> float:
    X, C, idx = _f32(X), _f32(C), _u32(idx)
    N, d = X.shape
    assert N == 0 or int(idx.max()) < C.shape[0]
    return float(_load().oracle_inertia(_p(X), N, d, _p(C), _p(idx)))


def decode(C, idx):
    C, idx = _f32(C), _u32(idx)
    K, d = C.shape
    N = idx.shape[0]
    assert N == 0 or int(idx.max()) < K
    out = np.empty((N, d), np.float32)
    _load().oracle_decode(_p(C), d, _p(idx), N, _p(out))
    return out


def kmeans_fit(X, C0, iters: int):
    """Returns (centroids f32[K,d], idx uint32[N], inertia float, history f64[iters+1])."""
    X, C0 = _f32(X), _f32(C0)
    N, d = X.shape
    K = C0.shape[0]
    C = np.empty_like(C0)
    idx = np.empty(N, np.uint32)
    J = ctypes.c_double(0.0)
    hist = np.empty(iters + 1, np.float64)
    _load().oracle_kmeans_fit(_p(X), N, d, K, iters, _p(C0), _p(C), _p(idx), ctypes.byref(J), _p(hist))
    return C, idx, float(J.value), hist


# ---- size accounting (Section 3.2, Eq. 1) -------------------------------------------------------

def parameter_counts(d_in: int, d_out: int, g: int, n: int):
    """(#codes k, #codebook parameters g*n) for one d_in x d_out matrix; k = d_in*d_out/g."""
    return d_in * d_out / g, g * n


def bits_per_parameter(d_in: int, d_out: int, g: int, n: int) -> float:
    """Eq. 1: 16-bit codes and a 16-bit codebook, (16k + 16gn)/(d_in d_out)."""
    k, cb = parameter_counts(d_in, d_out, g, n)
    return (16.0 * k + 16.0 * cb) / (d_in * d_out)


def code_bits_per_weight(K: int, d: int) -> float:
    """Packed-code bits only: each length-d vector costs log2(K) bits."""
    return math.log2(K) / d
