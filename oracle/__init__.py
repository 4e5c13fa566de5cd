"""ctypes front end of the CPU oracle (oracle/mmm_oracle.c).

TEST INFRASTRUCTURE ONLY: used by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  The product path never imports this package and
this package never imports the product path.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mmm_oracle.c")
_LIB = os.path.join(_HERE, "libmmm_oracle.so")

PRED_NONZERO, PRED_GT, PRED_ABS_GT = 0, 1, 2


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, no fast-math, OpenMP over rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _L():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.oracle_threads.restype = ctypes.c_int
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def _is64(a) -> bool:
    """Double-precision inputs take the *_f64 functions (same definitions, long double accumulation)."""
    return isinstance(a, np.ndarray) and a.dtype == np.float64


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def _u64(a) -> Optional[np.ndarray]:
    return None if a is None else np.ascontiguousarray(a, dtype=np.uint64)


def threads() -> int:
    return int(_L().oracle_threads())


def set_threads(n: int) -> None:
    _L().oracle_set_threads(int(n))


def a_bits(X, pred=PRED_NONZERO, threshold=0.0, keep_bits=None) -> np.ndarray:
    f64 = _is64(X)
    X = _f64(X) if f64 else _f32(X)
    M, K = X.shape
    out = np.empty((M, (K + 63) // 64), dtype=np.uint64)
    kb = _u64(keep_bits)
    if kb is not None:
        assert kb.shape == out.shape
    (_L().oracle_a_bits_f64 if f64 else _L().oracle_a_bits)(_p(X), ctypes.c_int64(M), ctypes.c_int64(K), ctypes.c_int64(K),
                       ctypes.c_int(pred), ctypes.c_float(threshold), _p(kb), _p(out))
    return out


def b_bits(Y, bw: int, keep_rows=None, keep_blocks=None) -> np.ndarray:
    f64 = _is64(Y)
    Y = _f64(Y) if f64 else _f32(Y)
    K, N = Y.shape
    assert N % bw == 0
    NB = N // bw
    out = np.empty((K, (NB + 63) // 64), dtype=np.uint64)
    kr, kb = _u64(keep_rows), _u64(keep_blocks)
    if kr is not None:
        assert kr.size == (K + 63) // 64
    if kb is not None:
        assert kb.shape == out.shape
    (_L().oracle_b_bits_f64 if f64 else _L().oracle_b_bits)(_p(Y), ctypes.c_int64(K), ctypes.c_int64(N), ctypes.c_int64(N),
                       ctypes.c_int64(bw), _p(kr), _p(kb), _p(out))
    return out


def materialize_a(X, abits) -> np.ndarray:
    X = _f32(X)
    M, K = X.shape
    A = np.empty((M, K), dtype=np.float32)
    _L().oracle_materialize_a(_p(X), ctypes.c_int64(M), ctypes.c_int64(K), ctypes.c_int64(K),
                              _p(_u64(abits)), _p(A))
    return A


def materialize_b(Y, bw: int, bbits) -> np.ndarray:
    Y = _f32(Y)
    K, N = Y.shape
    B = np.empty((K, N), dtype=np.float32)
    _L().oracle_materialize_b(_p(Y), ctypes.c_int64(K), ctypes.c_int64(N), ctypes.c_int64(N),
                              ctypes.c_int64(bw), _p(_u64(bbits)), _p(B))
    return B


def dense_ref(A, B) -> np.ndarray:
    A, B = _f32(A), _f32(B)
    M, K = A.shape
    K2, N = B.shape
    assert K == K2
    C = np.empty((M, N), dtype=np.float64)
    _L().oracle_dense_ref(_p(A), _p(B), ctypes.c_int64(M), ctypes.c_int64(K), ctypes.c_int64(N), _p(C))
    return C


def mmm(X, Y, abits, bbits, bw: int, C_in=None, want_mag: bool = True, rows=None):
    """Returns (C [M,N], absAB fp64 [M,N] or None); C is fp32, or fp64 for double inputs.  With C_in the product is
    added to it (accumulate mode).  rows=(r0,r1) computes only those rows (the others are left as C_in or zero)."""
    f64 = _is64(X)
    assert f64 == _is64(Y)
    X, Y = (_f64(X), _f64(Y)) if f64 else (_f32(X), _f32(Y))
    ct = np.float64 if f64 else np.float32
    M, K = X.shape
    K2, N = Y.shape
    assert K == K2 and N % bw == 0
    acc = C_in is not None
    C = np.array(C_in, dtype=ct, order="C", copy=True) if acc else np.zeros((M, N), ct)
    mag = np.zeros((M, N), dtype=np.float64) if want_mag else None
    r0, r1 = (0, M) if rows is None else rows
    (_L().oracle_mmm_rows_f64 if f64 else _L().oracle_mmm_rows)(
        _p(X), ctypes.c_int64(K), _p(Y), ctypes.c_int64(N),
        _p(_u64(abits)), _p(_u64(bbits)),
        ctypes.c_int64(M), ctypes.c_int64(K), ctypes.c_int64(N), ctypes.c_int64(bw),
        ctypes.c_int64(r0), ctypes.c_int64(r1),
        _p(C), ctypes.c_int64(N), _p(mag), ctypes.c_int(1 if acc else 0))
    return C, mag


def mmm_element(X, Y, abits, bbits, bw: int, i: int, j: int):
    X, Y = _f32(X), _f32(Y)
    K, N = Y.shape
    c, m = ctypes.c_double(), ctypes.c_double()
    _L().oracle_mmm_element(_p(X), ctypes.c_int64(X.shape[1]), _p(Y), ctypes.c_int64(N),
                            _p(_u64(abits)), _p(_u64(bbits)),
                            ctypes.c_int64(K), ctypes.c_int64(N), ctypes.c_int64(bw),
                            ctypes.c_int64(i), ctypes.c_int64(j), ctypes.byref(c), ctypes.byref(m))
    return c.value, m.value


def counts(abits, bbits, M: int, K: int, N: int, bw: int):
    na, nb, mac = ctypes.c_uint64(), ctypes.c_uint64(), ctypes.c_uint64()
    _L().oracle_counts(_p(_u64(abits)), _p(_u64(bbits)), ctypes.c_int64(M), ctypes.c_int64(K),
                       ctypes.c_int64(N), ctypes.c_int64(bw),
                       ctypes.byref(na), ctypes.byref(nb), ctypes.byref(mac))
    return na.value, nb.value, mac.value


def run_workload(w, rows=None, want_mag: bool = True):
    """Maps and product for a mmm_synth.Workload (duck-typed; no import needed)."""
    ab = a_bits(w.X, w.pred, w.threshold, w.keep_a)
    bb = b_bits(w.Y, w.bw, w.keep_rows, w.keep_blocks)
    C, mag = mmm(w.X, w.Y, ab, bb, w.bw, want_mag=want_mag, rows=rows)
    return ab, bb, C, mag
