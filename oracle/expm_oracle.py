"""ctypes binding of the plain-C oracle in expm_oracle.c.

TEST INFRASTRUCTURE ONLY.  Imported by tests/, by the smoke check and by the
benchmark's CPU-baseline leg; never by the GPU package.  It marshals numpy
arrays into the C routines and does no arithmetic of its own beyond widening
fp32 inputs to fp64 (exact).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "expm_oracle.c")
_LIB = os.path.join(_HERE, "libexpm_oracle.so")
_lib = None


def build_oracle(force: bool = False) -> str:
    """Compile expm_oracle.c with gcc (generic x86-64, no FMA contraction, OpenMP)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O3", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-shared", "-fPIC",
               "-std=c11", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB):
            build_oracle()
        lib = ctypes.CDLL(_LIB)
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int)
        lib.oracle_norm1.restype = ctypes.c_double
        lib.oracle_norm1.argtypes = [dp, ctypes.c_int]
        lib.oracle_matmul.restype = None
        lib.oracle_matmul.argtypes = [dp, dp, dp, ctypes.c_int]
        lib.oracle_b16.restype = ctypes.c_double
        lib.oracle_b16.argtypes = []
        lib.oracle_select_from_norms.restype = None
        lib.oracle_select_from_norms.argtypes = [ctypes.c_double, ctypes.c_double, ctypes.c_double, ip, ip]
        lib.oracle_select.restype = ctypes.c_int
        lib.oracle_select.argtypes = [dp, ctypes.c_int, ctypes.c_double, ip, ip, dp, dp, ip]
        lib.oracle_expm.restype = ctypes.c_int
        lib.oracle_expm.argtypes = [dp, ctypes.c_int, ctypes.c_double, dp, ip, ip, dp, dp, ip]
        lib.oracle_expm_batch.restype = ctypes.c_int
        lib.oracle_expm_batch.argtypes = [dp, ctypes.c_int, ctypes.c_int, ctypes.c_double, dp,
                                          ip, ip, dp, dp, ip, ctypes.c_int]
        lib.oracle_select_ps_from_norms.restype = None
        lib.oracle_select_ps_from_norms.argtypes = [ctypes.c_double] * 5 + [ip, ip]
        lib.oracle_select_ps.restype = ctypes.c_int
        lib.oracle_select_ps.argtypes = [dp, ctypes.c_int, ctypes.c_double, ip, ip, dp, ip]
        lib.oracle_expm_ps_batch.restype = ctypes.c_int
        lib.oracle_expm_ps_batch.argtypes = [dp, ctypes.c_int, ctypes.c_int, ctypes.c_double, dp,
                                             ip, ip, dp, ip, ctypes.c_int]
        lib.oracle_expm_baseline_batch.restype = ctypes.c_int
        lib.oracle_expm_baseline_batch.argtypes = [dp, ctypes.c_int, ctypes.c_int, ctypes.c_double, dp,
                                                   ip, ip, dp, ip, ctypes.c_int]
        lib.oracle_lowrank_select_from_norm.restype = None
        lib.oracle_lowrank_select_from_norm.argtypes = [ctypes.c_double, ctypes.c_double, ip, ip]
        lib.oracle_lowrank_batch.restype = ctypes.c_int
        lib.oracle_lowrank_batch.argtypes = [dp, dp, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_double, dp,
                                             ip, ip, dp, ip, ctypes.c_int]
        lib.oracle_max_threads.restype = ctypes.c_int
        lib.oracle_max_threads.argtypes = []
        lib.oracle_expm_forced.restype = ctypes.c_int
        lib.oracle_expm_forced.argtypes = [dp, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, dp, ctypes.c_int]
        lib.oracle_lowrank_forced.restype = ctypes.c_int
        lib.oracle_lowrank_forced.argtypes = [dp, dp, ctypes.c_int, ctypes.c_int, ctypes.c_int, dp]
        lib.oracle_matmul_threads.restype = ctypes.c_int
        lib.oracle_matmul_threads.argtypes = [dp, dp, dp, ctypes.c_int, ctypes.c_int]
        _lib = lib
    return _lib


def _dptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _iptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int))


def _as_f64(W) -> np.ndarray:
    a = np.ascontiguousarray(np.asarray(W), dtype=np.float64)
    return a


def unit_roundoff(dtype) -> float:
    """u of the working precision the tolerance defaults to (Sec. 3.2: eps >= u)."""
    return 2.0 ** -24 if np.dtype(dtype) == np.float32 else 2.0 ** -53


def oracle_norm1(W) -> float:
    a = _as_f64(W)
    assert a.ndim == 2 and a.shape[0] == a.shape[1]
    return float(_load().oracle_norm1(_dptr(a), a.shape[0]))


def oracle_matmul(A, B) -> np.ndarray:
    a, b = _as_f64(A), _as_f64(B)
    n = a.shape[0]
    assert a.shape == (n, n) and b.shape == (n, n)
    c = np.empty((n, n), dtype=np.float64)
    _load().oracle_matmul(_dptr(a), _dptr(b), _dptr(c), n)
    return c


def oracle_b16() -> float:
    return float(_load().oracle_b16())


def oracle_select_from_norms(n1: float, n2: float, tol: float) -> Tuple[int, int]:
    m, s = ctypes.c_int(0), ctypes.c_int(0)
    _load().oracle_select_from_norms(float(n1), float(n2), float(tol), ctypes.byref(m), ctypes.byref(s))
    return m.value, s.value


def oracle_select(W, tol: float):
    """Algorithm 4 for one matrix -> dict(m, s, n1, n2, near)."""
    a = _as_f64(W)
    n = a.shape[0]
    m, s, near = ctypes.c_int(0), ctypes.c_int(0), ctypes.c_int(0)
    n1, n2 = ctypes.c_double(0), ctypes.c_double(0)
    rc = _load().oracle_select(_dptr(a), n, float(tol), ctypes.byref(m), ctypes.byref(s),
                               ctypes.byref(n1), ctypes.byref(n2), ctypes.byref(near))
    if rc != 0:
        raise MemoryError("oracle_select")
    return dict(m=m.value, s=s.value, n1=n1.value, n2=n2.value, near=bool(near.value))


def oracle_expm(W, tol: float):
    """Algorithm 2 for one matrix -> (X fp64, dict(m, s, n1, n2, near))."""
    a = _as_f64(W)
    n = a.shape[0]
    X = np.empty((n, n), dtype=np.float64)
    m, s, near = ctypes.c_int(0), ctypes.c_int(0), ctypes.c_int(0)
    n1, n2 = ctypes.c_double(0), ctypes.c_double(0)
    rc = _load().oracle_expm(_dptr(a), n, float(tol), _dptr(X), ctypes.byref(m), ctypes.byref(s),
                             ctypes.byref(n1), ctypes.byref(n2), ctypes.byref(near))
    if rc != 0:
        raise MemoryError("oracle_expm")
    return X, dict(m=m.value, s=s.value, n1=n1.value, n2=n2.value, near=bool(near.value))


def oracle_expm_batch(W, tol: float, threads: int = 0):
    """Batch [b][n][n] -> (X fp64 [b][n][n], dict of arrays m, s, n1, n2, near, threads)."""
    a = _as_f64(W)
    assert a.ndim == 3 and a.shape[1] == a.shape[2]
    b, n = a.shape[0], a.shape[1]
    X = np.empty_like(a)
    m = np.zeros(b, dtype=np.int32)
    s = np.zeros(b, dtype=np.int32)
    near = np.zeros(b, dtype=np.int32)
    n1 = np.zeros(b, dtype=np.float64)
    n2 = np.zeros(b, dtype=np.float64)
    used = 0
    if b > 0 and n > 0:
        used = _load().oracle_expm_batch(_dptr(a), n, b, float(tol), _dptr(X), _iptr(m), _iptr(s),
                                         _dptr(n1), _dptr(n2), _iptr(near), int(threads))
        if used < 0:
            raise MemoryError("oracle_expm_batch")
    return X, dict(m=m, s=s, n1=n1, n2=n2, near=near.astype(bool), threads=used)


def oracle_select_ps_from_norms(n1: float, n2: float, n3: float, n4: float, tol: float) -> Tuple[int, int]:
    """Algorithm 3 on the norms of W, W^2, W^3, W^4."""
    m, s = ctypes.c_int(0), ctypes.c_int(0)
    _load().oracle_select_ps_from_norms(float(n1), float(n2), float(n3), float(n4), float(tol),
                                        ctypes.byref(m), ctypes.byref(s))
    return m.value, s.value


def oracle_select_ps(W, tol: float):
    """Algorithm 3 for one matrix -> dict(m, s, norms[4], near)."""
    a = _as_f64(W)
    n = a.shape[0]
    m, s, near = ctypes.c_int(0), ctypes.c_int(0), ctypes.c_int(0)
    norms = np.zeros(4, dtype=np.float64)
    rc = _load().oracle_select_ps(_dptr(a), n, float(tol), ctypes.byref(m), ctypes.byref(s), _dptr(norms),
                                  ctypes.byref(near))
    if rc != 0:
        raise MemoryError("oracle_select_ps")
    return dict(m=m.value, s=s.value, norms=norms, near=bool(near.value))


def oracle_expm_ps_batch(W, tol: float, threads: int = 0):
    """Paterson-Stockmeyer variant on a batch -> (X fp64, dict of arrays m, s, norms[b][4], near, threads)."""
    a = _as_f64(W)
    if a.ndim == 2:
        a = a[None]
    assert a.ndim == 3 and a.shape[1] == a.shape[2]
    b, n = a.shape[0], a.shape[1]
    X = np.empty_like(a)
    m = np.zeros(b, dtype=np.int32)
    s = np.zeros(b, dtype=np.int32)
    near = np.zeros(b, dtype=np.int32)
    norms = np.zeros((b, 4), dtype=np.float64)
    used = 0
    if b > 0 and n > 0:
        used = _load().oracle_expm_ps_batch(_dptr(a), n, b, float(tol), _dptr(X), _iptr(m), _iptr(s),
                                            _dptr(norms), _iptr(near), int(threads))
        if used < 0:
            raise MemoryError("oracle_expm_ps_batch")
    return X, dict(m=m, s=s, norms=norms, near=near.astype(bool), threads=used)


def oracle_expm_baseline_batch(W, tol: float, threads: int = 0):
    """The paper's baseline (its Algorithm 1) on a batch -> (X fp64, dict of arrays m, s, n1, near, threads)."""
    a = _as_f64(W)
    if a.ndim == 2:
        a = a[None]
    assert a.ndim == 3 and a.shape[1] == a.shape[2]
    b, n = a.shape[0], a.shape[1]
    X = np.empty_like(a)
    m = np.zeros(b, dtype=np.int32)
    s = np.zeros(b, dtype=np.int32)
    near = np.zeros(b, dtype=np.int32)
    n1 = np.zeros(b, dtype=np.float64)
    used = 0
    if b > 0 and n > 0:
        used = _load().oracle_expm_baseline_batch(_dptr(a), n, b, float(tol), _dptr(X), _iptr(m), _iptr(s),
                                                  _dptr(n1), _iptr(near), int(threads))
        if used < 0:
            raise MemoryError("oracle_expm_baseline_batch")
    return X, dict(m=m, s=s, n1=n1, near=near.astype(bool), threads=used)


def oracle_lowrank_select_from_norm(v1: float, tol: float) -> Tuple[int, int]:
    """Order of the low-rank variant (Sec. 2.2) from ||A2 A1||_1 -> (m, flag); flag 2: tolerance not reached."""
    m, f = ctypes.c_int(0), ctypes.c_int(0)
    _load().oracle_lowrank_select_from_norm(float(v1), float(tol), ctypes.byref(m), ctypes.byref(f))
    return m.value, f.value


def oracle_lowrank_batch(A1, A2, tol: float, threads: int = 0):
    """e^(A1 A2) = I + A1 phi_m(A2 A1) A2 on a batch: A1 [b][n][t], A2 [b][t][n]
    -> (X fp64 [b][n][n], dict of arrays m, flag, v1, near, threads)."""
    a1 = np.ascontiguousarray(np.asarray(A1, dtype=np.float64))
    a2 = np.ascontiguousarray(np.asarray(A2, dtype=np.float64))
    if a1.ndim == 2:
        a1, a2 = a1[None], a2[None]
    assert a1.ndim == 3 and a2.ndim == 3 and a1.shape[0] == a2.shape[0]
    b, n, t = a1.shape
    assert a2.shape[1] == t and a2.shape[2] == n
    X = np.empty((b, n, n), dtype=np.float64)
    m = np.zeros(b, dtype=np.int32)
    flag = np.zeros(b, dtype=np.int32)
    near = np.zeros(b, dtype=np.int32)
    v1 = np.zeros(b, dtype=np.float64)
    used = 0
    if b > 0 and n > 0 and t > 0:
        used = _load().oracle_lowrank_batch(_dptr(a1), _dptr(a2), n, t, b, float(tol), _dptr(X), _iptr(m), _iptr(flag),
                                            _dptr(v1), _iptr(near), int(threads))
        if used < 0:
            raise MemoryError("oracle_lowrank_batch")
    return X, dict(m=m, flag=flag, v1=v1, near=near.astype(bool), threads=used)


def oracle_expm_forced(W, m: int, s: int, plus16=None, threads: int = 0) -> np.ndarray:
    """Algorithm 2 with the order and scaling given: sum_{k<=m} A^k/k! (+ b16 A^16 for the 15+ approximant), A = W/2^s,
    then s squarings.  plus16 defaults to (m == 15), the main scheme's meaning of order 15; pass False for the plain
    Taylor polynomial of the Paterson-Stockmeyer variant and of the baseline."""
    a = _as_f64(W)
    n = a.shape[0]
    assert a.shape == (n, n)
    X = np.empty((n, n), dtype=np.float64)
    p16 = (int(m) == 15) if plus16 is None else bool(plus16)
    rc = _load().oracle_expm_forced(_dptr(a), n, int(m), int(s), int(p16), _dptr(X), int(threads))
    if rc != 0:
        raise ValueError("oracle_expm_forced: status %d" % rc)
    return X


def oracle_lowrank_forced(A1, A2, m: int) -> np.ndarray:
    """I + A1 (sum_{i<=m} V^i/(i+1)!) A2, V = A2 A1, with the order m given."""
    a1 = np.ascontiguousarray(np.asarray(A1, dtype=np.float64))
    a2 = np.ascontiguousarray(np.asarray(A2, dtype=np.float64))
    n, t = a1.shape
    assert a2.shape == (t, n)
    X = np.empty((n, n), dtype=np.float64)
    rc = _load().oracle_lowrank_forced(_dptr(a1), _dptr(a2), n, t, int(m), _dptr(X))
    if rc != 0:
        raise ValueError("oracle_lowrank_forced: status %d" % rc)
    return X


def oracle_matmul_threads(A, B, threads: int = 0):
    """One triple-loop product with rows spread over the threads -> (C, threads used)."""
    a, b = _as_f64(A), _as_f64(B)
    n = a.shape[0]
    assert a.shape == (n, n) and b.shape == (n, n)
    c = np.empty((n, n), dtype=np.float64)
    used = _load().oracle_matmul_threads(_dptr(a), _dptr(b), _dptr(c), n, int(threads))
    return c, int(used)


def oracle_max_threads() -> int:
    return int(_load().oracle_max_threads())
