"""Thin ctypes binding of the C ABI in include/expm_mi355x.h.

Argument marshalling only: every step of the method runs in the library's HIP kernels.  torch is
used for device memory and the current stream.  There is no CPU fallback: if the shared library
has not been built, or no GPU is present, calls raise.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libexpm_mi355x.so")
_lib = None

DTYPE_F32 = 0
DTYPE_F64 = 1
SCHEME_SASTRE = 0   # Algorithm 4 + evaluation formulas of Sec. 3.1 (orders 1,2,4,8,15+)
SCHEME_PS = 1       # Algorithm 3 + Paterson-Stockmeyer (orders 1,2,4,6,9,12,16)
SCHEME_BASELINE = 2  # the paper's comparison baseline (its Algorithm 1); small matrices only
NORM_ONE = 0        # selection on 1-norms (the printed algorithms)
NORM_INF = 1        # selection on infinity-norms (the paper's PyTorch runs, Sec. 4.2)

EXPM_KCLASS = {"norm": 0, "select": 1, "gemm": 2, "fused": 3}


class ExpmError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__("expm status %d: %s" % (status, text))
        self.status = status


class _Stats(ctypes.Structure):
    _fields_ = [
        ("matrices", ctypes.c_int64), ("products", ctypes.c_int64), ("n", ctypes.c_int32), ("dtype", ctypes.c_int32),
        ("rounds", ctypes.c_int32), ("warning", ctypes.c_int32), ("fused_path", ctypes.c_int32),
        ("scheme", ctypes.c_int32), ("hist_m", ctypes.c_int64 * 17), ("hist_s", ctypes.c_int64 * 21),
        ("nonfinite", ctypes.c_int64), ("warning_bits", ctypes.c_int32), ("reserved", ctypes.c_int32),
    ]


class _Profile(ctypes.Structure):
    _fields_ = [
        ("launches", ctypes.c_int64 * 4), ("ms", ctypes.c_double * 4), ("flops", ctypes.c_double * 4),
        ("bytes", ctypes.c_double * 4),
    ]


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load the shared library (built in-tree by paper_2512_20777_amd.build); raise if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    # torch ships its own HIP runtime; it must be in the process first so that this library binds to
    # the same runtime instance (two runtimes in one process do not share device allocations)
    import torch  # noqa: F401
    if not os.path.exists(_LIB_PATH):
        raise ExpmError(-100, "shared library %s not built (run `python -m paper_2512_20777_amd.build`); "
                              "there is no CPU fallback" % _LIB_PATH)
    lib = ctypes.CDLL(_LIB_PATH)
    vp, ci, cd = ctypes.c_void_p, ctypes.c_int, ctypes.c_double
    i32p = ctypes.POINTER(ctypes.c_int32)
    lib.expm_select.restype = ci
    lib.expm_select.argtypes = [vp, ci, ci, ci, cd, i32p, i32p]
    lib.expm.restype = ci
    lib.expm.argtypes = [vp, ci, ci, ci, cd, vp, vp]
    lib.expm_noalloc.restype = ci
    lib.expm_noalloc.argtypes = [vp, ci, ci, ci, cd, vp, vp]
    lib.expm_select_scheme.restype = ci
    lib.expm_select_scheme.argtypes = [vp, ci, ci, ci, cd, ci, i32p, i32p]
    lib.expm_scheme.restype = ci
    lib.expm_scheme.argtypes = [vp, ci, ci, ci, cd, ci, vp, vp]
    lib.expm_select_ex.restype = ci
    lib.expm_select_ex.argtypes = [vp, ci, ci, ci, cd, ci, ci, i32p, i32p]
    lib.expm_ex.restype = ci
    lib.expm_ex.argtypes = [vp, ci, ci, ci, cd, ci, ci, vp, vp]
    lib.expm_lowrank_select.restype = ci
    lib.expm_lowrank_select.argtypes = [vp, vp, ci, ci, ci, ci, cd, i32p]
    lib.expm_lowrank.restype = ci
    lib.expm_lowrank.argtypes = [vp, vp, ci, ci, ci, ci, cd, vp, vp]
    lib.expm_workspace_bytes.restype = ctypes.c_size_t
    lib.expm_workspace_bytes.argtypes = [ci, ci, ci]
    lib.expm_reserve.restype = ci
    lib.expm_reserve.argtypes = [ci, ci, ci]
    lib.expm_get_stats.restype = ci
    lib.expm_get_stats.argtypes = [ctypes.POINTER(_Stats)]
    lib.expm_profile_enable.restype = ci
    lib.expm_profile_enable.argtypes = [ci]
    lib.expm_profile_reset.restype = ci
    lib.expm_profile_reset.argtypes = []
    lib.expm_profile_read.restype = ci
    lib.expm_profile_read.argtypes = [ctypes.POINTER(_Profile)]
    lib.expm_shutdown.restype = ci
    lib.expm_shutdown.argtypes = []
    lib.expm_last_hip_error.restype = ci
    lib.expm_last_hip_error.argtypes = []
    lib.expm_status_string.restype = ctypes.c_char_p
    lib.expm_status_string.argtypes = [ci]
    _lib = lib
    return lib


def expm_status_string(status: int) -> str:
    return load_library().expm_status_string(int(status)).decode()


def _check(status: int) -> int:
    if status < 0:
        lib = load_library()
        text = expm_status_string(status)
        if status in (-3, -4):
            text += " [hipError %d]" % lib.expm_last_hip_error()
        raise ExpmError(status, text)
    return status


def _describe(A) -> Tuple[int, int, int]:
    import torch
    if not isinstance(A, torch.Tensor) or not A.is_cuda:
        raise ExpmError(-1, "input must be a torch tensor in device memory")
    if A.dim() != 3 or A.shape[1] != A.shape[2]:
        raise ExpmError(-1, "input must have shape [batch][n][n]")
    if not A.is_contiguous():
        raise ExpmError(-1, "input must be contiguous (row-major [batch][n][n])")
    if A.dtype is torch.float32:
        dt = DTYPE_F32
    elif A.dtype is torch.float64:
        dt = DTYPE_F64
    else:
        raise ExpmError(-1, "dtype must be float32 or float64")
    return A.shape[1], A.shape[0], dt


def expm_select(A, tol: float = 0.0, scheme: int = SCHEME_SASTRE, norm: int = NORM_ONE):
    """(m, s) per matrix as two int32 numpy arrays, plus the status (0 or a warning code)."""
    import numpy as np
    import torch
    n, batch, dt = _describe(A)
    m = np.zeros(batch, dtype=np.int32)
    s = np.zeros(batch, dtype=np.int32)
    i32p = ctypes.POINTER(ctypes.c_int32)
    with torch.cuda.device(A.device):
        torch.cuda.current_stream().synchronize()  # the C entry point runs on the null stream
        st = load_library().expm_select_ex(A.data_ptr(), n, batch, dt, float(tol), int(scheme), int(norm),
                                           m.ctypes.data_as(i32p), s.ctypes.data_as(i32p))
    return m, s, _check(st)


def expm(A, tol: float = 0.0, out=None, stream=None, scheme: int = SCHEME_SASTRE, norm: int = NORM_ONE):
    """e^A for a [batch][n][n] device tensor; returns (out, status).  Runs on torch's current stream.

    Marshalling only, kept short: for small batches the call rate is bounded by this function.
    """
    import torch
    lib = _lib if _lib is not None else load_library()
    n, batch, dt = _describe(A)
    if out is None:
        out = torch.empty_like(A)
    elif out.shape != A.shape or out.dtype is not A.dtype or out.device != A.device or not out.is_contiguous():
        raise ExpmError(-1, "out must match the input's shape, dtype and device and be contiguous")
    dev = A.device.index
    if stream is not None:
        sp = stream.cuda_stream
    else:
        sp = torch.cuda.current_stream(dev).cuda_stream
    if dev == torch.cuda.current_device():
        st = lib.expm_ex(A.data_ptr(), n, batch, dt, tol, scheme, norm, out.data_ptr(), sp)
    else:
        with torch.cuda.device(dev):
            st = lib.expm_ex(A.data_ptr(), n, batch, dt, tol, scheme, norm, out.data_ptr(), sp)
    if st < 0:
        _check(st)
    return out, st


def expm_noalloc(A, tol: float = 0.0, out=None, stream=None):
    """expm() through the entry point that allocates nothing (static device scratch); `out` must be given by callers
    that may not allocate.  Returns (out, status)."""
    import torch
    lib = _lib if _lib is not None else load_library()
    n, batch, dt = _describe(A)
    if out is None:
        out = torch.empty_like(A)
    elif out.shape != A.shape or out.dtype is not A.dtype or out.device != A.device or not out.is_contiguous():
        raise ExpmError(-1, "out must match the input's shape, dtype and device and be contiguous")
    dev = A.device.index
    sp = stream.cuda_stream if stream is not None else torch.cuda.current_stream(dev).cuda_stream
    with torch.cuda.device(dev):
        st = lib.expm_noalloc(A.data_ptr(), n, batch, dt, tol, out.data_ptr(), sp)
    if st < 0:
        _check(st)
    return out, st


def _describe_pair(A1, A2):
    import torch
    for x in (A1, A2):
        if not isinstance(x, torch.Tensor) or not x.is_cuda:
            raise ExpmError(-1, "inputs must be torch tensors in device memory")
        if x.dim() != 3 or not x.is_contiguous():
            raise ExpmError(-1, "inputs must be contiguous [batch][n][t] and [batch][t][n]")
    b, n, t = A1.shape
    if tuple(A2.shape) != (b, t, n) or A2.dtype is not A1.dtype or A2.device != A1.device:
        raise ExpmError(-1, "A2 must be [batch][t][n] of the dtype and on the device of A1")
    if A1.dtype is torch.float32:
        dt = DTYPE_F32
    elif A1.dtype is torch.float64:
        dt = DTYPE_F64
    else:
        raise ExpmError(-1, "dtype must be float32 or float64")
    return n, t, b, dt


def expm_lowrank_select(A1, A2, tol: float = 0.0):
    """Order m of the low-rank variant per pair (int32 numpy array) and the status."""
    import numpy as np
    import torch
    n, t, batch, dt = _describe_pair(A1, A2)
    m = np.zeros(batch, dtype=np.int32)
    with torch.cuda.device(A1.device):
        torch.cuda.current_stream().synchronize()  # the C entry point runs on the null stream
        st = load_library().expm_lowrank_select(A1.data_ptr(), A2.data_ptr(), n, t, batch, dt, float(tol),
                                                m.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)))
    return m, _check(st)


def expm_lowrank(A1, A2, tol: float = 0.0, out=None, stream=None):
    """e^(A1 A2) = I + A1 phi(A2 A1) A2 for [batch][n][t] and [batch][t][n] device tensors; returns (out, status)."""
    import torch
    lib = _lib if _lib is not None else load_library()
    n, t, batch, dt = _describe_pair(A1, A2)
    if out is None:
        out = torch.empty((batch, n, n), dtype=A1.dtype, device=A1.device)
    elif tuple(out.shape) != (batch, n, n) or out.dtype is not A1.dtype or out.device != A1.device or not out.is_contiguous():
        raise ExpmError(-1, "out must be a contiguous [batch][n][n] tensor of the inputs' dtype and device")
    dev = A1.device.index
    sp = stream.cuda_stream if stream is not None else torch.cuda.current_stream(dev).cuda_stream
    with torch.cuda.device(dev):
        st = lib.expm_lowrank(A1.data_ptr(), A2.data_ptr(), n, t, batch, dt, tol, out.data_ptr(), sp)
    if st < 0:
        _check(st)
    return out, st


def expm_workspace_bytes(n: int, batch: int, dtype: int) -> int:
    return int(load_library().expm_workspace_bytes(int(n), int(batch), int(dtype)))


def expm_reserve(n: int, batch: int, dtype: int) -> int:
    return _check(load_library().expm_reserve(int(n), int(batch), int(dtype)))


def expm_get_stats() -> dict:
    st = _Stats()
    _check(load_library().expm_get_stats(ctypes.byref(st)))
    return dict(matrices=st.matrices, products=st.products, n=st.n, dtype=st.dtype, rounds=st.rounds,
                warning=st.warning, warning_bits=st.warning_bits, fused_path=st.fused_path, scheme=st.scheme,
                nonfinite=st.nonfinite,
                hist_m={m: int(c) for m, c in enumerate(st.hist_m)}, hist_s=list(st.hist_s))


def expm_profile_enable(on: bool) -> None:
    _check(load_library().expm_profile_enable(1 if on else 0))


def expm_profile_reset() -> None:
    _check(load_library().expm_profile_reset())


def expm_profile_read() -> dict:
    p = _Profile()
    _check(load_library().expm_profile_read(ctypes.byref(p)))
    return {name: dict(launches=p.launches[i], ms=p.ms[i], flops=p.flops[i], bytes=p.bytes[i])
            for name, i in EXPM_KCLASS.items()}


def expm_shutdown() -> None:
    if _lib is not None:
        _lib.expm_shutdown()
