"""Seeded synthetic inputs for the batched matrix exponential.

This module only makes input matrices.  It holds none of the method's
arithmetic (no selection, no polynomial, no squaring) and is the one module
that both the GPU tests/benchmark and the CPU oracle's tests may import.

The five workloads stand in for the matrices of the paper's experiments
(test-bed matrices of order 4..1024, Sec. 4.1; flow-layer weights with norms
between about 1e-5 and 12.8 and batches of 16x16 blocks, Sec. 4.2 and 5.1),
none of which are available here.  "N(0, v)" is a normal of variance v.
Values are drawn in fp64 with numpy's PCG64 from a fixed seed per workload,
scaled in fp64, and rounded to fp32 last for the fp32 workloads.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, Tuple

import numpy as np

SEED_BASE = 2512207770


@dataclass(frozen=True)
class Workload:
    name: str
    n: int
    batch: int
    dtype: str  # "f32" | "f64"
    seed: int
    note: str
    tolerance: float = 0.0   # 0: unit roundoff of the dtype
    norm: str = "one"        # norm the selection uses: "one" | "inf"

    @property
    def np_dtype(self):
        return np.float32 if self.dtype == "f32" else np.float64

    @property
    def tol(self) -> float:
        """Tolerance of the workload: the unit roundoff of its dtype unless it states one."""
        if self.tolerance > 0.0:
            return self.tolerance
        return 2.0 ** -24 if self.dtype == "f32" else 2.0 ** -53


WORKLOADS: Dict[str, Workload] = {
    "C1": Workload("C1", 32, 16, "f64", SEED_BASE + 1,
                   "16 x 32x32 fp64, iid N(0,1/32), 1-norm log-uniform in [0.05,5]"),
    "C2": Workload("C2", 16, 4096, "f32", SEED_BASE + 2,
                   "4096 x 16x16 fp32 flow-layer generators: skew part N(0,1) + diagonal N(0,0.1), "
                   "1-norm log-uniform in [0.01,10]"),
    "C3": Workload("C3", 128, 256, "f32", SEED_BASE + 3,
                   "256 x 128x128 fp32, iid N(0,1/128) times a log-uniform factor in [0.1,50]"),
    "C4": Workload("C4", 512, 32, "f64", SEED_BASE + 4,
                   "32 x 512x512 fp64, 16 dense iid N(0,1/512) + 16 upper-triangular non-normal, "
                   "1-norm log-uniform in [0.5,100]"),
    "C5f64": Workload("C5f64", 4096, 4, "f64", SEED_BASE + 5,
                      "4 x 4096x4096 fp64, iid N(0,1/4096), 1-norms 1, 10, 50, 200"),
    "C5f32": Workload("C5f32", 4096, 4, "f32", SEED_BASE + 5,
                      "4 x 4096x4096 fp32 (the fp64 draw rounded), 1-norms 1, 10, 50, 200"),
    # The setting of the paper's own flow-model runs (Sec. 4.2): tolerance 1e-8, infinity-norm selection,
    # norms between 1e-5 and 12.8, so that the low orders are exercised heavily.
    "F1": Workload("F1", 16, 4096, "f64", SEED_BASE + 6,
                   "4096 x 16x16 fp64 flow-layer generators, inf-norm log-uniform in [1e-5,12.8], tol 1e-8, "
                   "inf-norm selection", tolerance=1e-8, norm="inf"),
}


def _norm1(a: np.ndarray) -> np.ndarray:
    """Max column abs-sum of each matrix of a [b][n][n] stack (used only to rescale inputs)."""
    return np.abs(a).sum(axis=-2).max(axis=-1)


def _rescale_to(a: np.ndarray, target: np.ndarray) -> np.ndarray:
    cur = _norm1(a)
    return a * (target / cur)[:, None, None]


def _log_uniform(rng: np.random.Generator, lo: float, hi: float, size: int) -> np.ndarray:
    t = rng.random(size)
    return lo * (hi / lo) ** t


def make_workload(name: str, batch: int | None = None, n: int | None = None) -> np.ndarray:
    """Return the input stack [batch][n][n] of workload `name` in its dtype.

    `batch` / `n` override the size (same recipe, same seed) for reduced parity cases.
    """
    w = WORKLOADS[name]
    b = w.batch if batch is None else batch
    n = w.n if n is None else n
    rng = np.random.default_rng(w.seed)
    if name == "C1":
        a = rng.standard_normal((b, n, n)) * np.sqrt(1.0 / n)
        a = _rescale_to(a, _log_uniform(rng, 0.05, 5.0, b))
    elif name == "C2":
        g = rng.standard_normal((b, n, n))
        up = np.triu(g, 1)
        a = up - np.swapaxes(up, -1, -2)
        d = rng.standard_normal((b, n)) * np.sqrt(0.1)
        idx = np.arange(n)
        a[:, idx, idx] = d
        a = _rescale_to(a, _log_uniform(rng, 0.01, 10.0, b))
    elif name == "F1":
        g = rng.standard_normal((b, n, n))
        up = np.triu(g, 1)
        a = up - np.swapaxes(up, -1, -2)
        idx = np.arange(n)
        a[:, idx, idx] = rng.standard_normal((b, n)) * np.sqrt(0.1)
        target = _log_uniform(rng, 1e-5, 12.8, b)
        a = a * (target / np.abs(a).sum(axis=-1).max(axis=-1))[:, None, None]   # rescale the infinity-norm
    elif name == "C3":
        a = rng.standard_normal((b, n, n)) * np.sqrt(1.0 / n)
        a = a * _log_uniform(rng, 0.1, 50.0, b)[:, None, None]
    elif name == "C4":
        half = b // 2
        a = np.empty((b, n, n), dtype=np.float64)
        a[:half] = rng.standard_normal((half, n, n)) * np.sqrt(1.0 / n)
        t = np.triu(rng.standard_normal((b - half, n, n)), 1)
        idx = np.arange(n)
        t[:, idx, idx] = rng.uniform(-1.0, 1.0, (b - half, n))
        a[half:] = t
        a = _rescale_to(a, _log_uniform(rng, 0.5, 100.0, b))
    elif name in ("C5f64", "C5f32"):
        a = np.empty((b, n, n), dtype=np.float64)
        for i in range(b):  # one matrix at a time keeps the peak host memory low
            a[i] = rng.standard_normal((n, n)) * np.sqrt(1.0 / n)
        targets = np.array([1.0, 10.0, 50.0, 200.0])[np.arange(b) % 4]
        a = _rescale_to(a, targets)
    else:
        raise KeyError(name)
    return np.ascontiguousarray(a.astype(w.np_dtype))


def random_stack(seed: int, batch: int, n: int, dtype, norm_lo: float, norm_hi: float,
                 kind: str = "dense") -> np.ndarray:
    """Generic seeded stack for parity cases of arbitrary size.

    kind: "dense" iid N(0,1/n); "triu" non-normal upper triangular; "skew" skew-symmetric + diagonal.
    Each matrix is rescaled to a 1-norm log-uniform in [norm_lo, norm_hi].
    """
    rng = np.random.default_rng(seed)
    if batch == 0 or n == 0:
        return np.zeros((batch, n, n), dtype=dtype)
    if kind == "dense":
        a = rng.standard_normal((batch, n, n)) * np.sqrt(1.0 / n)
    elif kind == "triu":
        a = np.triu(rng.standard_normal((batch, n, n)), 1)
        idx = np.arange(n)
        a[:, idx, idx] = rng.uniform(-1.0, 1.0, (batch, n))
    elif kind == "skew":
        up = np.triu(rng.standard_normal((batch, n, n)), 1)
        a = up - np.swapaxes(up, -1, -2)
        idx = np.arange(n)
        a[:, idx, idx] = rng.standard_normal((batch, n)) * np.sqrt(0.1)
    else:
        raise KeyError(kind)
    a = _rescale_to(a, _log_uniform(rng, norm_lo, norm_hi, batch))
    return np.ascontiguousarray(a.astype(dtype))


# Low-rank workload (Sec. 2.2): W = A1 A2 with A1 n x t, A2 t x n.  L1 stands for a flow layer on high-dimensional
# data, the case that variant was proposed for: 64 pairs, n = 1024, t = 64, fp32, factors iid N(0,1) rescaled so that
# ||A2 A1||_1 is log-uniform in [1e-3, 2] (within reach of the unscaled series at fp32 roundoff).
LOWRANK_WORKLOADS = {
    "L1": dict(n=1024, t=64, batch=64, dtype="f32", seed=SEED_BASE + 7, lo=1e-3, hi=2.0,
               note="64 pairs A1 (1024x64), A2 (64x1024) fp32, iid N(0,1) rescaled, ||A2 A1||_1 log-uniform in [1e-3,2]"),
}


def lowrank_stack(seed: int, batch: int, n: int, t: int, dtype, norm_lo: float, norm_hi: float):
    """Seeded pairs (A1 [batch][n][t], A2 [batch][t][n]) whose ||A2 A1||_1 is log-uniform in [norm_lo, norm_hi];
    both factors of a pair get the same scale."""
    rng = np.random.default_rng(seed)
    a1 = rng.standard_normal((batch, n, t))
    a2 = rng.standard_normal((batch, t, n))
    if batch and n and t:
        v1 = np.abs(np.matmul(a2, a1)).sum(axis=1).max(axis=1)
        f = np.sqrt(_log_uniform(rng, norm_lo, norm_hi, batch) / v1)
        a1 *= f[:, None, None]
        a2 *= f[:, None, None]
    return np.ascontiguousarray(a1.astype(dtype)), np.ascontiguousarray(a2.astype(dtype))


def make_lowrank_workload(name: str):
    w = LOWRANK_WORKLOADS[name]
    dt = np.float32 if w["dtype"] == "f32" else np.float64
    return lowrank_stack(w["seed"], w["batch"], w["n"], w["t"], dt, w["lo"], w["hi"])


def products_for(m: np.ndarray, s: np.ndarray, scheme: str = "sastre") -> np.ndarray:
    """Matrix products the method spends on a matrix with order m and scaling s.

    Cost of the evaluation formulas (Sec. 3.1): 0 for m in {0,1}, 1 for m=2, 2 for m=4,
    3 for m=8, 4 for 15+; each squaring adds one.  Pure bookkeeping for FLOP accounting.
    """
    table = {0: 0, 1: 0, 2: 1, 4: 2, 8: 3, 15: 4}
    if scheme == "ps":  # Paterson-Stockmeyer (Table 1 of the paper): order 6 at 3, 9 at 4, 12 at 5, 16 at 6 products
        table = {0: 0, 1: 0, 2: 1, 4: 2, 6: 3, 9: 4, 12: 5, 16: 6}
    return np.array([table[int(x)] for x in np.asarray(m)], dtype=np.int64) + np.asarray(s, dtype=np.int64)
