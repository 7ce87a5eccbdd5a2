"""Low-rank variant of Sec. 2.2, e^(A1 A2) = I + A1 phi_m(A2 A1) A2 without scaling: pins of the oracle (CPU) and
GPU parity through the C ABI.

Pins (none of them re-types the oracle's summation):
* the identity behind the variant: the result agrees with the full-size oracle applied to W = A1 A2;
* rank one: V = v^T u is a scalar c and e^W = I + u v^T (e^c - 1)/c in closed form;
* A2 A1 = 0: W is nilpotent of index 2, the result I + A1 A2 is exact and the order is 0;
* the order chosen really delivers the tolerance (true remainder of the scalar series, exact rationals) and
  is the smallest of the order set whose printed bound does (bound evaluated in exact rationals);
* beyond the reach of the largest order the call is flagged, not silently wrong.
"""
from fractions import Fraction
from math import factorial

import numpy as np
import pytest

U64 = 2.0 ** -53
U32 = 2.0 ** -24
ORDERS = [1, 2, 4, 6, 9, 12, 16]


def _pair(rng, n, t, target_norm):
    a1 = rng.standard_normal((n, t))
    a2 = rng.standard_normal((t, n))
    v = a2 @ a1
    f = np.sqrt(target_norm / np.abs(v).sum(axis=0).max())
    return a1 * f, a2 * f


def test_oracle_lowrank_equals_the_full_size_exponential():
    from oracle import oracle_expm_batch, oracle_lowrank_batch
    rng = np.random.default_rng(5)
    for n, t, nv, eps, gate in ((12, 3, 0.4, U64, 5e-14), (20, 5, 2.5, 1e-8, 1e-7), (9, 9, 1e-3, U64, 5e-14),
                                (16, 2, 0.9, U64, 5e-14)):
        a1, a2 = _pair(rng, n, t, nv)
        X, info = oracle_lowrank_batch(a1, a2, eps)
        W = a1 @ a2
        Y, _ = oracle_expm_batch(W[None], U64)
        err = np.linalg.norm(X[0] - Y[0]) / np.linalg.norm(Y[0])
        assert info["flag"][0] == 0 and err < gate, (n, t, nv, info["m"][0], err)


def test_oracle_lowrank_rank_one_closed_form():
    from oracle import oracle_lowrank_batch
    rng = np.random.default_rng(6)
    for c in (-0.9, -0.2, 1e-6, 0.7, 1.0):
        n = 7
        u = rng.standard_normal((n, 1))
        v = rng.standard_normal((1, n))
        v *= c / (v @ u).item()
        X, info = oracle_lowrank_batch(u, v, U64)
        exact = np.eye(n) + (u @ v) * (np.expm1(c) / c)
        assert np.linalg.norm(X[0] - exact) / np.linalg.norm(exact) < 1e-14, (c, info["m"][0])


def test_oracle_lowrank_nilpotent_pair_is_exact_with_order_zero():
    from oracle import oracle_lowrank_batch
    n, t = 8, 3
    a1 = np.zeros((n, t)); a2 = np.zeros((t, n))
    a1[:4, :] = np.arange(12).reshape(4, 3) + 1.0      # columns live in rows 0..3
    a2[:, 4:] = np.arange(12).reshape(3, 4) - 5.0      # rows live in columns 4..7  ->  A2 A1 = 0
    X, info = oracle_lowrank_batch(a1, a2, U64)
    assert info["m"][0] == 0 and info["v1"][0] == 0.0
    assert np.array_equal(X[0], np.eye(n) + a1 @ a2)


def _bound(v: Fraction, m: int):
    if v >= m + 3:
        return None
    return v ** (m + 1) / factorial(m + 2) / (1 - v / (m + 3))


@pytest.mark.parametrize("eps", [U64, U32, 1e-8])
def test_oracle_lowrank_order_is_the_smallest_that_meets_the_printed_bound(eps):
    from oracle import oracle_lowrank_select_from_norm
    rng = np.random.default_rng(7)
    seen = set()
    for _ in range(400):
        v1 = float(10.0 ** rng.uniform(-9, 0.9))
        m, flag = oracle_lowrank_select_from_norm(v1, eps)
        v, e = Fraction(v1), Fraction(eps)
        ok = [q for q in ORDERS if _bound(v, q) is not None and _bound(v, q) <= e]
        if ok:
            # skip decisions within 1e-6 relative of a switch point (rounding of the fp64 evaluation)
            lo, hi = Fraction(v1 * (1 - 1e-6)), Fraction(v1 * (1 + 1e-6))
            oklo = [q for q in ORDERS if _bound(lo, q) is not None and _bound(lo, q) <= e]
            okhi = [q for q in ORDERS if _bound(hi, q) is not None and _bound(hi, q) <= e]
            if oklo[:1] == okhi[:1] == ok[:1]:
                assert (m, flag) == (ok[0], 0), (v1, eps, m, ok)
            # the true remainder of the scalar series is within the tolerance
            rem = sum(v ** i / factorial(i + 1) for i in range(m + 1, m + 60))
            assert rem <= e
        else:
            assert (m, flag) == (16, 2), (v1, eps, m, flag)
        seen.add(m)
    assert seen >= set(ORDERS)
    assert oracle_lowrank_select_from_norm(0.0, eps) == (0, 0)
    assert oracle_lowrank_select_from_norm(float("nan"), eps) == (-1, 1)
    assert oracle_lowrank_select_from_norm(50.0, eps) == (16, 2)
