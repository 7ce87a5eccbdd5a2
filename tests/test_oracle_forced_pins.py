"""Pins of the oracle's branches that the full-size GPU parity cases lean on, no GPU:

* the row-parallel products that the batch drivers switch to from order 256 on (bit-equal to the
  single-matrix calls, whose products are sequential);
* the entry points that take (m, s) as given (Algorithm 2 after the selection): bit-equal to the selecting
  calls for the pair those select, and equal to the closed form of the polynomial on 1 x 1 input for any pair;
* the `near` flags of the Paterson-Stockmeyer selection (Algorithm 3) and of the baseline (Algorithm 1) at
  hand-placed switch points.
"""
import math
from fractions import Fraction

import numpy as np
import pytest

from oracle import (oracle_b16, oracle_expm, oracle_expm_baseline_batch, oracle_expm_batch, oracle_expm_forced,
                    oracle_expm_ps_batch, oracle_lowrank_batch, oracle_lowrank_forced, oracle_matmul,
                    oracle_matmul_threads, oracle_select_ps, oracle_select_ps_from_norms)
from paper_2512_20777_amd import workloads

U64 = 2.0 ** -53
U32 = 2.0 ** -24


# ---- products of order >= 256: rows spread over threads, same arithmetic per element -------------------------
@pytest.mark.parametrize("n", [256, 260, 300])
def test_batch_driver_row_parallel_branch_is_bit_equal_to_single_matrix_calls(n):
    a = workloads.random_stack(7000 + n, 2, n, np.float64, 0.4, 30.0)
    X, info = oracle_expm_batch(a, U64, threads=3)   # n >= 256: one matrix after another, rows of a product in parallel
    for b in range(a.shape[0]):
        Xs, i1 = oracle_expm(a[b], U64)              # sequential products
        assert (i1["m"], i1["s"]) == (info["m"][b], info["s"][b])
        assert i1["n1"] == info["n1"][b] and i1["n2"] == info["n2"][b]
        assert np.array_equal(X[b], Xs)


def test_ps_batch_driver_row_parallel_branch_is_bit_equal_to_the_sequential_evaluation():
    n = 257
    a = workloads.random_stack(7100, 2, n, np.float64, 0.4, 30.0)
    X, info = oracle_expm_ps_batch(a, U64, threads=3)
    for b in range(2):
        # the same polynomial with sequential products (order < 256 is never row-parallel: embed nothing, call the
        # forced entry on one thread, whose products at this size are row-parallel only in name: one thread)
        Xs = oracle_expm_forced(a[b], int(info["m"][b]), int(info["s"][b]), plus16=False, threads=1)
        assert np.array_equal(X[b], Xs)
    # and the threaded product itself against the sequential one
    c_par, used = oracle_matmul_threads(a[0], a[1], threads=3)
    assert used == 3 and np.array_equal(c_par, oracle_matmul(a[0], a[1]))


# ---- (m, s) given ------------------------------------------------------------------------------------------------
def test_forced_evaluation_is_bit_equal_to_the_selecting_call_for_the_selected_pair():
    seen = set()
    for seed, n, lo, hi, dt in ((1, 7, 1e-9, 1e-2, np.float64), (2, 12, 1e-3, 40.0, np.float64),
                                (3, 33, 0.05, 200.0, np.float64), (4, 20, 1e-3, 30.0, np.float32)):
        a = workloads.random_stack(7200 + seed, 24, n, dt, lo, hi)
        tol = U32 if dt == np.float32 else U64
        X, info = oracle_expm_batch(a, tol)
        Xp, ip = oracle_expm_ps_batch(a, tol)
        for b in range(a.shape[0]):
            m, s = int(info["m"][b]), int(info["s"][b])
            seen.add((m, s > 0))
            assert np.array_equal(oracle_expm_forced(a[b], m, s), X[b])
            assert np.array_equal(oracle_expm_forced(a[b], int(ip["m"][b]), int(ip["s"][b]), plus16=False), Xp[b])
    assert {m for m, _ in seen} >= {1, 2, 4, 8, 15} and (15, True) in seen


@pytest.mark.parametrize("m,s,plus16", [(0, 0, False), (1, 0, False), (2, 3, False), (4, 0, False), (8, 1, False),
                                        (15, 0, True), (15, 2, True), (15, 2, False), (6, 1, False), (16, 4, False),
                                        (23, 2, False)])
def test_forced_evaluation_closed_form_on_scalars(m, s, plus16):
    """1 x 1 input x: the result is (sum_{k<=m} (x/2^s)^k/k! [+ b16 (x/2^s)^16])^(2^s), evaluated exactly."""
    for x in (0.75, -1.5, 3.0):
        a = Fraction(x) / 2 ** s
        p = sum(a ** k / math.factorial(k) for k in range(m + 1))
        if plus16:
            p += Fraction(oracle_b16()) * a ** 16
        want = float(p ** (2 ** s))
        got = oracle_expm_forced(np.array([[x]]), m, s, plus16=plus16)[0, 0]
        assert abs(got - want) <= 64 * 2 ** s * 2.0 ** -53 * abs(want), (x, m, s, got, want)


def test_forced_evaluation_with_the_neighbouring_choice_is_still_the_exponential():
    """The pairs on both sides of a switch point approximate the same matrix: (15, s) and (15, s + 1), (8, 0) and
    (15, 0) agree to the tolerance the selection works to (times the growth through the squarings)."""
    a = workloads.random_stack(7300, 6, 10, np.float64, 0.5, 20.0)
    X, info = oracle_expm_batch(a, U64)
    for b in range(6):
        m, s = int(info["m"][b]), int(info["s"][b])
        Y = oracle_expm_forced(a[b], 15, s + 1)
        assert np.linalg.norm(Y - X[b]) <= 1e-12 * np.linalg.norm(X[b]), (b, m, s)
    with pytest.raises(ValueError):
        oracle_expm_forced(a[0], 8, 0, plus16=True)     # the b16 term belongs to order 15 only


def test_lowrank_forced_is_bit_equal_for_the_selected_order_and_a_series_otherwise():
    a1, a2 = workloads.lowrank_stack(7400, 10, 30, 5, np.float64, 1e-3, 0.9)
    X, info = oracle_lowrank_batch(a1, a2, U64)
    assert len(set(info["m"].tolist())) >= 3
    for b in range(10):
        assert np.array_equal(oracle_lowrank_forced(a1[b], a2[b], int(info["m"][b])), X[b])
    # rank one: V is the scalar v = a2.a1, so the order-m result is I + (sum_{i<=m} v^i/(i+1)!) a1 a2
    u, w = a1[0][:, :1].copy(), a2[0][:1, :].copy()
    v = float((w @ u)[0, 0])
    for m in (0, 1, 3, 6):
        phi = sum(v ** i / math.factorial(i + 1) for i in range(m + 1))
        got = oracle_lowrank_forced(u, w, m)
        assert np.allclose(got, np.eye(30) + phi * (u @ w), rtol=0, atol=1e-15 * (1 + abs(phi)) * np.abs(u @ w).max() + 1e-16)


# ---- near flag of Algorithm 3 --------------------------------------------------------------------------------------
def _ps_switch_point(lower_m, eps):
    """x at which the choice for W = x I (norms x, x^2, x^3, x^4) leaves order lower_m: bisection on the rule."""
    lo, hi = 1e-12, 50.0
    for _ in range(200):
        mid = math.sqrt(lo * hi)
        m, s = oracle_select_ps_from_norms(mid, mid ** 2, mid ** 3, mid ** 4, eps)
        if (m, s) <= (lower_m, 0):
            lo = mid
        else:
            hi = mid
    return lo


@pytest.mark.parametrize("lower_m", [1, 2, 4, 6, 9, 12, 16])
def test_ps_near_flag_at_hand_placed_switch_points(lower_m):
    eps = 1e-8
    xs = _ps_switch_point(lower_m, eps)
    eye = np.eye(3)
    # E1 + E2 of order m = j k grows like the product of k + 1 norms (k factors ||W^j||, one of ||W|| or ||W^2||): moving
    # every norm by 1e-6 moves the bound by about (k + 1) e-6.  A point whose bound is 2.5e-6 away (relative) is
    # therefore near only because the corners move the high power as well -- that pins every norm's part in the flag.
    k_plus_1 = {1: 2, 2: 2, 4: 3, 6: 3, 9: 4, 12: 4, 16: 5}[lower_m]
    if k_plus_1 >= 3:
        degree = lower_m + 1                       # the bound is (about) homogeneous of this degree in x
        x = xs * (1.0 - 2.5e-6 / degree)           # bound 2.5e-6 below eps: one norm alone (1e-6) cannot cross
        r = oracle_select_ps(x * eye, eps)
        assert r["m"] == lower_m and r["near"], (lower_m, r)
    for f in (1.0 - 2e-7, 1.0 + 2e-7):
        assert oracle_select_ps(xs * f * eye, eps)["near"]
    for f in (1.0 - 1e-3, 1.0 + 1e-3):
        r = oracle_select_ps(xs * f * eye, eps)
        assert not r["near"], (lower_m, f, r)
    assert oracle_select_ps(xs * (1 - 1e-3) * eye, eps)["m"] == lower_m


def test_ps_near_flag_between_two_scalings():
    """Beyond order 16 the choice is (16, s): the switch from s to s + 1 is flagged too."""
    eps = U64
    lo, hi = 1.0, 400.0
    for _ in range(200):   # x where s goes from 2 to 3
        mid = 0.5 * (lo + hi)
        if oracle_select_ps_from_norms(mid, mid ** 2, mid ** 3, mid ** 4, eps)[1] <= 2:
            lo = mid
        else:
            hi = mid
    eye = np.eye(2)
    assert oracle_select_ps(lo * (1 - 1e-7) * eye, eps)["near"] and oracle_select_ps(lo * (1 + 1e-7) * eye, eps)["near"]
    a, b = oracle_select_ps(lo * 0.99 * eye, eps), oracle_select_ps(lo * 1.01 * eye, eps)
    assert not a["near"] and not b["near"] and (a["s"], b["s"]) == (2, 3)


# ---- near flag of the baseline (Algorithm 1) -----------------------------------------------------------------------
def test_baseline_near_flag_at_hand_placed_switch_points():
    eps = 1e-8
    eye = np.eye(4)

    def run(x, tol=eps):
        _, info = oracle_expm_baseline_batch((x * eye)[None], tol)
        return int(info["m"][0]), int(info["s"][0]), bool(info["near"][0])

    # scaling rule ||W|| / 2^s < 1/2: norm 4 (1 -+ 3e-7) sits on the switch from s = 3 to s = 4
    m_lo, s_lo, near_lo = run(4.0 * (1 - 3e-7))
    m_hi, s_hi, near_hi = run(4.0 * (1 + 3e-7))
    assert (s_lo, s_hi) == (3, 4) and near_lo and near_hi
    # the terms of a = 0.3: ||Y_k|| = a^k / k!; none of them within 1e-6 of eps, norm far from a power of two / 2
    a = 0.3
    terms = [a ** k / math.factorial(k) for k in range(1, 40)]
    assert all(abs(t / eps - 1.0) > 1e-3 for t in terms)
    m, s, near = run(a)
    assert s == 0 and not near and m == sum(1 for t in terms if t > eps)
    # stopping rule ||Y|| > eps: put eps within 3e-7 of the sixth term, on either side
    t6 = terms[5]
    m_a, _, near_a = run(a, t6 * (1 + 3e-7))    # term 6 no longer exceeds eps: 5 terms
    m_b, _, near_b = run(a, t6 * (1 - 3e-7))    # term 6 still exceeds it: 6 terms
    assert (m_a, m_b) == (5, 6) and near_a and near_b
    assert not run(a, t6 * 1.01)[2] and not run(a, t6 * 0.99)[2]
