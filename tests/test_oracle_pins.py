"""Pins of the CPU oracle to things other than itself (no GPU needed).

Each test ties a part of oracle/expm_oracle.c to a value the paper prints, a closed form,
an invariant, or a brute-force computation written independently here, chosen so that a
plausible slip in the oracle (dropped term, wrong index, transposed operand, wrong norm)
fails at least one of them.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

from conftest import read_coefficients
from oracle import (oracle_b16, oracle_expm, oracle_expm_batch, oracle_matmul, oracle_norm1,
                    oracle_select, oracle_select_from_norms)

U64 = 2.0 ** -53
U32 = 2.0 ** -24


# ----------------------------------------------------------------------------------------
# products and norms: hand-computed small cases
# ----------------------------------------------------------------------------------------
def test_matmul_hand_2x2_and_3x3():
    A = np.array([[1.0, 2.0], [3.0, 4.0]])
    B = np.array([[0.0, 1.0], [5.0, -2.0]])
    # by hand: row1 = [1*0+2*5, 1*1+2*(-2)], row2 = [3*0+4*5, 3*1+4*(-2)]
    assert np.array_equal(oracle_matmul(A, B), np.array([[10.0, -3.0], [20.0, -5.0]]))
    # the reversed product differs (catches swapped operands / a transposed index)
    assert np.array_equal(oracle_matmul(B, A), np.array([[3.0, 4.0], [-1.0, 2.0]]))
    C = np.array([[1.0, 0.0, 2.0], [0.0, 3.0, 0.0], [4.0, 0.0, 5.0]])
    D = np.array([[0.0, 1.0, 0.0], [2.0, 0.0, 0.0], [0.0, 0.0, 7.0]])
    assert np.array_equal(oracle_matmul(C, D), np.array([[0.0, 1.0, 14.0], [6.0, 0.0, 0.0], [0.0, 4.0, 35.0]]))


def test_norm1_is_max_column_sum_not_row_sum():
    W = np.array([[1.0, -2.0, 3.0], [0.0, 0.5, -4.0], [0.0, 0.0, 0.25]])
    # column abs sums 1, 2.5, 7.25 ; row abs sums 6, 4.5, 0.25
    assert oracle_norm1(W) == 7.25
    assert oracle_norm1(W.T) == 6.0


def test_squaring_a_rotation_doubles_the_angle():
    th = 0.3
    R = np.array([[math.cos(th), -math.sin(th)], [math.sin(th), math.cos(th)]])
    R2 = oracle_matmul(R, R)
    E = np.array([[math.cos(2 * th), -math.sin(2 * th)], [math.sin(2 * th), math.cos(2 * th)]])
    assert np.allclose(R2, E, rtol=0, atol=4e-16)


# ----------------------------------------------------------------------------------------
# selection: values the paper states
# ----------------------------------------------------------------------------------------
def _examples(golden_dir):
    rows = []
    with open(os.path.join(golden_dir, "paper_selection_examples.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            name, _mat, eps, m, s, prod, _where = [x.strip() for x in line.split("|")]
            rows.append((name, float(eps), int(m), int(s), int(prod)))
    return {r[0]: r[1:] for r in rows}


def test_selection_examples_printed_in_the_paper(golden_dir):
    ex = _examples(golden_dir)
    eps, m, s, prod = ex["remark1"]
    got = oracle_select(np.array([[1.0, 10.0], [0.0, -1.0]]), eps)
    assert (got["m"], got["s"]) == (m, s)
    assert got["n1"] == 11.0 and got["n2"] == 1.0  # W^2 = I
    eps, m, s, prod = ex["normal12.8"]
    got = oracle_select(12.8 * np.eye(5), eps)
    assert (got["m"], got["s"]) == (m, s)
    assert 4 + got["s"] == prod  # 4 products for 15+, one per squaring
    eps, m, s, prod = ex["zero"]
    got = oracle_select(np.zeros((4, 4)), eps)
    assert (got["m"], got["s"]) == (m, s)


def test_b16_matches_the_printed_value_and_deviation(golden_dir):
    co = read_coefficients(os.path.join(golden_dir, "paper_coefficients.txt"))
    assert oracle_b16() == pytest.approx(co["b16"]["b16"], rel=2e-15)
    assert oracle_b16() == pytest.approx(co["T15+"]["c1"] ** 4, rel=1e-15)
    dev = abs(oracle_b16() - 1.0 / math.factorial(16)) * math.factorial(16)
    assert round(dev, 3) == co["b16"]["reldev"]


# ----------------------------------------------------------------------------------------
# selection: for W = x*I every ||W^k|| equals x^k, so Algorithm 4 must return the smallest
# order of {1,2,4,8,15+} whose first two remainder terms sum to <= eps (the criterion the
# paper states right after Algorithm 3), computed here exactly with rationals.
# ----------------------------------------------------------------------------------------
def _first_two_terms(x: Fraction, m: int, b16: Fraction) -> Fraction:
    if m == 15:
        return abs(Fraction(1, math.factorial(16)) - b16) * x ** 16 + x ** 17 / math.factorial(17)
    return x ** (m + 1) / math.factorial(m + 1) + x ** (m + 2) / math.factorial(m + 2)


def _expected_for_scalar(x: float, eps: float):
    xf, ef = Fraction(x), Fraction(eps)
    b16 = Fraction(oracle_b16())
    for m in (1, 2, 4, 8, 15):
        if _first_two_terms(xf, m, b16) <= ef:
            return m, 0
    # scaling: smallest s with each of the two terms of order 15+ <= eps after x -> x/2^s
    s = 0
    while s < 20:
        y = xf / 2 ** s
        t1 = abs(Fraction(1, math.factorial(16)) - b16) * y ** 16
        t2 = y ** 17 / math.factorial(17)
        if t1 <= ef and t2 <= ef:
            break
        s += 1
    return 15, s


@pytest.mark.parametrize("eps", [U64, U32, 1e-8])
def test_selection_on_scalar_matrices_matches_exact_rational_rule(eps):
    rng = np.random.default_rng(7)
    xs = np.concatenate([10.0 ** rng.uniform(-9, 3.5, 400), [1e-12, 0.5, 1.0, 12.8, 1e4, 1e7]])
    for x in xs:
        x = float(x)
        exp_m, exp_s = _expected_for_scalar(x, eps)
        # skip draws that sit on a switch point to within rounding of the floating-point rule
        lo, hi = _expected_for_scalar(x * (1 - 1e-9), eps), _expected_for_scalar(x * (1 + 1e-9), eps)
        if lo != hi:
            continue
        # the product x*x inside the oracle rounds, hence norms via a diagonal matrix are x and fl(x*x)
        got = oracle_select(x * np.eye(3), eps)
        assert (got["m"], got["s"]) == (exp_m, exp_s), (x, eps, got)


def test_selection_switch_points_of_scalar_matrices():
    """Just below / just above each closed-form switch point the order changes as it must."""
    from scipy.optimize import brentq
    for eps in (U64, U32, 1e-8):
        b16 = oracle_b16()
        for m, nxt in ((1, 2), (2, 4), (4, 8), (8, 15)):
            f = lambda x: x ** (m + 1) / math.factorial(m + 1) + x ** (m + 2) / math.factorial(m + 2) - eps
            x0 = brentq(f, 1e-12, 10.0, xtol=1e-18, rtol=1e-15)
            below = oracle_select_from_norms(x0 * (1 - 1e-5), (x0 * (1 - 1e-5)) ** 2, eps)
            above = oracle_select_from_norms(x0 * (1 + 1e-5), (x0 * (1 + 1e-5)) ** 2, eps)
            assert below == (m, 0) and above == (nxt, 0), (eps, m, x0, below, above)
        g = lambda x: abs(1 / math.factorial(16) - b16) * x ** 16 + x ** 17 / math.factorial(17) - eps
        x0 = brentq(g, 1e-3, 50.0, xtol=1e-18, rtol=1e-15)
        assert oracle_select_from_norms(x0 * (1 - 1e-5), (x0 * (1 - 1e-5)) ** 2, eps) == (15, 0)
        # Algorithm 4 accepts on the SUM of the two terms but scales on each term alone, so just
        # above the acceptance point both terms are still <= eps and the scaling stays 0 ...
        assert oracle_select_from_norms(x0 * (1 + 1e-5), (x0 * (1 + 1e-5)) ** 2, eps) == (15, 0)
        # ... and s = 1 starts where the larger single term crosses eps
        h = lambda x: max(abs(1 / math.factorial(16) - b16) * x ** 16, x ** 17 / math.factorial(17)) - eps
        x1 = brentq(h, 1e-3, 50.0, xtol=1e-18, rtol=1e-15)
        assert x1 > x0
        assert oracle_select_from_norms(x1 * (1 - 1e-5), (x1 * (1 - 1e-5)) ** 2, eps) == (15, 0)
        assert oracle_select_from_norms(x1 * (1 + 1e-5), (x1 * (1 + 1e-5)) ** 2, eps) == (15, 1)


def test_selection_uses_the_norm_of_w_squared_not_the_square_of_the_norm():
    """Non-normal matrix: ||W^2|| << ||W||^2 must lower the scaling (the point of Remark 1)."""
    W = np.array([[1.0, 1e3], [0.0, -1.0]])
    got = oracle_select(W, 1e-8)
    assert got["n2"] == 1.0 and got["n1"] == 1001.0
    # from the bounds of the table after Algorithm 4 with n2 = 1:
    #   E1 = |1/16!-b16| < 1e-8 and E2 = 1001/17! = 2.8e-12 < 1e-8, sum <= eps -> no scaling at all
    assert (got["m"], got["s"]) == (15, 0)
    # whereas a normal matrix of the same norm needs heavy scaling
    m, s = oracle_select_from_norms(1001.0, 1001.0 ** 2, 1e-8)
    assert m == 15 and s >= 9


def test_selection_cap_and_monotonicity():
    assert oracle_select_from_norms(1e30, 1e60, U64) == (15, 20)
    assert oracle_select_from_norms(1e200, 1e300, U64) == (15, 20)  # overflow of the bound -> cap
    prev = 0
    for x in np.logspace(0, 5, 60):
        m, s = oracle_select_from_norms(x, x * x, U64)
        assert m == 15 and s >= prev
        prev = s


def test_selection_scaling_formula_by_hand():
    # x = 100, eps = 2^-53, normal: E1 = |1/16!-b16| * 100^16 ; E2 = 100^17/17!
    eps, x = U64, 100.0
    E1 = abs(1 / math.factorial(16) - oracle_b16()) * 1e32
    E2 = 1e34 / math.factorial(17)
    s = max(math.ceil(math.log2(E1 / eps) / 16), math.ceil(math.log2(E2 / eps) / 17))
    assert oracle_select_from_norms(x, x * x, eps) == (15, s)
    assert s == 8  # log2(2.17e18 * 9.0e15)/16 = 7.6 ; log2(2.81e19 * 9.0e15)/17 = 7.4


def test_near_flag_marks_only_matrices_close_to_a_switch_point():
    from scipy.optimize import brentq
    eps = U64
    f = lambda x: x ** 9 / math.factorial(9) + x ** 10 / math.factorial(10) - eps
    x0 = brentq(f, 1e-3, 1.0, xtol=1e-18, rtol=1e-15)
    assert oracle_select(x0 * (1 + 1e-8) * np.eye(2), eps)["near"] is True
    assert oracle_select(x0 * (1 + 1e-3) * np.eye(2), eps)["near"] is False
    assert oracle_select(x0 * (1 - 1e-3) * np.eye(2), eps)["near"] is False


# ----------------------------------------------------------------------------------------
# the polynomial: oracle's direct summation against the paper's evaluation formulas with the
# printed coefficients, evaluated independently here (long double, scalars and small matrices)
# ----------------------------------------------------------------------------------------
def _paper_formula(A, I, co8, co15, m):
    """Evaluate T_m(A) with the formulas of Sec. 3.1 on numpy operands (matrix or 1x1)."""
    A2 = A @ A
    if m == 1:
        return A + I
    if m == 2:
        return A2 / 2 + A + I
    if m == 4:
        return ((A2 / 4 + A) / 3 + I) @ A2 / 2 + A + I
    if m == 8:
        c = co8
        y02 = A2 @ (c["c1"] * A2 + c["c2"] * A)
        return (y02 + c["c3"] * A2 + c["c4"] * A) @ (y02 + c["c5"] * A2) + c["c6"] * y02 + A2 / 2 + A + I
    c = co15
    y02 = A2 @ (c["c1"] * A2 + c["c2"] * A)
    y12 = (y02 + c["c3"] * A2 + c["c4"] * A) @ (y02 + c["c5"] * A2) + c["c6"] * y02 + c["c7"] * A2
    return ((y12 + c["c8"] * A2 + c["c9"] * A) @ (y12 + c["c10"] * y02 + c["c11"] * A)
            + c["c12"] * y12 + c["c13"] * y02 + c["c14"] * A2 + c["c15"] * A + c["c16"] * I)


def _eps_selecting(m_wanted, x):
    """A tolerance for which W = x*I gets order m_wanted with s = 0 (found by search)."""
    for e in np.logspace(2, -16, 400):
        if oracle_select_from_norms(x, x * x, e) == (m_wanted, 0):
            return float(e)
    raise AssertionError("no tolerance found")


@pytest.mark.parametrize("m", [1, 2, 4, 8, 15])
def test_polynomial_equals_paper_formulas_on_scalars(m, golden_dir):
    co = read_coefficients(os.path.join(golden_dir, "paper_coefficients.txt"))
    co8 = {k: np.longdouble(v) for k, v in co["T8"].items()}
    co15 = {k: np.longdouble(v) for k, v in co["T15+"].items()}
    for x in (0.37, -0.81, 1.6):
        eps = _eps_selecting(m, abs(x))
        X, info = oracle_expm(np.array([[x]]), eps)
        assert (info["m"], info["s"]) == (m, 0)
        A = np.array([[np.longdouble(x)]])
        ref = _paper_formula(A, np.array([[np.longdouble(1)]]), co8, co15, m)[0, 0]
        assert abs(X[0, 0] - float(ref)) <= 4e-15 * abs(float(ref)), (m, x, X[0, 0], float(ref))
    if m == 15:
        # the b16*A^16 term is really there: T_15 alone is measurably different at x = 1.6
        x = 1.6
        t15 = sum(Fraction(x) ** k / math.factorial(k) for k in range(16))
        X, _ = oracle_expm(np.array([[x]]), _eps_selecting(15, x))
        extra = X[0, 0] - float(t15)
        assert extra == pytest.approx(oracle_b16() * x ** 16, rel=1e-4)


@pytest.mark.parametrize("m", [2, 4, 8, 15])
def test_polynomial_equals_paper_formulas_on_small_matrices(m, golden_dir):
    co = read_coefficients(os.path.join(golden_dir, "paper_coefficients.txt"))
    rng = np.random.default_rng(100 + m)
    for n in (2, 3, 5):
        W = rng.standard_normal((n, n))
        W *= 0.9 / np.abs(W).sum(0).max()
        # find a tolerance that selects exactly this order without scaling
        eps = None
        for e in np.logspace(-1, -16, 300):
            g = oracle_select(W, float(e))
            if (g["m"], g["s"]) == (m, 0):
                eps = float(e)
                break
        assert eps is not None
        X, info = oracle_expm(W, eps)
        ref = _paper_formula(W.astype(np.longdouble), np.eye(n, dtype=np.longdouble), co["T8"], co["T15+"], m)
        err = np.linalg.norm((X - ref.astype(np.float64))) / np.linalg.norm(ref.astype(np.float64))
        assert err < 5e-15, (m, n, err)


def test_coefficient_tables_expand_to_taylor_coefficients(golden_dir):
    """The printed tables reproduce 1/k! (k<=8, resp. k<=15) and b16 at degree 16 (Sec. 3.1, note 3)."""
    from numpy.polynomial import polynomial as P
    co = read_coefficients(os.path.join(golden_dir, "paper_coefficients.txt"))
    x, x2, one = np.array([0.0, 1.0]), np.array([0.0, 0.0, 1.0]), np.array([1.0])
    c = co["T8"]
    y02 = P.polymul(x2, P.polyadd(c["c1"] * x2, c["c2"] * x))
    t8 = P.polyadd(P.polymul(P.polyadd(y02, P.polyadd(c["c3"] * x2, c["c4"] * x)), P.polyadd(y02, c["c5"] * x2)),
                   P.polyadd(c["c6"] * y02, P.polyadd(x2 / 2, P.polyadd(x, one))))
    assert len(t8) == 9
    for k in range(9):
        assert t8[k] * math.factorial(k) == pytest.approx(1.0, abs=2e-14)
    c = co["T15+"]
    y02 = P.polymul(x2, P.polyadd(c["c1"] * x2, c["c2"] * x))
    y12 = P.polyadd(P.polymul(P.polyadd(y02, P.polyadd(c["c3"] * x2, c["c4"] * x)), P.polyadd(y02, c["c5"] * x2)),
                    P.polyadd(c["c6"] * y02, c["c7"] * x2))
    lin = P.polyadd(c["c12"] * y12, P.polyadd(c["c13"] * y02, P.polyadd(c["c14"] * x2, P.polyadd(c["c15"] * x, c["c16"] * one))))
    y22 = P.polyadd(P.polymul(P.polyadd(y12, P.polyadd(c["c8"] * x2, c["c9"] * x)),
                              P.polyadd(y12, P.polyadd(c["c10"] * y02, c["c11"] * x))), lin)
    assert len(y22) == 17
    for k in range(16):
        assert y22[k] * math.factorial(k) == pytest.approx(1.0, abs=5e-12), k
    assert y22[16] == pytest.approx(co["b16"]["b16"], rel=1e-12)


# ----------------------------------------------------------------------------------------
# whole expm: closed forms and invariants
# ----------------------------------------------------------------------------------------
def _relerr(X, E):
    return np.linalg.norm(X - E) / np.linalg.norm(E)


def test_expm_of_diagonal_matrix():
    d = np.array([-3.0, -0.5, 0.0, 0.25, 1.0, 2.5, 4.0])
    X, info = oracle_expm(np.diag(d), U64)
    assert np.array_equal(X - np.diag(np.diag(X)), np.zeros_like(X))  # off-diagonal exactly zero
    assert np.allclose(np.diag(X), np.exp(d), rtol=2e-13, atol=0)
    assert info["m"] == 15 and info["s"] >= 2


def test_expm_of_nilpotent_matrices_is_a_finite_series():
    # index-2 nilpotent: e^W = I + W exactly; n2 = 0 makes order 2 pass immediately
    W = np.zeros((4, 4))
    W[0, 3] = 7.0
    X, info = oracle_expm(W, U64)
    assert (info["m"], info["s"]) == (2, 0)
    assert np.array_equal(X, np.eye(4) + W)
    # strictly upper triangular 4x4: e^W = I + W + W^2/2 + W^3/6
    N = np.triu(np.arange(1.0, 17.0).reshape(4, 4), 1) / 8.0
    X, info = oracle_expm(N, U64)
    E = np.eye(4) + N + N @ N / 2 + N @ N @ N / 6
    assert _relerr(X, E) < 1e-14


@pytest.mark.parametrize("theta", [1e-3, 0.4, 2.0, 31.0])
def test_expm_of_skew_generator_is_a_rotation(theta):
    W = np.array([[0.0, -theta], [theta, 0.0]])
    X, info = oracle_expm(W, U64)
    E = np.array([[math.cos(theta), -math.sin(theta)], [math.sin(theta), math.cos(theta)]])
    assert np.abs(X - E).max() < 2e-14 * 2 ** info["s"]


def test_expm_of_remark1_matrix_closed_form():
    # W^2 = I  =>  e^W = cosh(1) I + sinh(1) W
    b = 10.0
    X, info = oracle_expm(np.array([[1.0, b], [0.0, -1.0]]), 1e-8)
    E = np.array([[math.e, b * math.sinh(1.0)], [0.0, 1.0 / math.e]])
    assert (info["m"], info["s"]) == (15, 0)
    assert X[1, 0] == 0.0
    assert np.abs(X - E).max() < 1e-13  # truncation after degree 16 at norm(W^2)=1 is ~5e-14


def test_det_trace_and_inverse_identities():
    rng = np.random.default_rng(3)
    for n, scale in ((3, 0.3), (6, 2.0), (8, 9.0)):
        W = rng.standard_normal((n, n)) * scale / math.sqrt(n)
        X, _ = oracle_expm(W, U64)
        Y, _ = oracle_expm(-W, U64)
        assert np.linalg.det(X) == pytest.approx(math.exp(np.trace(W)), rel=1e-11)
        assert np.abs(oracle_matmul(X, Y) - np.eye(n)).max() < 1e-10


def test_upper_triangular_input_keeps_structure_and_diagonal():
    rng = np.random.default_rng(5)
    n = 9
    W = np.triu(rng.standard_normal((n, n)))
    X, info = oracle_expm(W, U64)
    assert np.array_equal(np.tril(X, -1), np.zeros((n, n)))
    assert np.allclose(np.diag(X), np.exp(np.diag(W)), rtol=1e-12, atol=0)


def _brute_force_expm_longdouble(W):
    """e^W by heavy scaling (||W/2^j|| <= 2^-10), 30 Taylor terms, j squarings, in long double."""
    Wl = np.asarray(W, dtype=np.longdouble)
    n = Wl.shape[0]
    nrm = float(np.abs(W).sum(0).max())
    j = max(0, int(math.ceil(math.log2(max(nrm, 1e-300)))) + 10)
    A = Wl / np.longdouble(2.0) ** j
    X = np.eye(n, dtype=np.longdouble)
    term = np.eye(n, dtype=np.longdouble)
    for k in range(1, 31):
        term = (term @ A) / np.longdouble(k)
        X = X + term
    for _ in range(j):
        X = X @ X
    return X


@pytest.mark.parametrize("seed,n,norm", [(0, 2, 0.01), (1, 3, 0.6), (2, 4, 3.0), (3, 6, 20.0), (4, 8, 150.0)])
def test_against_brute_force_long_double_series(seed, n, norm):
    rng = np.random.default_rng(seed)
    W = rng.standard_normal((n, n))
    W *= norm / np.abs(W).sum(0).max()
    X, info = oracle_expm(W, U64)
    E = _brute_force_expm_longdouble(W).astype(np.float64)
    # the selection must deliver roughly the tolerance on the scaled matrix; squaring s times
    # amplifies rounding and truncation by about 2^s relative to ||e^W||, times the conditioning
    bound = 200 * U64 * 2 ** info["s"] * max(1.0, norm)
    assert _relerr(X, E) < bound, (_relerr(X, E), bound, info)


@pytest.mark.parametrize("eps", [1e-3, 1e-5, 1e-8, 1e-11])
def test_selection_delivers_the_requested_tolerance(eps):
    """Absolute error of the polynomial on the scaled matrix stays near eps (Theorem 2 + eq. for s)."""
    rng = np.random.default_rng(11)
    for n, norm in ((3, 0.2), (5, 1.5), (8, 12.8)):
        W = rng.standard_normal((n, n))
        W *= norm / np.abs(W).sum(0).max()
        g = oracle_select(W, eps)
        A = W / 2.0 ** g["s"]
        # the oracle on A with the same tolerance must not scale again and keep the same order
        X, info = oracle_expm(A, eps)
        if info["s"] != 0 or info["m"] != g["m"]:
            continue  # A sits within rounding of a switch point
        E = _brute_force_expm_longdouble(A).astype(np.float64)
        err1 = np.abs(X - E).sum(0).max()
        assert err1 <= 2.5 * eps, (eps, n, norm, g, err1)


def test_zero_matrix_and_batch_driver_agree_with_single_calls():
    rng = np.random.default_rng(21)
    stack = rng.standard_normal((5, 6, 6)) * np.array([0.0, 1e-9, 0.1, 1.0, 30.0])[:, None, None]
    X, info = oracle_expm_batch(stack, U64)
    assert np.array_equal(X[0], np.eye(6)) and (info["m"][0], info["s"][0]) == (0, 0)
    assert info["m"][1] == 1 and np.array_equal(X[1], np.eye(6) + stack[1])
    for b in range(5):
        Xb, ib = oracle_expm(stack[b], U64)
        assert np.array_equal(X[b], Xb) and ib["m"] == info["m"][b] and ib["s"] == info["s"][b]


def test_fp32_inputs_are_widened_exactly():
    rng = np.random.default_rng(8)
    W32 = (rng.standard_normal((4, 4)) * 0.5).astype(np.float32)
    X32, i32 = oracle_expm(W32, U32)
    X64, i64 = oracle_expm(W32.astype(np.float64), U32)
    assert np.array_equal(X32, X64) and i32 == i64


def test_oracle_default_thread_count_survives_an_explicit_one():
    """A batch call with threads=1 must not turn later "all threads" calls into one-thread calls (the benchmark
    times the oracle both ways in one process)."""
    from oracle import oracle_expm_batch, oracle_max_threads
    a = np.random.default_rng(77).standard_normal((8, 6, 6)) * 0.2
    _, first = oracle_expm_batch(a, 1e-8)
    _, one = oracle_expm_batch(a, 1e-8, threads=1)
    _, again = oracle_expm_batch(a, 1e-8)
    assert one["threads"] == 1
    assert first["threads"] == again["threads"] == oracle_max_threads()
