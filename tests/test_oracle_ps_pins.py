"""Pins of the oracle's Paterson-Stockmeyer variant (Algorithm 3 + plain Taylor polynomial), no GPU."""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import oracle_expm_ps_batch, oracle_select_ps, oracle_select_ps_from_norms

U64 = 2.0 ** -53
U32 = 2.0 ** -24


def _table(golden_dir):
    rows = []
    with open(os.path.join(golden_dir, "paper_ps_table.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            rows.append(tuple(int(x) for x in line.split()))
    return rows  # (m, j, k, c1den, c2den, products)


def _expected_from_table(table, norms, eps):
    """Algorithm 3 evaluated exactly (rationals) from the printed table; s by brute force over the two terms."""
    n = [Fraction(x) for x in norms]
    e = Fraction(eps)
    if n[0] == 0:
        return 0, 0
    E1 = E2 = None
    for (m, j, k, d1, d2, _p) in table:
        if m == 1:
            E1, E2 = n[0] ** 2 / math.factorial(2), n[0] ** 3 / math.factorial(3)
        else:
            E1 = n[j - 1] ** k * n[0] / math.factorial(d1)
            E2 = n[j - 1] ** k * n[1] / math.factorial(d2)
        if E1 + E2 <= e:
            return m, 0
    # smallest s >= 0 with E1 / 2^(17 s) <= eps and E2 / 2^(18 s) <= eps  (ceil(log2(E_i/eps)/(16+i)) each)
    s = 0
    while s < 20 and not (E1 / Fraction(2) ** (17 * s) <= e and E2 / Fraction(2) ** (18 * s) <= e):
        s += 1
    return 16, s


def test_table_matches_the_printed_vectors(golden_dir):
    t = _table(golden_dir)
    assert [r[0] for r in t] == [1, 2, 4, 6, 9, 12, 16]                       # M
    assert [r[1] for r in t] == [math.ceil(math.sqrt(r[0])) for r in t]       # J = ceil(sqrt(M))
    assert all(r[1] * r[2] == r[0] for r in t)                                # K = M./J
    assert [(r[3], r[4]) for r in t] == [(r[0] + 1, r[0] + 2) for r in t]     # C holds 1/(m+1)!, 1/(m+2)!
    assert all(r[5] == (0 if r[0] < 2 else r[1] - 1 + r[2] - 1) for r in t)   # powers + Horner steps (Table 1)


@pytest.mark.parametrize("eps", [U64, U32, 1e-8])
def test_selection_on_random_norm_tuples_matches_the_table(eps, golden_dir):
    table = _table(golden_dir)
    rng = np.random.default_rng(31)
    checked = 0
    for _ in range(600):
        n1 = float(10.0 ** rng.uniform(-9, 3))
        # sub-multiplicative tuples, possibly far below n1^r (non-normal matrices)
        n2 = n1 * n1 * float(10.0 ** rng.uniform(-2, 0))
        n3 = min(n2 * n1, n1 ** 3) * float(10.0 ** rng.uniform(-2, 0))
        n4 = min(n3 * n1, n2 * n2) * float(10.0 ** rng.uniform(-2, 0))
        exp = _expected_from_table(table, (n1, n2, n3, n4), eps)
        # skip tuples within rounding of a switch point
        lo = _expected_from_table(table, [x * (1 - 1e-9) for x in (n1, n2, n3, n4)], eps)
        hi = _expected_from_table(table, [x * (1 + 1e-9) for x in (n1, n2, n3, n4)], eps)
        if lo != hi:
            continue
        assert oracle_select_ps_from_norms(n1, n2, n3, n4, eps) == exp, (n1, n2, n3, n4, eps)
        checked += 1
    assert checked > 500


def test_each_order_is_reachable_and_uses_its_own_power(golden_dir):
    """Order m = j*k must look at ||W^j|| (and not at another power): make all other powers hopeless."""
    eps = 1e-8
    big = 1e6
    for (m, j, k, d1, d2, _p) in _table(golden_dir)[2:]:   # m >= 4
        norms = [1.0, 1.0, big, big]
        norms[j - 1] = 1e-3 if j > 2 else 1.0
        if j == 2:
            norms = [0.05 if m == 4 else 1.0, 0.0025 if m == 4 else 1.0, big, big]
        got = oracle_select_ps_from_norms(*norms, eps)
        exp = _expected_from_table(_table(golden_dir), norms, eps)
        assert got == exp
    # a tuple built so that exactly order 12 is the first to pass (needs ||W^4||, rejects via ||W^3||)
    norms = [2.0, 4.0, 8.0, 1e-2]
    assert oracle_select_ps_from_norms(*norms, 1e-8) == _expected_from_table(_table(golden_dir), norms, 1e-8) == (12, 0)


@pytest.mark.parametrize("eps", [U64, 1e-8])
def test_scalar_matrices_get_the_smallest_sufficient_order(eps, golden_dir):
    """W = x I: every ||W^r|| = x^r, so the rule is 'first two remainder terms <= eps' over M (paper, after Alg. 3)."""
    rng = np.random.default_rng(5)
    for x in 10.0 ** rng.uniform(-8, 2.5, 150):
        x = float(x)
        xf, ef = Fraction(x), Fraction(eps)
        exp = None
        for m in (1, 2, 4, 6, 9, 12, 16):
            if xf ** (m + 1) / math.factorial(m + 1) + xf ** (m + 2) / math.factorial(m + 2) <= ef:
                exp = (m, 0)
                break
        got = oracle_select_ps(x * np.eye(3), eps)
        if exp is None:
            assert got["m"] == 16 and got["s"] >= 0
            y = xf / 2 ** got["s"]
            assert y ** 17 / math.factorial(17) <= ef * (1 + Fraction(1, 10 ** 9))
            if got["s"] > 0:
                y2 = xf / 2 ** (got["s"] - 1)
                assert max(y2 ** 17 / math.factorial(17), y2 ** 18 / math.factorial(18)) > ef * (1 - Fraction(1, 10 ** 9))
        elif not got["near"]:
            assert (got["m"], got["s"]) == exp, (x, eps, got)


@pytest.mark.parametrize("m", [1, 2, 4, 6, 9, 12, 16])
def test_polynomial_is_the_taylor_polynomial_on_scalars(m):
    """1x1 'matrices': the result must be sum_{i<=m} x^i / i! exactly to rounding (rational reference)."""
    for x in (0.31, -0.77, 1.9):
        eps = None
        for e in np.logspace(2, -30, 900):
            if oracle_select_ps_from_norms(abs(x), x * x, abs(x) ** 3, x ** 4, float(e)) == (m, 0):
                eps = float(e)
                break
        assert eps is not None, (m, x)
        X, info = oracle_expm_ps_batch(np.array([[x]]), eps)
        assert (info["m"][0], info["s"][0]) == (m, 0)
        ref = float(sum(Fraction(x) ** i / math.factorial(i) for i in range(m + 1)))
        assert abs(X[0, 0, 0] - ref) <= 4e-16 * abs(ref)


def _ps_horner(A, m, j, k):
    """T_m(A) in Paterson-Stockmeyer form (powers up to A^j, Horner in A^j), plain numpy float64."""
    n = A.shape[0]
    pw = [np.eye(n), A]
    for _ in range(2, j + 1):
        pw.append(pw[-1] @ A)
    c = [1.0 / math.factorial(i) for i in range(m + 1)]
    H = sum(c[(k - 1) * j + r] * pw[r] for r in range(j + 1))
    for q in range(k - 2, -1, -1):
        H = H @ pw[j] + sum(c[q * j + r] * pw[r] for r in range(j))
    return H


def test_direct_summation_equals_the_paterson_stockmeyer_form(golden_dir):
    rng = np.random.default_rng(9)
    for (m, j, k, *_rest) in _table(golden_dir)[1:]:
        for n in (2, 4, 7):
            W = rng.standard_normal((n, n))
            W *= 0.8 / np.abs(W).sum(0).max()
            eps = None
            for e in np.logspace(1, -30, 800):
                g = oracle_select_ps(W, float(e))
                if (g["m"], g["s"]) == (m, 0):
                    eps = float(e)
                    break
            assert eps is not None, (m, n)
            X, info = oracle_expm_ps_batch(W, eps)
            ref = _ps_horner(W, m, j, k)
            assert np.linalg.norm(X[0] - ref) / np.linalg.norm(ref) < 5e-15


def test_closed_forms_and_brute_force():
    d = np.array([-2.0, -0.3, 0.0, 0.7, 3.0])
    X, info = oracle_expm_ps_batch(np.diag(d), U64)
    assert np.allclose(np.diag(X[0]), np.exp(d), rtol=2e-13, atol=0)
    th = 0.9
    X, _ = oracle_expm_ps_batch(np.array([[0.0, -th], [th, 0.0]]), U64)
    assert np.abs(X[0] - np.array([[math.cos(th), -math.sin(th)], [math.sin(th), math.cos(th)]])).max() < 1e-14
    # Remark-1 matrix: W^2 = I, e^W = cosh(1) I + sinh(1) W ; truncation after degree 12 is ~ 1/13! * 11
    X, info = oracle_expm_ps_batch(np.array([[1.0, 10.0], [0.0, -1.0]]), 1e-8)
    assert (info["m"][0], info["s"][0]) == (12, 0)   # ||W^4|| = 1: order 12 passes without scaling
    E = np.array([[math.e, 10.0 * math.sinh(1.0)], [0.0, 1.0 / math.e]])
    assert np.abs(X[0] - E).max() < 1e-8
    # zero matrix and tiny norm
    X, info = oracle_expm_ps_batch(np.zeros((1, 3, 3)), U64)
    assert (info["m"][0], info["s"][0]) == (0, 0) and np.array_equal(X[0], np.eye(3))


def test_both_schemes_of_the_oracle_agree_on_the_exponential():
    from oracle import oracle_expm_batch
    rng = np.random.default_rng(2)
    stack = rng.standard_normal((6, 9, 9)) * np.array([1e-6, 1e-2, 0.2, 1.0, 5.0, 40.0])[:, None, None] / 3.0
    Xa, ia = oracle_expm_batch(stack, U64)
    Xb, ib = oracle_expm_ps_batch(stack, U64)
    for b in range(6):
        assert np.linalg.norm(Xa[b] - Xb[b]) / np.linalg.norm(Xa[b]) < 1e-12 * 2 ** max(ia["s"][b], ib["s"][b])
