"""Pins for oracle/prism_ref.py against what the paper and the mathematics fix (CPU only).

Each test names what it would catch.  No expected value comes from the HIP path.
"""
import os
from math import comb

import numpy as np
import pytest

from oracle import gauss_sketch as gs
from oracle import prism_ref as P

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rng(seed):
    return np.random.default_rng(seed)


def _sym_with_eigs(lam, seed):
    q, _ = np.linalg.qr(_rng(seed).standard_normal((len(lam), len(lam))))
    return (q * lam) @ q.T


def _tall(m, n, cond, seed):
    r = _rng(seed)
    u, _ = np.linalg.qr(r.standard_normal((m, n)))
    v, _ = np.linalg.qr(r.standard_normal((n, n)))
    s = np.logspace(0, -np.log10(cond), n)
    return (u * s) @ v.T, u @ v.T


# ----------------------------------------------------------------- (i) limits

@pytest.mark.parametrize("degree", [3, 5])
@pytest.mark.parametrize("shape", [(40, 24), (24, 24), (16, 48)])
def test_polar_limit_is_svd_polar_factor(degree, shape):
    m, n = shape
    if m >= n:
        A, UVt = _tall(m, n, 200.0, 3)
    else:
        At, UVtt = _tall(n, m, 200.0, 3)
        A, UVt = At.T, UVtt.T
    X, info = P.polar(A, degree, 60, 8, 11, 1e-13)
    assert info["status"] == P.STATUS_CONVERGED
    assert np.linalg.norm(X - UVt) < 1e-10
    k = min(m, n)
    gram = X.T @ X if m >= n else X @ X.T
    assert np.linalg.norm(gram - np.eye(k)) < 1e-11          # U^T U = I


@pytest.mark.parametrize("degree", [3, 5])
def test_sqrt_limit_is_eigh_root(degree):
    lam = np.logspace(0, -2.5, 30)
    A = _sym_with_eigs(lam, 5)
    S, Si, info = P.sqrt(A, degree, 60, 8, 7, 1e-13)
    assert info["status"] == P.STATUS_CONVERGED
    w, q = np.linalg.eigh(A)
    assert np.linalg.norm(S - (q * np.sqrt(w)) @ q.T) < 1e-10
    assert np.linalg.norm(Si - (q / np.sqrt(w)) @ q.T) < 1e-8
    assert np.linalg.norm(S @ S - A) < 1e-10                    # S^2 = A
    assert np.linalg.norm(S @ Si - np.eye(30)) < 1e-9           # X Y = I


@pytest.mark.parametrize("p", [1, 2, 3, 4])
def test_inv_root_limit_is_eigh_root(p):
    lam = np.logspace(0, -2, 24)
    A = _sym_with_eigs(lam, 9)
    X, info = P.inv_root(A, p, 80, 8, 3, 1e-13)
    assert info["status"] == P.STATUS_CONVERGED
    w, q = np.linalg.eigh(A)
    assert np.linalg.norm(X - (q * w ** (-1.0 / p)) @ q.T) < 1e-9
    assert np.linalg.norm(np.linalg.matrix_power(X, p) @ A - np.eye(24)) < 1e-9   # (A^-1/p)^p A = I


# ------------------------------------------- (ii) special case: classical iteration

def test_polar_without_fit_is_classical_newton_schulz():
    A, _ = _tall(30, 12, 50.0, 1)
    for degree, steps in ((3, 9), (5, 6)):
        X, info = P.polar(A, degree, steps, 0, 1, 0.0)
        Z = A / np.linalg.norm(A)
        for _ in range(steps):
            B = Z.T @ Z
            if degree == 3:
                Z = 1.5 * Z - 0.5 * Z @ B                                  # 3/2 X - 1/2 X^3
            else:
                Z = 15 / 8 * Z - 10 / 8 * Z @ B + 3 / 8 * Z @ B @ B        # 15/8, -10/8, 3/8
        assert info["iters"] == steps and info["status"] == P.STATUS_BUDGET
        assert np.linalg.norm(X - Z) < 1e-12


def test_sqrt_without_fit_is_classical_coupled_iteration():
    A = _sym_with_eigs(np.linspace(0.2, 1.0, 10), 2)
    S, Si, info = P.sqrt(A, 3, 7, 0, 1, 0.0)
    s = np.linalg.norm(A)
    Y, Z = A / s, np.eye(10)
    for _ in range(7):
        T = 0.5 * (3 * np.eye(10) - Z @ Y)          # textbook coupled Newton-Schulz for the square root
        Y, Z = Y @ T, T @ Z
    assert np.linalg.norm(S - np.sqrt(s) * Y) < 1e-12
    assert np.linalg.norm(Si - Z / np.sqrt(s)) < 1e-12


def test_inv_root_without_fit_is_classical_inverse_newton():
    A = _sym_with_eigs(np.linspace(0.1, 1.0, 8), 4)
    p = 3
    X, info = P.inv_root(A, p, 6, 0, 1, 0.0)
    c = (2 * np.linalg.norm(A) / (p + 1)) ** (1 / p)
    Z, M = np.eye(8) / c, A / c ** p
    for _ in range(6):
        T = ((p + 1) * np.eye(8) - M) / p
        Z, M = Z @ T, np.linalg.matrix_power(T, p) @ M
    assert np.linalg.norm(X - Z) < 1e-12
    assert info["alpha"] == [1 / p] * 6


# ------------------------------------------------------- (iii) invariants, Theorem 1

def test_exact_fit_beats_every_other_alpha():
    """alpha* minimises the next residual over [l, u] (eq. (2)-(3)), in particular it is
    no worse than the Taylor value: catches a wrong sign or index in any W block."""
    A, _ = _tall(20, 14, 300.0, 8)
    X = A / np.linalg.norm(A)
    for _ in range(3):
        X = X @ P.g_poly(np.eye(14) - X.T @ X, 2, 1.45)
    G = X.T @ X
    R = np.eye(14) - G
    for d in (1, 2):
        lo, hi = P.clamp_interval(d)
        a_star = P.fit_alpha_ns(R, G, np.eye(14), d)
        def next_res(a):
            Xn = X @ P.g_poly(R, d, a)
            return np.linalg.norm(np.eye(14) - Xn.T @ Xn)
        grid = np.linspace(lo, hi, 4001)
        vals = np.array([next_res(a) for a in grid])
        assert next_res(a_star) <= vals.min() * (1 + 1e-9)
        assert abs(a_star - grid[vals.argmin()]) <= (hi - lo) / 4000 * 1.01


def test_theorem1_bound_exact_fit_d1():
    """||R_k||_2 <= ||R_0||_2^(2^(k-2)) for d = 1 with exact fit on [1/2, 1] (Theorem 1).
    For a symmetric positive definite input the polar iteration is the sign iteration."""
    lam = np.concatenate([np.logspace(-6, 0, 25), [0.3, 0.31]])
    A = _sym_with_eigs(lam, 12)
    A = A / np.linalg.norm(A, 2)                # ||A||_2 = 1; polar() divides by ||A||_F again (allowed: <= 1)
    X = A / np.linalg.norm(A)
    r0 = np.linalg.norm(np.eye(27) - X.T @ X, 2)
    n = 27
    for k in range(0, 40):
        G = X.T @ X
        R = np.eye(n) - G
        rk = np.linalg.norm(R, 2)
        assert rk <= r0 ** (2.0 ** (k - 2)) + 1e-12
        if rk < 1e-13:
            break
        X = X @ P.g_poly(R, 1, P.fit_alpha_ns(R, G, np.eye(n), 1))
    assert rk < 1e-13


def test_scale_and_rotation_invariance():
    A, _ = _tall(18, 10, 100.0, 21)
    X1, i1 = P.polar(A, 5, 40, 8, 5, 1e-12)
    X2, i2 = P.polar(37.5 * A, 5, 40, 8, 5, 1e-12)
    assert np.allclose(X1, X2, atol=1e-12) and np.allclose(i1["alpha"], i2["alpha"], atol=1e-12)
    q, _ = np.linalg.qr(_rng(1).standard_normal((18, 18)))
    z, _ = np.linalg.qr(_rng(2).standard_normal((10, 10)))
    _, ie = P.polar(A, 5, 40, 0, 5, 1e-12, exact_fit=True)
    _, ir = P.polar(q @ A @ z.T, 5, 40, 0, 5, 1e-12, exact_fit=True)
    assert np.allclose(ie["alpha"], ir["alpha"], atol=1e-8)


def test_residual_history_and_counts():
    A, _ = _tall(20, 10, 30.0, 4)
    X, info = P.polar(A, 5, 40, 8, 1, 1e-8)
    assert len(info["residual"]) == info["iters"] + 1 == len(info["alpha"]) + 1
    assert info["residual"][-1] <= 1e-8 < info["residual"][-2]
    Z = A / np.linalg.norm(A)
    assert abs(info["residual"][0] - np.linalg.norm(np.eye(10) - Z.T @ Z) / np.sqrt(10)) < 1e-14
    lo, hi = P.clamp_interval(2)
    assert all(lo <= a <= hi for a in info["alpha"])
    # fixed budget: exactly max_iters updates, status "budget"
    _, fixed = P.polar(A, 5, 3, 8, 1, 0.0)
    assert fixed["iters"] == 3 and fixed["status"] == P.STATUS_BUDGET
    # alpha starts at the upper end for an ill-conditioned input and ends near the Taylor value (App. C)
    B, _ = _tall(40, 30, 1e5, 6)
    _, ib = P.polar(B, 5, 60, 8, 1, 1e-10)
    assert ib["alpha"][0] == hi and abs(ib["alpha"][-1] - lo) < 0.05


def test_degenerate_inputs():
    Z = np.zeros((5, 3))
    X, info = P.polar(Z)
    assert info["status"] == P.STATUS_ZERO and info["iters"] == 0 and not X.any()
    N = np.ones((4, 4)); N[1, 2] = np.inf
    assert P.polar(N)[1]["status"] == P.STATUS_NONFINITE
    assert P.inv_root(N, 2)[1]["status"] == P.STATUS_NONFINITE
    # indefinite input to the square root: the residual grows, reported as diverged
    A = _sym_with_eigs(np.array([1.0, 0.5, -0.8, 0.3]), 3)
    _, _, info = P.sqrt(A, 3, 60, 4, 1, 1e-10)
    assert info["status"] in (P.STATUS_DIVERGED, P.STATUS_BUDGET) and info["status"] != P.STATUS_CONVERGED


# ------------------------------------------------------------- (iv) closed forms

def _golden_scalars():
    out = {}
    for l in open(os.path.join(GOLDEN, "scalar_identities.txt")):
        if l.strip() and not l.startswith("#"):
            k, v = l.split()
            out[k] = float(v)
    return out


def test_scalar_identities_of_h():
    """n = 1: m(alpha) = h(x, alpha)^2 with h = 1 - (1-x)(1+alpha x)^2 (Lemma 1)."""
    gold = _golden_scalars()
    for x in (0.9, 0.5, 0.1, -0.2):
        R = np.array([[x]]); G = 1 - R; St = np.array([[1.0]])
        c = P.fit_coefficients_ns(R, G, St, 1)
        m = lambda a: np.polyval(c[::-1], a)
        assert abs(m(0.5) - (0.75 * x ** 2 + 0.25 * x ** 3) ** 2) < 1e-14
        assert abs(m(1.0) - (-x + x ** 2 + x ** 3) ** 2) < 1e-14
    c = P.fit_coefficients_ns(np.array([[0.5]]), np.array([[0.5]]), np.array([[1.0]]), 1)
    assert abs(np.polyval(c[::-1], 1.0) - gold["h_half_1"] ** 2) < 1e-15
    # d = 2: h_2(x, alpha) = 1 - (1-x)(1 + x/2 + alpha x^2)^2
    for x in (0.7, -0.1):
        c = P.fit_coefficients_ns(np.array([[x]]), np.array([[1 - x]]), np.array([[1.0]]), 2)
        for a in (0.375, 1.0, 1.45):
            assert abs(np.polyval(c[::-1], a) - (1 - (1 - x) * (1 + x / 2 + a * x * x) ** 2) ** 2) < 1e-14


def test_one_point_spectrum_closed_form():
    """R = lambda I: every sketch gives alpha = clamp(beta(lambda)), beta = (1/sqrt(1-l) - 1)/l,
    and an unclamped beta zeroes the next residual (proof of Lemma 1)."""
    gold = _golden_scalars()
    n = 6
    St = gs.sketch(1, 0, 1, 3, n).astype(np.float64).T
    lam = 0.25
    a = P.fit_alpha_ns(lam * np.eye(n), (1 - lam) * np.eye(n), St, 1)
    assert abs(a - gold["beta_quarter"]) < 1e-12
    assert abs(gold["beta_quarter"] - (8 / np.sqrt(3) - 4)) < 1e-15
    assert abs(1 - (1 - lam) * (1 + a * lam) ** 2) < 1e-12
    for lam, want in ((0.9, 1.0), (0.05, (1 / np.sqrt(0.95) - 1) / 0.05), (-0.2, 0.5)):
        got = P.fit_alpha_ns(lam * np.eye(n), (1 - lam) * np.eye(n), St, 1)
        assert abs(got - min(max(want, 0.5), 1.0)) < 1e-12
    # whole driver: X0 with all singular values equal converges after one fitted step
    q, _ = np.linalg.qr(_rng(3).standard_normal((9, 4)))
    X, info = P.polar(3.0 * q, 3, 10, 2, 1, 1e-12)
    # ||X0||_F-normalised: sigma = 1/2, lambda = 3/4, beta = (2 - 1)/(3/4) = 4/3 > 1 -> clamped to 1
    assert info["alpha"][0] == 1.0
    assert np.linalg.norm(X - q) < 1e-10


# ------------------------------------------------------------ (v) printed tables

def _printed_tables():
    tabs = {}
    for l in open(os.path.join(GOLDEN, "printed_m_alpha_tables.txt")):
        if not l.strip() or l.startswith("#"):
            continue
        head, body = l.split(":")
        name, idx = head.split()
        terms = [(float(t.split("*t")[0]), int(t.split("*t")[1])) for t in body.split()]
        tabs.setdefault(name, {})[int(idx)] = terms
    return tabs


def _traces(R, S, upto):
    out, Rp = [], np.eye(R.shape[0])
    for _ in range(upto + 1):
        out.append(np.trace(S @ Rp @ S.T))
        Rp = Rp @ R
    return out


@pytest.mark.parametrize("d", [1, 2])
def test_coefficients_match_printed_trace_tables_ns(d):
    tabs = _printed_tables()["ns%d" % d]
    n = 12
    R = _sym_with_eigs(_rng(5).uniform(-0.2, 0.9, n), 6)
    S = gs.sketch(9, 1, 1, 5, n).astype(np.float64)
    t = _traces(R, S, 4 * d + 2)
    c = P.fit_coefficients_ns(R, np.eye(n) - R, S.T, d)
    for idx, terms in tabs.items():
        printed = sum(coef * t[i] for coef, i in terms)
        assert abs(c[idx] - printed) < 1e-10 * max(1.0, abs(printed))


@pytest.mark.parametrize("p", [1, 2])
def test_coefficients_match_printed_trace_tables_inverse_newton(p):
    tabs = _printed_tables()["inv%d" % p]
    n = 10
    R = _sym_with_eigs(_rng(7).uniform(-0.4, 0.9, n), 8)
    S = gs.sketch(4, 0, 3, 4, n).astype(np.float64)
    t = _traces(R, S, 2 * p + 2)
    c = P.fit_coefficients_inv(R, np.eye(n) - R, S.T, p)
    assert len(c) == 2 * p + 1
    for idx, terms in tabs.items():
        printed = sum(coef * t[i] for coef, i in terms)
        assert abs(c[idx] - printed) < 1e-10 * max(1.0, abs(printed))
    assert abs(c[0] - t[2]) < 1e-10


# ------------------------------------------------ (vi) literal objective, brute force

@pytest.mark.parametrize("d", [1, 2])
def test_quartic_equals_literal_sketched_objective(d):
    """m(alpha) of eq. (4) written out: || S (I - G g_d(R; alpha)^2) ||_F^2."""
    n = 9
    A, _ = _tall(15, n, 40.0, 31)
    X = A / np.linalg.norm(A)
    G = X.T @ X
    R = np.eye(n) - G
    S = gs.sketch(2, 5, 1, 4, n).astype(np.float64) / 2.0
    c = P.fit_coefficients_ns(R, G, S.T, d)
    for a in np.linspace(0.3, 1.5, 7):
        g = P.g_poly(R, d, a)
        literal = np.linalg.norm(S @ (np.eye(n) - G @ g @ g)) ** 2
        assert abs(np.polyval(c[::-1], a) - literal) < 1e-12 * max(1.0, literal)


@pytest.mark.parametrize("p", [1, 2, 3, 4])
def test_inverse_newton_polynomial_equals_literal_objective(p):
    """m(alpha) = || S (I - (I + alpha R)^p M) ||_F^2, the next residual of App. A.3."""
    n = 8
    R = _sym_with_eigs(_rng(11).uniform(-1.2, 0.95, n), 12)
    M = np.eye(n) - R
    S = gs.sketch(3, 2, 3, 3, n).astype(np.float64)
    c = P.fit_coefficients_inv(R, M, S.T, p)
    for a in np.linspace(0.1, 1.0, 6):
        T = np.eye(n) + a * R
        literal = np.linalg.norm(S @ (np.eye(n) - np.linalg.matrix_power(T, p) @ M)) ** 2
        assert abs(np.polyval(c[::-1], a) - literal) < 1e-11 * max(1.0, literal)
        # and the form printed in the paper: R + sum_i C(p,i) alpha^i (R^{i+1} - R^i)
        acc = R.copy()
        for i in range(1, p + 1):
            acc = acc + comb(p, i) * a ** i * (np.linalg.matrix_power(R, i + 1) - np.linalg.matrix_power(R, i))
        assert abs(np.linalg.norm(S @ acc) ** 2 - literal) < 1e-11 * max(1.0, literal)


def test_minimiser_against_brute_force_grid():
    rng = _rng(17)
    for trial in range(40):
        deg = int(rng.choice([2, 4, 6, 8]))
        c = rng.standard_normal(deg + 1)
        c[-1] = abs(c[-1]) + 0.1
        lo, hi = sorted(rng.uniform(-1.5, 1.5, 2))
        a = P.minimize_poly_on_interval(c, lo, hi)
        grid = np.linspace(lo, hi, 200001)
        vals = np.polyval(c[::-1], grid)
        assert lo <= a <= hi
        assert np.polyval(c[::-1], a) <= vals.min() + 1e-9 * (1 + abs(vals.min()))
    # degenerate: constant / zero polynomial, and minimum at an end point
    assert P.minimize_poly_on_interval([0, 0, 0, 0, 0], 0.375, 1.45) == 0.375
    assert P.minimize_poly_on_interval([1.0, 1.0, 0, 0, 0], 0.5, 1.0) == 0.5
    assert P.minimize_poly_on_interval([1.0, -1.0, 0, 0, 0], 0.5, 1.0) == 1.0
    assert abs(P.minimize_poly_on_interval([0.49, -1.4, 1.0, 0, 0], 0.5, 1.0) - 0.7) < 1e-12
    assert P.minimize_poly_on_interval([np.nan, 1, 1, 1, 1], 0.5, 1.0) == 0.5


# -------------------------------------------------------------- (vii) sketch quality

def test_sketched_traces_are_unbiased_and_alpha_close_to_exact():
    n = 48
    A, _ = _tall(60, n, 500.0, 41)
    X = A / np.linalg.norm(A)
    lo, hi = P.clamp_interval(2)
    for _ in range(20):                     # advance until the exact-fit alpha is interior
        G = X.T @ X
        R = np.eye(n) - G
        if lo + 0.1 < P.fit_alpha_ns(R, G, np.eye(n), 2) < hi - 0.1:
            break
        X = X @ P.g_poly(R, 2, P.fit_alpha_ns(R, G, np.eye(n), 2))
    est = np.mean([np.trace((s := gs.sketch(seed, 0, 1, 8, n).astype(np.float64) / np.sqrt(8)) @ R @ s.T)
                   for seed in range(400)])
    assert abs(est - np.trace(R)) < 0.03 * abs(np.trace(R))
    exact = P.fit_alpha_ns(R, G, np.eye(n), 2)
    assert lo < exact < hi
    sk = [P.fit_alpha_ns(R, G, gs.sketch(seed, 0, 1, n, n).astype(np.float64).T, 2) for seed in range(20)]
    assert abs(np.median(sk) - exact) < 0.1 * exact


def test_prism_needs_fewer_iterations_than_classical():
    A, _ = _tall(64, 32, 1e3, 51)
    _, fitted = P.polar(A, 5, 60, 8, 22137, 1e-6)
    _, classic = P.polar(A, 5, 60, 0, 22137, 1e-6)
    assert fitted["iters"] < classic["iters"]
    B = _sym_with_eigs(np.logspace(0, -4, 40), 52)
    _, f4 = P.inv_root(B, 4, 80, 8, 22137, 1e-8)
    _, c4 = P.inv_root(B, 4, 80, 0, 22137, 1e-8)
    assert f4["iters"] < c4["iters"]


def test_sqrt_residual_stays_at_rounding_level():
    """With the product order of Theorem 3 the coupled iteration is stable: running far past
    convergence leaves the residual at rounding level (the other order, I - X_k Y_k, grows again
    by a constant factor per step; checked here on a copy of the loop with that order)."""
    A = _sym_with_eigs(np.logspace(0, -2.5, 30), 5)
    _, _, info = P.sqrt(A, 5, 25, 0, 1, 0.0)
    assert info["iters"] == 25 and info["residual"][-1] < 1e-13
    s = np.linalg.norm(A); X = A / s; Y = np.eye(30)
    for _ in range(25):
        Pm = P.g_poly(np.eye(30) - X @ Y, 2, 0.375)
        X, Y = X @ Pm, Pm @ Y
    assert np.linalg.norm(np.eye(30) - X @ Y) > 1e-3
