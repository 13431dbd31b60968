"""Pins for the PRISM DB Newton iteration of oracle/prism_ref.py (CPU only).

Each test names what it would catch.  No expected value comes from the HIP path.
"""
import os

import numpy as np
import pytest

from oracle import prism_ref as P

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rng(seed):
    return np.random.default_rng(seed)


def _spd(lam, seed):
    q, _ = np.linalg.qr(_rng(seed).standard_normal((len(lam), len(lam))))
    a = (q * lam) @ q.T
    return 0.5 * (a + a.T), q


def test_limit_is_eigh_square_root():
    """Converged X, Y against Q diag(lambda^(+-1/2)) Q^T; a swapped (1 - a) / a weight or a missing
    identity term in M_{k+1} does not reach it."""
    lam = np.logspace(-3, 2, 24)
    A, q = _spd(lam, 1)
    X, Y, info = P.sqrt_db_newton(A, 60, 1e-13)
    assert info["status"] == P.STATUS_CONVERGED
    assert np.linalg.norm(X - (q * np.sqrt(lam)) @ q.T) < 1e-9 * np.linalg.norm(X)
    assert np.linalg.norm(Y - (q / np.sqrt(lam)) @ q.T) < 1e-9 * np.linalg.norm(Y)
    assert np.linalg.norm(X @ Y - np.eye(24)) < 1e-9


def test_without_fit_is_classical_db_newton():
    """alpha = 1/2 is the Denman-Beavers iteration X <- (X + Y^-1)/2, Y <- (Y + X^-1)/2 written
    with two inverses (App. A.2, before the product form)."""
    A, _ = _spd(np.linspace(0.5, 4.0, 9), 2)
    X, Y, info = P.sqrt_db_newton(A, 7, 0.0, fit=False)
    Xc, Yc = A.copy(), np.eye(9)
    for _ in range(7):
        Xc, Yc = 0.5 * (Xc + np.linalg.inv(Yc)), 0.5 * (Yc + np.linalg.inv(Xc))
    assert info["alpha"] == [0.5] * 7
    assert np.linalg.norm(X - Xc) < 1e-11 * np.linalg.norm(Xc)
    assert np.linalg.norm(Y - Yc) < 1e-11 * np.linalg.norm(Yc)


def test_coefficients_match_printed_traces_and_literal_objective():
    tabs = {}
    for l in open(os.path.join(GOLDEN, "printed_m_alpha_tables.txt")):
        if l.startswith("dbn"):
            head, body = l.split(":")
            tabs[int(head.split()[1])] = [(float(t.split("*t")[0]), int(t.split("*t")[1])) for t in body.split()]
    M, _ = _spd(_rng(3).uniform(0.2, 3.0, 11), 4)
    N = np.linalg.inv(M)
    t = [11.0, np.trace(M), np.trace(M @ M), np.trace(N), np.trace(N @ N)]
    c = P.db_newton_coefficients(M, N)
    assert set(tabs) == {1, 2, 3, 4}
    for idx, terms in tabs.items():
        printed = sum(coef * t[i] for coef, i in terms)
        assert abs(c[idx] - printed) < 1e-10 * max(1.0, abs(printed))
    for a in np.linspace(-0.5, 1.5, 9):      # m(alpha) written out
        Mn = 2 * a * (1 - a) * np.eye(11) + (1 - a) ** 2 * M + a * a * N
        literal = np.linalg.norm(np.eye(11) - Mn) ** 2
        assert abs(np.polyval(c[::-1], a) - literal) < 1e-10 * max(1.0, literal)


def test_product_form_keeps_m_equal_to_x_times_y():
    """M_k = X_k Y_k along the fitted iteration (how the product form is derived)."""
    A, _ = _spd(np.logspace(-1, 1, 10), 5)
    n = 10
    X, Y, M = A.copy(), np.eye(n), A.copy()
    for _ in range(4):
        N = np.linalg.inv(M)
        a = P.minimize_poly_on_interval(P.db_newton_coefficients(M, N), 0.0, 1.0)
        X, Y = (1 - a) * X + a * X @ N, (1 - a) * Y + a * Y @ N
        M = 2 * a * (1 - a) * np.eye(n) + (1 - a) ** 2 * M + a * a * N
        assert np.linalg.norm(X @ Y - M) < 1e-11 * np.linalg.norm(M)


def test_unconstrained_global_minimiser_lies_in_the_unit_interval():
    """The reading [0, 1]: on spectra with more than one point the global minimiser over the whole
    real line (all real roots of m') is the one found on [0, 1]."""
    rng = _rng(7)
    for trial in range(50):
        n = int(rng.integers(2, 9))
        lam = np.exp(rng.uniform(-4, 4, n))
        lam[1] = lam[0] * (1.5 + rng.uniform())         # at least two distinct points
        M = np.diag(lam)
        c = P.db_newton_coefficients(M, np.diag(1.0 / lam))
        roots = np.roots((c[1:] * np.arange(1, 5))[::-1])
        real = [r.real for r in roots if abs(r.imag) < 1e-9 * max(1.0, abs(r.real))]
        best = min(real, key=lambda a: np.polyval(c[::-1], a))
        a = P.minimize_poly_on_interval(c, 0.0, 1.0)
        assert 0.0 < best < 1.0
        assert abs(a - best) < 1e-8


def test_one_point_spectrum_converges_in_one_step():
    """M = mu I: alpha = sqrt(mu) / (sqrt(mu) + 1) makes M_1 = I exactly, X_1 = sqrt(mu) I."""
    for mu in (0.04, 0.5, 9.0):
        X, Y, info = P.sqrt_db_newton(mu * np.eye(3), 5, 1e-12)
        assert info["iters"] == 1
        assert abs(info["alpha"][0] - np.sqrt(mu) / (np.sqrt(mu) + 1.0)) < 1e-9
        assert np.allclose(X, np.sqrt(mu) * np.eye(3), atol=1e-12)
        assert np.allclose(Y, np.eye(3) / np.sqrt(mu), atol=1e-12)


def test_fit_needs_fewer_iterations_than_classical():
    A, _ = _spd(np.logspace(-4, 3, 40), 9)
    _, _, fit = P.sqrt_db_newton(A, 100, 1e-10)
    _, _, classical = P.sqrt_db_newton(A, 100, 1e-10, fit=False)
    assert fit["status"] == classical["status"] == P.STATUS_CONVERGED
    assert fit["iters"] < classical["iters"]
    assert all(0.0 < a < 1.0 for a in fit["alpha"])
