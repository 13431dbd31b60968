"""Pins for the matrix sign and Chebyshev inverse iterations of oracle/prism_ref.py (CPU only).

Each test names what it would catch.  No expected value comes from the HIP path.
"""
import os

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


def _general(n, cond, seed):
    r = _rng(seed)
    u, _ = np.linalg.qr(r.standard_normal((n, n)))
    v, _ = np.linalg.qr(r.standard_normal((n, n)))
    return (u * np.logspace(0, -np.log10(cond), n)) @ v.T


# ------------------------------------------------------------------ limits

@pytest.mark.parametrize("degree", [3, 5])
def test_sign_limit_symmetric_indefinite(degree):
    """sign(A) = Q sign(lambda) Q^T; a wrong residual (I - X^T X written as I + X^2, a sign slip)
    or a wrong Taylor coefficient does not reach it."""
    lam = np.concatenate([np.linspace(0.05, 1.0, 9), -np.linspace(0.02, 0.7, 7)])
    A = _sym_with_eigs(lam, 3)
    X, info = P.sign(A, degree, 60, 8, 5, 1e-13)
    w, q = np.linalg.eigh(A)
    assert info["status"] == P.STATUS_CONVERGED
    assert np.linalg.norm(X - (q * np.sign(w)) @ q.T) < 1e-10
    assert np.linalg.norm(X @ X - np.eye(16)) < 1e-10          # involutory
    assert np.linalg.norm(X @ A - A @ X) < 1e-10               # commutes with A


@pytest.mark.parametrize("degree", [3, 5])
def test_sign_of_block_matrix_gives_both_square_roots(degree):
    """sign([[0, A], [I, 0]]) = [[0, A^{1/2}], [A^{-1/2}, 0]] (Section 5, before Theorem 3): a
    non-symmetric input whose square is symmetric.  Catches a transposed product in the residual."""
    n = 7
    A = _sym_with_eigs(np.linspace(0.3, 2.0, n), 8)
    B = np.block([[np.zeros((n, n)), A], [np.eye(n), np.zeros((n, n))]])
    X, info = P.sign(B, degree, 60, 6, 5, 1e-13)
    w, q = np.linalg.eigh(A)
    assert info["status"] == P.STATUS_CONVERGED
    assert np.linalg.norm(X[:n, n:] - (q * np.sqrt(w)) @ q.T) < 1e-10
    assert np.linalg.norm(X[n:, :n] - (q / np.sqrt(w)) @ q.T) < 1e-10
    assert np.linalg.norm(X[:n, :n]) < 1e-10 and np.linalg.norm(X[n:, n:]) < 1e-10


def test_inverse_limit_is_numpy_inverse():
    """Non-symmetric A: X_0 = A (not A^T), or R = I - X A with the wrong apply side, diverges or
    lands elsewhere."""
    A = _general(14, 30.0, 5) * 3.7
    X, info = P.inverse(A, 80, 8, 3, 1e-13)
    assert info["status"] == P.STATUS_CONVERGED
    assert np.linalg.norm(X - np.linalg.inv(A)) < 1e-9 * np.linalg.norm(np.linalg.inv(A))
    assert np.linalg.norm(A @ X - np.eye(14)) < 1e-10


# ------------------------------------------------- special case: classical iterations

def test_sign_without_fit_is_classical_newton_schulz():
    A = _sym_with_eigs(np.concatenate([np.linspace(0.2, 1, 5), -np.linspace(0.3, 0.9, 4)]), 2)
    for degree, steps in ((3, 8), (5, 5)):
        X, info = P.sign(A, degree, steps, 0, 1, 0.0)
        Z = A / np.linalg.norm(A)
        for _ in range(steps):
            Z2 = Z @ Z
            Z = 1.5 * Z - 0.5 * Z @ Z2 if degree == 3 else 15 / 8 * Z - 10 / 8 * Z @ Z2 + 3 / 8 * Z @ Z2 @ Z2
        assert info["iters"] == steps and info["status"] == P.STATUS_BUDGET
        assert np.linalg.norm(X - Z) < 1e-12


def test_inverse_without_fit_is_classical_chebyshev():
    """X_{k+1} = 3 X - 3 X A X + X A X A X (App. A.4)."""
    A = _general(9, 5.0, 4)
    X, info = P.inverse(A, 6, 0, 1, 0.0)
    s = np.linalg.norm(A)
    As = A / s
    Z = As.T.copy()
    for _ in range(6):
        Z = 3 * Z - 3 * Z @ As @ Z + Z @ As @ Z @ As @ Z
    assert info["alpha"] == [1.0] * 6
    assert np.linalg.norm(X - Z / s) < 1e-12 * np.linalg.norm(Z / s)


# --------------------------------------------------------------- Theorem 1, invariants

def test_theorem1_bound_for_sign_exact_fit_d1():
    """||I - X_k^2||_2 <= ||I - A^2||_2^(2^(k-2)) for d = 1, exact fit on [1/2, 1] (Theorem 1),
    on an indefinite input."""
    lam = np.concatenate([np.logspace(-5, 0, 20), -np.logspace(-4, -0.1, 12)])
    A = _sym_with_eigs(lam, 21)
    A = A / np.linalg.norm(A, 2)
    X, info = P.sign(A, 3, 60, 0, 1, 1e-13, exact_fit=True)
    Z = A / np.linalg.norm(A)
    r0 = np.linalg.norm(np.eye(32) - Z @ Z, 2)
    for k, alpha in enumerate(info["alpha"]):
        R = np.eye(32) - Z @ Z
        assert np.linalg.norm(R, 2) <= r0 ** (2.0 ** (k - 2)) + 1e-12
        assert 0.5 <= alpha <= 1.0
        Z = Z @ (np.eye(32) + alpha * R)
    assert info["status"] == P.STATUS_CONVERGED


def test_inverse_exact_fit_beats_every_other_alpha_and_classical():
    """With S = I the fitted alpha gives the smallest next residual over [1/2, 2] (definition of
    the fit), in particular no larger than the classical alpha = 1; fewer iterations overall."""
    A = _general(12, 200.0, 9)
    s = np.linalg.norm(A)
    As = A / s
    X = As.T.copy()
    for _ in range(3):
        G = As @ X
        R = np.eye(12) - G
        a = P.fit_alpha_cheb(R, G, np.eye(12))

        def nxt(al):
            return np.linalg.norm(np.eye(12) - As @ X @ (np.eye(12) + R + al * R @ R))
        for other in np.linspace(0.5, 2.0, 31):
            assert nxt(a) <= nxt(other) + 1e-12
        X = X @ (np.eye(12) + R + a * R @ R)
    _, fit = P.inverse(A, 200, 12, 3, 1e-10)
    _, classical = P.inverse(A, 200, 0, 3, 1e-10)
    assert fit["status"] == classical["status"] == P.STATUS_CONVERGED
    assert fit["iters"] < classical["iters"]


# ------------------------------------------------------------------ closed forms, tables

def test_chebyshev_one_point_spectrum_closed_form():
    """R = lambda I: m(alpha) = n lambda^4 (1 - alpha (1 - lambda))^2, so alpha = 1 / (1 - lambda)
    clamped to [1/2, 2], and the next residual lambda^2 (1 - alpha (1 - lambda)) vanishes when
    the clamp is inactive."""
    n = 5
    for lam, want in ((0.25, 4.0 / 3.0), (0.4, 1.0 / 0.6), (0.8, 2.0), (-1.5, 0.5), (-0.25, 0.8)):
        R = lam * np.eye(n)
        a = P.fit_alpha_cheb(R, np.eye(n) - R, np.eye(n))
        assert abs(a - want) < 1e-12
    # driver level: A = c I gives R_0 = (1 - 1/n) I; for n = 2, alpha_0 = 2 exactly and R_1 = 0
    X, info = P.inverse(3.0 * np.eye(2), 5, 0, 1, 1e-12, exact_fit=True)
    assert abs(info["alpha"][0] - 2.0) < 1e-14 and info["iters"] == 1
    assert np.allclose(X, np.eye(2) / 3.0, atol=1e-14)


def test_chebyshev_coefficients_match_printed_traces():
    tabs = {}
    for l in open(os.path.join(GOLDEN, "printed_m_alpha_tables.txt")):
        if l.startswith("cheb"):
            head, body = l.split(":")
            tabs[int(head.split()[1])] = [(float(t.split("*t")[0]), int(t.split("*t")[1])) for t in body.split()]
    n = 11
    R = _sym_with_eigs(_rng(3).uniform(-0.3, 0.9, n), 4)
    S = gs.sketch(6, 2, gs.TAG_INVERSE, 4, n).astype(np.float64)
    t, Rp = [], np.eye(n)
    for _ in range(7):
        t.append(np.trace(S @ Rp @ S.T))
        Rp = Rp @ R
    c = P.fit_coefficients_cheb(R, np.eye(n) - R, S.T)
    assert set(tabs) == {1, 2}
    for idx, terms in tabs.items():
        printed = sum(coef * t[i] for coef, i in terms)
        assert abs(c[idx] - printed) < 1e-10 * max(1.0, abs(printed))
    assert abs(c[0] - t[4]) < 1e-10


def test_chebyshev_quadratic_equals_literal_next_residual():
    """m(alpha) = || S (I - A X (I + R + alpha R^2)) ||_F^2 written out on an actual iterate."""
    A = _general(8, 10.0, 6)
    As = A / np.linalg.norm(A)
    X = As.T
    G = As @ X
    R = np.eye(8) - G
    S = gs.sketch(1, 0, gs.TAG_INVERSE, 3, 8).astype(np.float64)
    c = P.fit_coefficients_cheb(R, G, S.T)
    for a in np.linspace(0.2, 2.2, 6):
        literal = np.linalg.norm(S @ (np.eye(8) - As @ X @ (np.eye(8) + R + a * R @ R))) ** 2
        assert abs(np.polyval(c[::-1], a) - literal) < 1e-12 * max(1.0, literal)


def test_sign_uses_its_own_sketch_stream_and_schedule():
    """Function tag 4 (sign) and 5 (inverse) select sketch streams of their own; a schedule
    overrides the fit for its leading iterations only."""
    A = _sym_with_eigs(np.concatenate([np.logspace(-3, 0, 12), -np.logspace(-2, -0.2, 8)]), 13)
    _, a = P.sign(A, 5, 6, 4, 77, 0.0)
    St = gs.sketch(77, 0, gs.TAG_SIGN, 4, 20).astype(np.float64).T / 2.0
    X = A / np.linalg.norm(A)
    G = X @ X
    assert abs(a["alpha"][0] - P.fit_alpha_ns(np.eye(20) - G, G, St, 2)) < 1e-14
    _, b = P.sign(A, 5, 6, 4, 77, 0.0, alpha_schedule=[1.45, 1.0])
    assert b["alpha"][:2] == [1.45, 1.0] and len(b["alpha"]) == 6
    _, c = P.inverse(A, 6, 4, 77, 0.0, alpha_schedule=[2.0])
    assert c["alpha"][0] == 2.0 and 0.5 <= min(c["alpha"][1:]) and max(c["alpha"][1:]) <= 2.0
