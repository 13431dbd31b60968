"""PRISM-accelerated Newton-Schulz-like iterations in plain fp64 numpy.

TEST INFRASTRUCTURE ONLY - see the package docstring.  Written from the paper
(Sections 3-5, Table 1, Appendix A.1 and A.3), step by step, in its notation:

  d      order of the update polynomial in the residual (degree 3 <-> d = 1,
         degree 5 <-> d = 2: the "3rd-order" and "5th-order" rows of Table 1)
  R_k    residual matrix, G_k = I - R_k
  g_d    g_d(xi; alpha) = f_{d-1}(xi) + alpha xi^d, f = Taylor polynomial of
         (1 - xi)^(-1/2)                                   (meta-algorithm, step 4)
  alpha  fitted per iteration by the sketched least-squares problem of eq. (4),
         constrained to [l, u]

Inputs are promoted to fp64 and every operation is fp64.  There is no blocking
or fusion: each line is one matrix operation of the paper.

Readings of the paper taken here (the paper is silent or garbled):
  * classical d = 1 step is 3/2 X - 1/2 X^3 (the printed "1/2 X - 3/2 X^3" in
    Section 3 contradicts x(1 + (1 - x^2)/2) two paragraphs later);
  * Appendix A.1 "R_k = I - X_k, g_d(X_k; alpha)" is read as eq. (1)-(2):
    R_k = I - X_k^2, g_d(R_k; alpha); "[l,u] = [1, 1/2]" is read as [1/2, 1];
  * the objective for polar / sqrt is eq. (4) with X_k^2 replaced by I - R_k
    (= X_k^T X_k resp. X_k Y_k), as the text after each display says;
  * the coupled square-root iteration: Table 1 and App. A.1 print R_k = I - X_k Y_k,
    Theorem 3 prints h(Y_k X_k).  The two agree in exact arithmetic (X_k and Y_k
    are polynomials in A), but only X_{k+1} = X_k g(I - Y_k X_k),
    Y_{k+1} = g(I - Y_k X_k) Y_k is stable in floating point; with X_k Y_k the
    residual grows again by a constant factor per step once it has reached
    rounding level.  Theorem 3's order is taken;
  * sketch entries are centred (mean 0, variance 1/p_s);
  * the interval for the coupled inverse Newton fit is not given; [1/p, 2/p] is
    used (lower end = Taylor value, upper end by analogy with p = 2 where the
    printed coefficient formulas coincide with d = 1 and [1/2, 1] = [1/p, 2/p]).
    The paper prints no value to pin it to; the tests pin it to the mathematics: on the
    spectrum reachable from M_0 every alpha in it keeps 1 + alpha x > 0 and contracts the
    residual eigenvalue, which the other plausible upper ends do not;
  * the stop rule is not given: the residual ||R_k||_F / sqrt(n) is tested
    before each update, `iters` counts updates;
  * when m'(alpha) = 0 has several roots the global minimiser over
    {l, u} U {roots in [l, u]} is taken, ties to the smallest alpha (own rule; pinned
    in the tests on polynomials with exactly equal minima);
  * m < n for the polar factor: run on the transpose (the paper assumes m >= n);
  * the same S_k serves all matrices of a call;
  * Chebyshev inverse (App. A.4): the input is normalised by its Frobenius norm as the
    text says, A_s = A / ||A||_F, X_0 = A_s^T, and the result is un-scaled at the end;
    without a fit alpha_k is the Taylor value 1 (the classical iteration), which
    is not the lower end of the printed interval [1/2, 2]; the objective is taken
    with R_k symmetric (it is, for X_0 = A_s^T: R_k is a polynomial in A A^T), so
    ||S h(R)||_F = ||h(R) S^T||_F and the chain again multiplies from the left;
  * DB Newton (App. A.2, product form): X_0 = M_0 = A and Y_0 = I as printed (no
    normalisation); the residual of the stop rule is I - M_k (Table 1: I - X_k Y_k);
    alpha_k minimises the printed quartic over [0, 1].  The paper imposes no interval;
    every eigenvalue mu of M_k contributes a term whose two zeros are
    sqrt(mu)/(sqrt(mu)+1), inside (0, 1), and sqrt(mu)/(sqrt(mu)-1), outside [0, 1],
    where (1-alpha) + alpha/mu < 0 and X_{k+1} loses definiteness; the zeros outside
    scatter over the real line, those inside cluster, so the unconstrained global
    minimiser lies in (0, 1) whenever the spectrum has more than one point (pinned
    on random spectra) and the interval only breaks the exact tie of a one-point
    spectrum; without a fit alpha_k = 1/2, the classical iteration.
"""
from math import comb

import numpy as np

from . import gauss_sketch

STATUS_CONVERGED, STATUS_BUDGET, STATUS_NONFINITE, STATUS_ZERO, STATUS_DIVERGED = 0, 1, 2, 3, 4

# Taylor coefficients of (1 - xi)^(-1/2): a_j = C(2j, j) / 4^j   (Section 3)
TAYLOR = tuple(comb(2 * j, j) / 4.0 ** j for j in range(4))


def clamp_interval(d):
    """[l, u] of eq. (3)-(4): [1/2, 1] for d = 1 (Theorem 1), [3/8, 29/20] for d = 2."""
    return {1: (0.5, 1.0), 2: (0.375, 1.45)}[d]


def inv_root_interval(p):
    """Reading for the coupled inverse Newton fit (see module docstring)."""
    return (1.0 / p, 2.0 / p)


def g_poly(R, d, alpha):
    """g_d(R; alpha) = f_{d-1}(R) + alpha R^d as a dense matrix."""
    n = R.shape[0]
    out = np.eye(n)
    Rj = np.eye(n)
    for j in range(1, d):
        Rj = Rj @ R
        out = out + TAYLOR[j] * Rj
    Rj = Rj @ R
    return out + alpha * Rj


# --------------------------------------------------------------------------- fit

def minimize_poly_on_interval(c, lo, hi):
    """argmin over [lo, hi] of m(alpha) = sum_s c[s] alpha^s  (Section 4.2, App. A.3):
    evaluate m at the end points and at the roots of m'; smallest alpha wins ties.
    Real parts of all roots of m' that fall in the interval are candidates
    (a non-critical extra candidate can never beat the true minimiser)."""
    c = np.asarray(c, dtype=np.float64)
    if not np.all(np.isfinite(c)) or np.all(np.abs(c) < 1e-300):
        return lo
    dc = c[1:] * np.arange(1, len(c))
    cands = [lo, hi]
    dc_trim = np.trim_zeros(dc[::-1], 'f')          # highest power first, leading zeros removed
    if len(dc_trim) > 1:
        for r in np.roots(dc_trim):
            if lo <= r.real <= hi:
                cands.append(float(r.real))
    cands.sort()
    vals = [np.polyval(c[::-1], a) for a in cands]
    best = 0
    for i in range(1, len(cands)):
        if vals[i] < vals[best]:
            best = i
    return cands[best]


def fit_coefficients_ns(R, G, St, d):
    """Coefficients c_0..c_4 of the quartic m(alpha) of eq. (4),
        m(alpha) = || (I - G g_d(R; alpha)^2) S^T ||_F^2,    G = I - R,
    for symmetric R (S h(R) and h(R) S^T then have the same norm).
    With h = 1 - (1 - xi) g_d^2 = u0 + alpha u1 + alpha^2 u2:
        d = 1:  u0 = xi,              u1 = -2 (1-xi) xi,        u2 = -(1-xi) xi^2
        d = 2:  u0 = xi^2 (3+xi)/4,   u1 = -(1-xi)(2+xi) xi^2,  u2 = -(1-xi) xi^4
    the three blocks W_i = u_i(R) S^T are built from the chain V_j = R V_{j-1},
    V_0 = S^T (App. A.1: products taken from the right), with the factor (1 - xi)
    applied as a product by G.  St is S^T, n x p_s."""
    V = [St]
    for _ in range(2 * d):
        V.append(R @ V[-1])
    if d == 1:
        W0 = V[1]
        W1 = -2.0 * (G @ V[1])
        W2 = -(G @ V[2])
    elif d == 2:
        W0 = (3.0 * V[2] + V[3]) / 4.0
        W1 = -(G @ (2.0 * V[2] + V[3]))
        W2 = -(G @ V[4])
    else:
        raise ValueError("d must be 1 or 2")
    W = (W0, W1, W2)
    c = np.zeros(5)
    for i in range(3):
        for l in range(3):
            c[i + l] += np.sum(W[i] * W[l])
    return c


def fit_alpha_ns(R, G, St, d):
    lo, hi = clamp_interval(d)
    return minimize_poly_on_interval(fit_coefficients_ns(R, G, St, d), lo, hi)


def fit_coefficients_inv(R, M, St, p):
    """Coefficients c_0..c_{2p} of (App. A.3)
        m(alpha) = || (R + sum_{i=1..p} C(p,i) alpha^i (R^{i+1} - R^i)) S^T ||_F^2 .
    Since M = I - R,  R^{i+1} - R^i = -M R^i:  W_0 = R S^T, W_i = -C(p,i) M R^i S^T."""
    V = [St]
    for _ in range(p):
        V.append(R @ V[-1])
    W = [V[1]] + [-comb(p, i) * (M @ V[i]) for i in range(1, p + 1)]
    c = np.zeros(2 * p + 1)
    for i in range(p + 1):
        for l in range(p + 1):
            c[i + l] += np.sum(W[i] * W[l])
    return c


def fit_alpha_inv(R, M, St, p):
    lo, hi = inv_root_interval(p)
    return minimize_poly_on_interval(fit_coefficients_inv(R, M, St, p), lo, hi)


def fit_coefficients_cheb(R, G, St):
    """Coefficients c_0, c_1, c_2 of the quadratic (App. A.4)
        m(alpha) = || (R^2 - alpha (R^2 - R^3)) S^T ||_F^2,
    R symmetric, G = I - R = A X:  W_0 = R^2 S^T,  W_1 = -(R^2 - R^3) S^T = -G R^2 S^T."""
    V1 = R @ St
    V2 = R @ V1
    W0 = V2
    W1 = -(G @ V2)
    return np.array([np.sum(W0 * W0), 2.0 * np.sum(W0 * W1), np.sum(W1 * W1)])


CHEB_INTERVAL = (0.5, 2.0)      # App. A.4


def fit_alpha_cheb(R, G, St):
    return minimize_poly_on_interval(fit_coefficients_cheb(R, G, St), *CHEB_INTERVAL)


def _sketch_T(seed, k, tag, p_s, n, exact_fit):
    """S_k^T (n x p_s) with variance-1/p_s entries; exact_fit replaces S by the
    identity, which turns eq. (4) into eq. (3)."""
    if exact_fit:
        return np.eye(n)
    S = gauss_sketch.sketch(seed, k, tag, p_s, n).astype(np.float64) / np.sqrt(p_s)
    return np.ascontiguousarray(S.T)


# ----------------------------------------------------------------------- drivers

class _Loop:
    """Shared stop logic: test before each update; `iters` = updates done."""

    def __init__(self, n, max_iters, tol):
        self.sqrt_n = np.sqrt(n)
        self.max_iters = max_iters
        self.tol = tol
        self.residual = []
        self.alpha = []
        self.status = None

    def stop(self, R, k):
        res = np.linalg.norm(R, 'fro') / self.sqrt_n
        self.residual.append(float(res))
        r = self.residual
        if not np.isfinite(res):
            self.status = STATUS_DIVERGED
        elif self.tol > 0 and res <= self.tol:
            self.status = STATUS_CONVERGED
        elif k == self.max_iters:
            self.status = STATUS_BUDGET
        elif self.tol > 0 and k >= 2 and r[k] > r[k - 1] > r[k - 2] and r[k] > r[0]:
            self.status = STATUS_DIVERGED
        return self.status is not None

    def info(self):
        return {"iters": len(self.alpha), "status": self.status,
                "residual": list(self.residual), "alpha": list(self.alpha)}


def _precheck(A):
    if not np.all(np.isfinite(A)):
        return STATUS_NONFINITE
    if not np.any(A):
        return STATUS_ZERO
    return None


def _early(A, status):
    return {"iters": 0, "status": status, "residual": [], "alpha": []}


def polar(A, degree=5, max_iters=30, sketch_dim=8, seed=22137, tol=1e-6,
          exact_fit=False, alpha_schedule=None):
    """Polar factor U V^T of A (m x n) by the PRISM Newton-Schulz iteration
    (Table 1, rows "Newton-Schulz (3rd/5th-order), U V^T"; App. A.1):
        X_0 = A / ||A||_F,  R_k = I - X_k^T X_k,  X_{k+1} = X_k g_d(R_k; alpha_k).
    sketch_dim = 0 keeps alpha_k at the Taylor value l (classical Newton-Schulz);
    alpha_schedule (a list) overrides the fit for its leading iterations.
    Returns (X, info)."""
    A = np.asarray(A, dtype=np.float64)
    bad = _precheck(A)
    if bad is not None:
        return A.copy(), _early(A, bad)
    if A.shape[0] < A.shape[1]:
        X, info = polar(A.T, degree, max_iters, sketch_dim, seed, tol, exact_fit, alpha_schedule)
        return np.ascontiguousarray(X.T), info
    d = {3: 1, 5: 2}[degree]
    n = A.shape[1]
    X = A / np.linalg.norm(A, 'fro')
    loop = _Loop(n, max_iters, tol)
    k = 0
    while True:
        G = X.T @ X
        R = np.eye(n) - G
        if loop.stop(R, k):
            break
        if alpha_schedule is not None and k < len(alpha_schedule):
            alpha = float(alpha_schedule[k])
        elif sketch_dim == 0 and not exact_fit:
            alpha = clamp_interval(d)[0]
        else:
            St = _sketch_T(seed, k, gauss_sketch.TAG_POLAR, sketch_dim, n, exact_fit)
            alpha = fit_alpha_ns(R, G, St, d)
        loop.alpha.append(alpha)
        X = X @ g_poly(R, d, alpha)
        k += 1
    return X, loop.info()


def sqrt(A, degree=5, max_iters=30, sketch_dim=8, seed=22137, tol=1e-6,
         exact_fit=False, alpha_schedule=None):
    """A^{1/2} and A^{-1/2} of a symmetric positive definite A by the coupled
    PRISM Newton-Schulz iteration (Table 1, rows "A^{1/2}, A^{-1/2}"; Theorem 3;
    App. A.1):  X_0 = A / s, Y_0 = I (s = ||A||_F), R_k = I - Y_k X_k,
        X_{k+1} = X_k g_d(R_k; alpha_k),   Y_{k+1} = g_d(R_k; alpha_k) Y_k,
    and A^{1/2} = sqrt(s) X, A^{-1/2} = Y / sqrt(s).  The residual takes the
    product in the order of Theorem 3 (see the module docstring).
    Returns (root, inv_root, info)."""
    A = np.asarray(A, dtype=np.float64)
    bad = _precheck(A)
    if bad is not None:
        return A.copy(), np.zeros_like(A), _early(A, bad)
    d = {3: 1, 5: 2}[degree]
    n = A.shape[0]
    s = np.linalg.norm(A, 'fro')
    X = A / s
    Y = np.eye(n)
    loop = _Loop(n, max_iters, tol)
    k = 0
    while True:
        G = Y @ X
        R = np.eye(n) - G
        if loop.stop(R, k):
            break
        if alpha_schedule is not None and k < len(alpha_schedule):
            alpha = float(alpha_schedule[k])
        elif sketch_dim == 0 and not exact_fit:
            alpha = clamp_interval(d)[0]
        else:
            St = _sketch_T(seed, k, gauss_sketch.TAG_SQRT, sketch_dim, n, exact_fit)
            alpha = fit_alpha_ns(R, G, St, d)
        loop.alpha.append(alpha)
        P = g_poly(R, d, alpha)
        X = X @ P
        Y = P @ Y
        k += 1
    return np.sqrt(s) * X, Y / np.sqrt(s), loop.info()


def inv_root(A, p, max_iters=30, sketch_dim=8, seed=22137, tol=1e-6,
             exact_fit=False, alpha_schedule=None):
    """A^{-1/p} of a symmetric positive definite A by the PRISM coupled inverse
    Newton iteration (Table 1, row "Coupled Inverse Newton"; App. A.3):
        c = (2 ||A||_F / (p+1))^{1/p},  X_0 = I / c,  M_0 = A / c^p,
        R_k = I - M_k,  X_{k+1} = X_k (I + alpha_k R_k),
        M_{k+1} = (I + alpha_k R_k)^p M_k.
    Returns (X, info)."""
    A = np.asarray(A, dtype=np.float64)
    bad = _precheck(A)
    if bad is not None:
        return A.copy(), _early(A, bad)
    n = A.shape[0]
    cp = 2.0 * np.linalg.norm(A, 'fro') / (p + 1)          # c^p
    X = np.eye(n) / cp ** (1.0 / p)
    M = A / cp
    loop = _Loop(n, max_iters, tol)
    k = 0
    while True:
        R = np.eye(n) - M
        if loop.stop(R, k):
            break
        if alpha_schedule is not None and k < len(alpha_schedule):
            alpha = float(alpha_schedule[k])
        elif sketch_dim == 0 and not exact_fit:
            alpha = inv_root_interval(p)[0]
        else:
            St = _sketch_T(seed, k, gauss_sketch.TAG_INV_ROOT, sketch_dim, n, exact_fit)
            alpha = fit_alpha_inv(R, M, St, p)
        loop.alpha.append(alpha)
        T = np.eye(n) + alpha * R
        X = X @ T
        M = np.linalg.matrix_power(T, p) @ M
        k += 1
    return X, loop.info()


def sign(A, degree=5, max_iters=30, sketch_dim=8, seed=22137, tol=1e-6,
         exact_fit=False, alpha_schedule=None):
    """sign(A) = A (A^2)^{-1/2} of a square A with A^2 symmetric, by the PRISM
    Newton-Schulz iteration of Section 4, eq. (2)-(4):
        X_0 = A / ||A||_F,  R_k = I - X_k^2,  X_{k+1} = X_k g_d(R_k; alpha_k).
    Returns (X, info)."""
    A = np.asarray(A, dtype=np.float64)
    bad = _precheck(A)
    if bad is not None:
        return A.copy(), _early(A, bad)
    d = {3: 1, 5: 2}[degree]
    n = A.shape[0]
    X = A / np.linalg.norm(A, 'fro')
    loop = _Loop(n, max_iters, tol)
    k = 0
    while True:
        G = X @ X
        R = np.eye(n) - G
        if loop.stop(R, k):
            break
        if alpha_schedule is not None and k < len(alpha_schedule):
            alpha = float(alpha_schedule[k])
        elif sketch_dim == 0 and not exact_fit:
            alpha = clamp_interval(d)[0]
        else:
            St = _sketch_T(seed, k, gauss_sketch.TAG_SIGN, sketch_dim, n, exact_fit)
            alpha = fit_alpha_ns(R, G, St, d)
        loop.alpha.append(alpha)
        X = X @ g_poly(R, d, alpha)
        k += 1
    return X, loop.info()


def inverse(A, max_iters=30, sketch_dim=8, seed=22137, tol=1e-6,
            exact_fit=False, alpha_schedule=None):
    """A^{-1} of a full-rank square A by the PRISM Chebyshev iteration
    (Table 1, row "Chebyshev"; App. A.4):  A_s = A / s (s = ||A||_F),
        X_0 = A_s^T,  R_k = I - A_s X_k,  X_{k+1} = X_k (I + R_k + alpha_k R_k^2),
    and A^{-1} = X / s.  Returns (X / s, info)."""
    A = np.asarray(A, dtype=np.float64)
    bad = _precheck(A)
    if bad is not None:
        return A.copy(), _early(A, bad)
    n = A.shape[0]
    s = np.linalg.norm(A, 'fro')
    As = A / s
    X = As.T.copy()
    loop = _Loop(n, max_iters, tol)
    k = 0
    while True:
        G = As @ X
        R = np.eye(n) - G
        if loop.stop(R, k):
            break
        if alpha_schedule is not None and k < len(alpha_schedule):
            alpha = float(alpha_schedule[k])
        elif sketch_dim == 0 and not exact_fit:
            alpha = 1.0
        else:
            St = _sketch_T(seed, k, gauss_sketch.TAG_INVERSE, sketch_dim, n, exact_fit)
            alpha = fit_alpha_cheb(R, G, St)
        loop.alpha.append(alpha)
        R2 = R @ R
        X = X @ (np.eye(n) + R + alpha * R2)
        k += 1
    return X / s, loop.info()


def db_newton_coefficients(M, N):
    """Coefficients c_0..c_4 of m(alpha) = ||I - M_{k+1}(alpha)||_F^2 for the product form of
    DB Newton (App. A.2), M_{k+1} = 2 alpha (1 - alpha) I + (1 - alpha)^2 M + alpha^2 N, N = M^{-1}:
        M_{k+1} - I = (1 - 2 alpha) D_0 + alpha^2 D_2,   D_0 = M - I,   D_2 = M + N - 2 I,
    so c_0 = <D_0,D_0>, c_1 = -4 <D_0,D_0>, c_2 = 4 <D_0,D_0> + 2 <D_0,D_2>, c_3 = -4 <D_0,D_2>,
    c_4 = <D_2,D_2> (Frobenius inner products: O(n^2), no matrix product).  Expanding the inner
    products gives the printed combinations of n, tr M, tr M^2, tr M^-1, tr M^-2 (pinned in the
    tests); those subtract nearly equal numbers once M is close to I and stall the iteration at
    a residual of about sqrt(machine epsilon), this form does not."""
    n = M.shape[0]
    D0 = M - np.eye(n)
    D2 = M + N - 2.0 * np.eye(n)
    g00, g02, g22 = np.sum(D0 * D0), np.sum(D0 * D2), np.sum(D2 * D2)
    return np.array([g00, -4.0 * g00, 4.0 * g00 + 2.0 * g02, -4.0 * g02, g22])


DB_NEWTON_INTERVAL = (0.0, 1.0)     # reading, see the module docstring


def sqrt_db_newton(A, max_iters=30, tol=1e-6, fit=True, alpha_schedule=None):
    """A^{1/2} and A^{-1/2} of a symmetric positive definite A by the PRISM-accelerated DB Newton
    iteration in product form (Table 1, row "DB Newton"; App. A.2):
        M_0 = X_0 = A, Y_0 = I, N_k = M_k^{-1},
        M_{k+1} = 2 a (1 - a) I + (1 - a)^2 M_k + a^2 N_k,
        X_{k+1} = (1 - a) X_k + a X_k N_k,   Y_{k+1} = (1 - a) Y_k + a Y_k N_k,   a = alpha_k,
    alpha_k = argmin ||I - M_{k+1}||_F^2 (exact traces, no sketch).  fit = False keeps
    alpha_k = 1/2.  Returns (X, Y, info)."""
    A = np.asarray(A, dtype=np.float64)
    bad = _precheck(A)
    if bad is not None:
        return A.copy(), np.zeros_like(A), _early(A, bad)
    n = A.shape[0]
    I = np.eye(n)
    X, Y, M = A.copy(), I.copy(), A.copy()
    loop = _Loop(n, max_iters, tol)
    k = 0
    while True:
        if loop.stop(I - M, k):
            break
        N = np.linalg.inv(M)
        if alpha_schedule is not None and k < len(alpha_schedule):
            a = float(alpha_schedule[k])
        elif not fit:
            a = 0.5
        else:
            a = minimize_poly_on_interval(db_newton_coefficients(M, N), *DB_NEWTON_INTERVAL)
        loop.alpha.append(a)
        X = (1.0 - a) * X + a * (X @ N)
        Y = (1.0 - a) * Y + a * (Y @ N)
        M = 2.0 * a * (1.0 - a) * I + (1.0 - a) ** 2 * M + a * a * N
        k += 1
    return X, Y, loop.info()
