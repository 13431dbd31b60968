"""Pins for the three readings of oracle/prism_ref.py that the paper leaves open (CPU only):
the fit interval of the coupled inverse Newton iteration (App. A.3 prints none), the tie rule of
the minimiser of m(alpha) (Section 4.2 says only "minimise"), and the stop rule with its
DIVERGED / BUDGET outcomes (the paper gives no stop rule).  Each test states the mistake it catches.
"""
import numpy as np
import pytest

from oracle import prism_ref as P


# ------------------------------------------------ inverse Newton interval [1/p, 2/p]

def _reachable_x(p, count=4001):
    # M_0 = A (p+1) / (2 ||A||_F) of an SPD A has its spectrum in (0, (p+1)/2], so the
    # eigenvalues x = 1 - mu of R_0 lie in [-(p-1)/2, 1)   (App. A.3, initialisation)
    return np.linspace(-(p - 1) / 2.0, 1.0, count, endpoint=False)


def _step_is_safe(p, alpha, x):
    """Scalar form of one update (App. A.3): mu' = (1 + alpha x)^p mu, x' = 1 - mu'.
    Safe = the factor stays positive (X_{k+1} stays definite) and the residual eigenvalue
    stays inside the unit disc, on every reachable x."""
    t = 1.0 + alpha * x
    nxt = 1.0 - (1.0 - x) * t ** p
    return bool(np.all(t > 0.0) and np.all(np.abs(nxt) < 1.0))


@pytest.mark.parametrize("p", [1, 2, 3, 4, 5, 6, 7, 8])
def test_inv_root_interval_is_safe_on_the_reachable_spectrum(p):
    """A wrong upper end (2/(p-1), 1, 4/p ...) or a lower end above 1/p fails here."""
    lo, hi = P.inv_root_interval(p)
    assert lo == pytest.approx(1.0 / p, rel=0, abs=1e-15)      # Taylor value: classical iteration at the lower end
    assert lo < hi
    x = _reachable_x(p)
    for alpha in np.linspace(lo, hi, 101):
        assert _step_is_safe(p, alpha, x), (p, alpha)
    # the scalar iteration started anywhere on the reachable spectrum converges to x = 0 (at the upper
    # end itself the map is only neutral at 0, slope 1 - p alpha = -1: the interval is closed there)
    for alpha in (lo, 0.5 * (lo + hi), lo + 0.95 * (hi - lo)):
        xs = x.copy()
        for _ in range(2000):
            xs = 1.0 - (1.0 - xs) * (1.0 + alpha * xs) ** p
        assert np.max(np.abs(xs)) < 1e-12, (p, alpha)


@pytest.mark.parametrize("p", [3, 4, 5, 7])
def test_the_safety_pin_rejects_plausible_wrong_upper_ends(p):
    """The check above has teeth: the upper ends one could misread into App. A.3 are unsafe."""
    x = _reachable_x(p)
    for wrong_u in (2.0 / (p - 1), 1.0, 4.0 / p):
        assert not _step_is_safe(p, wrong_u, x), (p, wrong_u)


def test_inv_root_interval_coincides_with_d1_interval_for_p2():
    """p = 2: the printed coefficient tables of App. A.3 equal those of d = 1 (App. A.1), whose
    interval the paper does print (Theorem 1): the two readings must agree there."""
    assert P.inv_root_interval(2) == P.clamp_interval(1)


def test_fitted_inverse_newton_alpha_stays_in_its_interval_and_reaches_both_ends():
    """On a power-law spectrum the fit starts at the upper end and ends at the lower one (the
    behaviour Fig. 3-4 show for the Newton-Schulz family): a transposed interval would clamp the
    other way round."""
    n, p = 48, 4
    lam = np.arange(1, n + 1) ** -1.5 + 1e-6
    q, _ = np.linalg.qr(np.random.default_rng(3).standard_normal((n, n)))
    A = (q * lam) @ q.T
    X, info = P.inv_root(A, p, 60, 8, 5, 1e-12)
    lo, hi = P.inv_root_interval(p)
    al = np.array(info["alpha"])
    assert info["status"] == P.STATUS_CONVERGED
    assert np.all(al >= lo - 1e-15) and np.all(al <= hi + 1e-15)
    assert al[0] == hi and abs(al[-1] - lo) < 1e-3
    w, v = np.linalg.eigh(A)
    assert np.linalg.norm(X - (v * w ** (-1.0 / p)) @ v.T) / np.linalg.norm((v * w ** (-1.0 / p)) @ v.T) < 1e-9


# ------------------------------------------------ tie rule of the minimiser

def test_minimiser_constant_polynomial_returns_the_lower_end():
    """m is flat: every candidate ties, the smallest alpha wins (a `<=` in the scan returns hi)."""
    assert P.minimize_poly_on_interval([5.0, 0.0, 0.0, 0.0, 0.0], 0.375, 1.45) == 0.375
    assert P.minimize_poly_on_interval([2.5], 0.5, 1.0) == 0.5


def test_minimiser_equal_values_at_both_ends_returns_the_lower_end():
    """m = -(alpha - 1/2)(alpha - 1): interior maximum, both ends evaluate to exactly 0."""
    c = [-0.5, 1.5, -1.0]
    assert np.polyval(c[::-1], 0.5) == 0.0 and np.polyval(c[::-1], 1.0) == 0.0
    assert P.minimize_poly_on_interval(c, 0.5, 1.0) == 0.5


def test_minimiser_two_equal_interior_minima_returns_the_smaller():
    """m = (alpha^2 - 1/4)^2 on [-1, 1]: minima at -1/2 and +1/2 with the same value (m is even,
    so the two evaluations agree bit for bit), a maximum at 0 between them."""
    c = [1.0 / 16.0, 0.0, -0.5, 0.0, 1.0]
    a = P.minimize_poly_on_interval(c, -1.0, 1.0)
    assert a == pytest.approx(-0.5, abs=1e-12)
    # and the rule is about ties only: tilt the polynomial and the lower minimum wins wherever it is
    assert P.minimize_poly_on_interval([1.0 / 16.0, -1e-3, -0.5, 0.0, 1.0], -1.0, 1.0) == pytest.approx(0.5, abs=2e-3)
    assert P.minimize_poly_on_interval([1.0 / 16.0, +1e-3, -0.5, 0.0, 1.0], -1.0, 1.0) == pytest.approx(-0.5, abs=2e-3)


# ------------------------------------------------ stop rule: CONVERGED / BUDGET / DIVERGED

def _run_loop(residuals, max_iters, tol, n=4):
    """Feeds a residual history to the oracle's stop logic through matrices of that norm."""
    loop = P._Loop(n, max_iters, tol)
    for k, r in enumerate(residuals):
        R = np.diag(np.full(n, float(r)))            # ||r I||_F / sqrt(n) = |r|
        if loop.stop(R, k):
            return k, loop.status
        loop.alpha.append(0.0)
    return None, loop.status


def test_stop_rule_diverged_needs_two_rises_in_a_row_above_the_start():
    # rises twice in a row but stays below r_0: not diverged; the next rise passes r_0: diverged at that k
    k, st = _run_loop([1.0, 0.5, 0.6, 0.7, 1.1, 2.0], 20, 1e-3)
    assert (k, st) == (4, P.STATUS_DIVERGED)
    # one rise above r_0 followed by a fall is not divergence; it ends on the budget
    k, st = _run_loop([1.0, 1.5, 1.2, 1.3, 1.25, 1.24, 1.23], 6, 1e-3)
    assert (k, st) == (6, P.STATUS_BUDGET)
    # two rises above r_0 from the very start: the earliest k at which the rule can fire is 2
    k, st = _run_loop([1.0, 1.1, 1.2, 1.3], 20, 1e-3)
    assert (k, st) == (2, P.STATUS_DIVERGED)
    # non-finite residual: diverged at once
    k, st = _run_loop([1.0, float("inf")], 20, 1e-3)
    assert (k, st) == (1, P.STATUS_DIVERGED)
    k, st = _run_loop([float("nan")], 20, 1e-3)
    assert (k, st) == (0, P.STATUS_DIVERGED)


def test_stop_rule_budget_and_converged_are_exact():
    k, st = _run_loop([0.9] * 10, 7, 1e-3)                     # stalled: budget, at k = max_iters exactly
    assert (k, st) == (7, P.STATUS_BUDGET)
    k, st = _run_loop([0.9, 0.1, 1e-3], 7, 1e-3)               # res == tol counts as converged
    assert (k, st) == (2, P.STATUS_CONVERGED)
    k, st = _run_loop([0.9, 0.1, 1.0000001e-3, 1e-4], 7, 1e-3)
    assert (k, st) == (3, P.STATUS_CONVERGED)
    # convergence is tested before the budget: the residual of the last permitted evaluation may still converge
    k, st = _run_loop([0.9, 0.5, 1e-4], 2, 1e-3)
    assert (k, st) == (2, P.STATUS_CONVERGED)
    # fixed budget (tol <= 0): never converged, never diverged, exactly max_iters updates
    k, st = _run_loop([1.0, 2.0, 3.0, 4.0, 5.0], 4, 0.0)
    assert (k, st) == (4, P.STATUS_BUDGET)


def test_polar_driver_reports_diverged_exactly_when_the_rule_fires():
    """A coefficient schedule far above the interval blows the iteration up: status is DIVERGED
    (not BUDGET) and `iters` is the first k at which the residual has risen twice above r_0."""
    A = np.random.default_rng(9).standard_normal((24, 12))
    X, info = P.polar(A, 3, 30, 0, 1, 1e-8, alpha_schedule=[6.0] * 30)
    r = info["residual"]
    assert info["status"] == P.STATUS_DIVERGED
    first = next(k for k in range(2, len(r)) if not np.isfinite(r[k]) or (r[k] > r[k - 1] > r[k - 2] and r[k] > r[0]))
    assert info["iters"] == first == len(r) - 1 and len(info["alpha"]) == first


def test_polar_driver_reports_budget_exactly_on_a_stalled_iteration():
    """alpha = 0 with d = 1 makes the update the identity: the residual never moves, the call ends
    with exactly max_iters updates and BUDGET (a divergence rule with `>=` would fire here)."""
    A = np.random.default_rng(10).standard_normal((24, 12))
    X, info = P.polar(A, 3, 9, 0, 1, 1e-8, alpha_schedule=[-0.0] * 9)
    # g_1(R; 0) = I: X never changes
    assert info["status"] == P.STATUS_BUDGET and info["iters"] == 9
    assert len(info["residual"]) == 10 and len(set(info["residual"])) == 1
    assert np.array_equal(X, A / np.linalg.norm(A))
