"""Pins for oracle/gauss_sketch.py (CPU only)."""
import os

import numpy as np
import pytest
from scipy import stats

from oracle import gauss_sketch as gs

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_philox_known_answers():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for row in rows:
        v = [int(x, 16) for x in row]
        out = gs.philox4x32_10(v[0], v[1], v[2], v[3], v[4], v[5])
        assert [int(o) for o in out] == v[6:]


def test_philox_vectorised_matches_scalar():
    rng = np.random.default_rng(0)
    c = rng.integers(0, 2 ** 32, size=(4, 50), dtype=np.uint64).astype(np.uint32)
    vec = gs.philox4x32_10(c[0], c[1], c[2], c[3], 0x12345678, 0x9ABCDEF0)
    for i in range(50):
        one = gs.philox4x32_10(c[0, i], c[1, i], c[2, i], c[3, i], 0x12345678, 0x9ABCDEF0)
        assert [int(o) for o in one] == [int(v[i]) for v in vec]


def test_radius_against_libm():
    a = np.unique(np.concatenate([np.arange(1, 5000), np.arange(2 ** 24 - 5000, 2 ** 24 + 1),
                                  np.random.default_rng(1).integers(1, 2 ** 24, size=200000),
                                  2 ** np.arange(0, 25)]))
    ref = np.sqrt(-2.0 * np.log(a * 2.0 ** -24))
    got = gs.radius(a)
    assert got[-1] == 0.0 and a[-1] == 2 ** 24
    # relative error of r is that of ln u1 halved; ln u1 -> 0 at the top end, so test absolute there
    assert np.max(np.abs(got - ref)) < 4e-15 * np.max(ref)
    assert np.max(np.abs(got[:-1] - ref[:-1]) / ref[:-1]) < 2e-12
    assert abs(got[0] - np.sqrt(48 * np.log(2.0))) < 1e-14      # u1 = 2^-24


def test_cos_sin_against_libm():
    b = np.unique(np.concatenate([np.arange(0, 4096), np.arange(2 ** 24 - 4096, 2 ** 24),
                                  np.arange(0, 2 ** 24, 2 ** 21),          # octant boundaries
                                  np.arange(0, 2 ** 24, 2 ** 21) - 1 + (np.arange(8) == 0),
                                  np.random.default_rng(2).integers(0, 2 ** 24, size=200000)]))
    theta = 2.0 * np.pi * b * 2.0 ** -24
    c, s = gs.cos_sin(b)
    assert np.max(np.abs(c - np.cos(theta))) < 2e-15
    assert np.max(np.abs(s - np.sin(theta))) < 2e-15
    assert np.max(np.abs(c * c + s * s - 1.0)) < 1e-15
    # exact values at the axes
    c, s = gs.cos_sin(np.array([0, 2 ** 22, 2 ** 23, 3 * 2 ** 22]))
    assert list(c) == [1.0, 0.0, -1.0, 0.0] or np.allclose(c, [1, 0, -1, 0], atol=1e-16)
    assert np.allclose(s, [0, 1, 0, -1], atol=1e-16)


def test_normal_law():
    S = gs.sketch(22137, 0, gs.TAG_POLAR, 64, 8192).astype(np.float64).ravel()
    n = S.size
    assert abs(S.mean()) < 4.0 / np.sqrt(n)
    assert abs(S.var() - 1.0) < 4.0 * np.sqrt(2.0 / n)
    assert abs((S ** 4).mean() - 3.0) < 4.0 * np.sqrt(96.0 / n)
    assert abs((S ** 3).mean()) < 4.0 * np.sqrt(15.0 / n)
    assert stats.kstest(S, "norm").pvalue > 1e-3
    # rows and columns uncorrelated
    M = gs.sketch(5, 3, gs.TAG_SQRT, 16, 4096).astype(np.float64)
    C = M @ M.T / 4096
    assert np.max(np.abs(C - np.eye(16))) < 5.0 / np.sqrt(4096)


def test_counter_layout():
    base = gs.sketch(22137, 2, gs.TAG_POLAR, 16, 200)
    # entry (r, j) does not depend on the sketch dimension or on n
    assert np.array_equal(gs.sketch(22137, 2, gs.TAG_POLAR, 8, 100), base[:8, :100])
    assert np.array_equal(gs.sketch(22137, 2, gs.TAG_POLAR, 6, 100), base[:6, :100])
    # iteration, tag and both seed words all enter
    for other in (gs.sketch(22137, 3, gs.TAG_POLAR, 16, 200), gs.sketch(22137, 2, gs.TAG_SQRT, 16, 200),
                  gs.sketch(22138, 2, gs.TAG_POLAR, 16, 200), gs.sketch(22137 + 2 ** 32, 2, gs.TAG_POLAR, 16, 200)):
        assert not np.any(other == base)
    # rows 4q..4q+3 of column j come from one Philox call with counter (j, q, k, tag)
    j, q = 37, 2
    x = gs.philox4x32_10(j, q, 2, gs.TAG_POLAR, 22137, 0)
    z0, z1 = gs.box_muller(x[0], x[1])
    z2, z3 = gs.box_muller(x[2], x[3])
    assert [float(z0), float(z1), float(z2), float(z3)] == [float(v) for v in base[8:12, j]]
    assert base.dtype == np.float32


def test_box_muller_definition():
    # z = sqrt(-2 ln u1) (cos, sin)(2 pi u2) with u1 = ((xa >> 8) + 1) 2^-24, u2 = (xb >> 8) 2^-24
    xa = np.array([0, 0xFFFFFFFF, 0x80000000, 12345 << 8], dtype=np.uint32)
    xb = np.array([0, 0x40000000, 0xC0000000, 0x12345678], dtype=np.uint32)
    z0, z1 = gs.box_muller(xa, xb)
    u1 = ((xa.astype(np.int64) >> 8) + 1) * 2.0 ** -24
    u2 = (xb.astype(np.int64) >> 8) * 2.0 ** -24
    r = np.sqrt(-2 * np.log(u1))
    assert np.allclose(z0, r * np.cos(2 * np.pi * u2), rtol=1e-6, atol=1e-7)
    assert np.allclose(z1, r * np.sin(2 * np.pi * u2), rtol=1e-6, atol=1e-7)
