"""Gaussian sketch matrices S_k for the PRISM fit (paper Section 4.2: the sketch
S_k in eq. (4) is a p_s x n matrix of i.i.d. Gaussian entries, a fresh one for
every iteration k).

TEST INFRASTRUCTURE ONLY - see the package docstring.

The paper fixes only the distribution.  To make the fitted coefficients
reproducible on any machine the entries are defined here by a counter-based
generator, so that entry (r, j) of S_k depends on nothing but
(seed, k, function tag, r, j):

  bits    Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers:
          as easy as 1, 2, 3", SC'11) with key (seed low word, seed high word)
          and counter (j, r // 4, k, tag).  The four output words x0..x3 give
          rows 4q..4q+3 of column j:  (x0, x1) -> rows 4q, 4q+1 and
          (x2, x3) -> rows 4q+2, 4q+3.
  normal  Box-Muller on a word pair (xa, xb):
            a = (xa >> 8) + 1   in [1, 2^24]      u1 = a * 2^-24  in (0, 1]
            b = (xb >> 8)       in [0, 2^24)      u2 = b * 2^-24  in [0, 1)
            z_first  = fl32( radius(a) * cos(2 pi u2) )
            z_second = fl32( radius(a) * sin(2 pi u2) )
          where radius(a) = sqrt(-2 ln u1) and the cos/sin pair are evaluated
          by the fixed sequences of IEEE binary64 operations written out in
          `radius` and `cos_sin` below (+, -, *, /, sqrt only, each rounded
          once, nothing fused), then the product is rounded to binary32.

Entries have unit variance; the 1/sqrt(p_s) scale of the paper is applied by
the caller (it does not change the minimiser of the fit).

Pins (tests/test_oracle_sketch.py): published Philox known-answer vectors;
radius/cos/sin against libm in fp64; moments and a Kolmogorov-Smirnov test of
the normal law; counter layout (changing k, tag, seed or position changes the
entry it should and no other).
"""
import numpy as np

_M0 = np.uint64(0xD2511F53)
_M1 = np.uint64(0xCD9E8D57)
_W0 = 0x9E3779B9
_W1 = 0xBB67AE85
_MASK = np.uint64(0xFFFFFFFF)
_SH32 = np.uint64(32)


def philox4x32_10(c0, c1, c2, c3, k0, k1):
    """Ten rounds of Philox-4x32.  Counter words are uint32 arrays (broadcast
    against each other), key words are Python ints.  Returns four uint32 arrays."""
    c0, c1, c2, c3 = np.broadcast_arrays(
        *[np.asarray(c, dtype=np.uint64) & _MASK for c in (c0, c1, c2, c3)])
    k0 = int(k0) & 0xFFFFFFFF
    k1 = int(k1) & 0xFFFFFFFF
    for _ in range(10):
        p0 = _M0 * c0                      # 32x32 -> 64 bit products, exact in uint64
        p1 = _M1 * c2
        hi0, lo0 = p0 >> _SH32, p0 & _MASK
        hi1, lo1 = p1 >> _SH32, p1 & _MASK
        c0, c1, c2, c3 = (hi1 ^ c1 ^ np.uint64(k0), lo1,
                          hi0 ^ c3 ^ np.uint64(k1), lo0)
        k0 = (k0 + _W0) & 0xFFFFFFFF       # key schedule: bumped after every round
        k1 = (k1 + _W1) & 0xFFFFFFFF
    return tuple(c.astype(np.uint32) for c in (c0, c1, c2, c3))


_SQRT2 = np.float64(1.4142135623730951)
_LN2 = np.float64(0.6931471805599453)
_PIO4 = np.float64(0.7853981633974483)
_ONE = np.float64(1.0)
_TWO = np.float64(2.0)


def radius(a):
    """sqrt(-2 ln(a * 2^-24)) for integer a in [1, 2^24], binary64 arrays.

    ln is split as (e - 24) ln 2 + ln m with a = m 2^e, m in [1/sqrt2, sqrt2);
    ln m = 2 atanh(s), s = (m-1)/(m+1), by the odd series through s^21."""
    a = np.asarray(a, dtype=np.int64)
    e = np.zeros(a.shape, dtype=np.int64)
    for sh in (16, 8, 4, 2, 1):            # e = floor(log2 a), integer only
        big = (a >> (e + sh)) > 0
        e = np.where(big, e + sh, e)
    m = np.ldexp(a.astype(np.float64), -e.astype(np.int32))   # exact, in [1, 2)
    up = m > _SQRT2
    m = np.where(up, m * np.float64(0.5), m)
    e = np.where(up, e + 1, e)
    f = m - _ONE                           # exact
    s = f / (_TWO + f)
    w = s * s
    p = _ONE / np.float64(21.0)
    for odd in (19.0, 17.0, 15.0, 13.0, 11.0, 9.0, 7.0, 5.0, 3.0, 1.0):
        p = p * w + _ONE / np.float64(odd)
    lnm = (_TWO * s) * p
    lnu = (e - 24).astype(np.float64) * _LN2 + lnm
    return np.sqrt(np.float64(0.0) - _TWO * lnu)


_COS_DEN = (1.0, 2.0, 24.0, 720.0, 40320.0, 3628800.0, 479001600.0,
            87178291200.0, 20922789888000.0)                      # (2k)!,   k = 0..8
_SIN_DEN = (1.0, 6.0, 120.0, 5040.0, 362880.0, 39916800.0, 6227020800.0,
            1307674368000.0, 355687428096000.0)                   # (2k+1)!, k = 0..8


def cos_sin(b):
    """(cos, sin) of 2 pi b 2^-24 for integer b in [0, 2^24), binary64 arrays.

    The top three bits of b select the octant; the remaining 21 bits give
    t in [0, 1) (odd octants use 1 - t), the reduced angle is x = t pi/4 and
    cos x, sin x are Taylor sums through x^16 and x^17."""
    b = np.asarray(b, dtype=np.int64)
    octant = b >> 21
    t = (b & 0x1FFFFF).astype(np.float64) * np.float64(2.0 ** -21)   # exact
    t = np.where(octant & 1, _ONE - t, t)                            # exact
    x = t * _PIO4
    y = x * x
    # Horner in y with coef_k = (-1)^k / (2k)!  (resp. / (2k+1)!), k = 8 down to 0
    c = _ONE / np.float64(_COS_DEN[8])                   # k = 8 is even: + sign
    s = _ONE / np.float64(_SIN_DEN[8])
    for k in range(7, -1, -1):
        ck = _ONE / np.float64(_COS_DEN[k])
        sk = _ONE / np.float64(_SIN_DEN[k])
        if k & 1:
            ck, sk = -ck, -sk
        c = c * y + ck
        s = s * y + sk
    s = s * x
    cos_t = np.select([octant == 0, octant == 1, octant == 2, octant == 3,
                       octant == 4, octant == 5, octant == 6], [c, s, -s, -c, -c, -s, s], c)
    sin_t = np.select([octant == 0, octant == 1, octant == 2, octant == 3,
                       octant == 4, octant == 5, octant == 6], [s, c, c, s, -s, -c, -c], -s)
    return cos_t, sin_t


def box_muller(xa, xb):
    """Two unit normals (binary32) from two uint32 words."""
    a = (np.asarray(xa, dtype=np.int64) >> 8) + 1
    b = np.asarray(xb, dtype=np.int64) >> 8
    r = radius(a)
    c, s = cos_sin(b)
    return (r * c).astype(np.float32), (r * s).astype(np.float32)


TAG_POLAR, TAG_SQRT, TAG_INV_ROOT, TAG_SIGN, TAG_INVERSE = 1, 2, 3, 4, 5


def sketch(seed, k, tag, p_s, n):
    """S_k as a (p_s, n) binary32 array of unit normals (see module docstring)."""
    seed = int(seed) & 0xFFFFFFFFFFFFFFFF
    groups = (p_s + 3) // 4
    j = np.arange(n, dtype=np.uint32)[None, :]
    q = np.arange(groups, dtype=np.uint32)[:, None]
    x0, x1, x2, x3 = philox4x32_10(j, q, np.uint32(k), np.uint32(tag),
                                   seed & 0xFFFFFFFF, seed >> 32)
    z0, z1 = box_muller(x0, x1)
    z2, z3 = box_muller(x2, x3)
    rows = np.stack([z0, z1, z2, z3], axis=1).reshape(4 * groups, n)
    return np.ascontiguousarray(rows[:p_s])
