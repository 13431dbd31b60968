"""Seeded synthetic inputs shaped like the paper's workloads (Section 6: Gaussian /
Marchenko-Pastur and heavy-tailed spectra; Muon on GPT-2-like gradients; Shampoo
preconditioners up to a few thousand wide).  They stand in for the paper's data,
which is not reproduced here.

This module holds none of the method's arithmetic: it only draws matrices with
numpy's PCG64 and rounds them to the storage type.  Both the HIP path and the
CPU oracle are fed from here so that they see the same bits.
"""
import numpy as np

SKETCH_SEED = 22137


# ------------------------------------------------------------------ bf16 helpers

def to_bf16_bits(x):
    """Round float array to bfloat16 (nearest even); returns the uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def from_bf16_bits(b):
    """uint16 bfloat16 bit patterns -> float32 (exact)."""
    return (np.asarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


def _orthogonal(rng, n):
    q, r = np.linalg.qr(rng.standard_normal((n, n)))
    return q * np.sign(np.diag(r))[None, :]


# ---------------------------------------------------------------------- configs

def c1_polar_small(m=64, n=32, data_seed=1001):
    """One fp32 matrix, N(0,1) entries, columns scaled by log-uniform factors in
    [1e-3, 1] (condition number about 1e3)."""
    rng = _rng(data_seed)
    z = rng.standard_normal((m, n))
    v = rng.uniform(np.log(1e-3), 0.0, size=n)
    return (z * np.exp(v)[None, :]).astype(np.float32)[None]


C2_SHAPES = ((768, 768), (768, 3072), (3072, 768), (768, 2304))


def c2_muon_group(shape_idx, batch=16, scale=1, data_seed=1002):
    """One shape group of the Muon-like batch: bf16, N(0,1) entries times a
    log-normal(0,1) per-row scale, Frobenius-normalised.  `scale` divides both
    dimensions (reduced-size parity cases).  Returns uint16 bf16 bits [batch, m, n]."""
    m, n = C2_SHAPES[shape_idx]
    m, n = m // scale, n // scale
    rng = _rng(data_seed + shape_idx)
    out = np.empty((batch, m, n), dtype=np.uint16)
    for b in range(batch):
        z = rng.standard_normal((m, n))
        w = rng.standard_normal(m)
        a = z * np.exp(w)[:, None]
        out[b] = to_bf16_bits(a / np.linalg.norm(a))
    return out


def c3_polar_large(n=4096, batch=8, data_seed=1003, sigma_decades=4.0):
    """bf16 square matrices U diag(sigma) V^T with Haar U, V and log-uniform
    singular values in [10^-sigma_decades, 1].  Returns uint16 bf16 bits [batch, n, n]."""
    out = np.empty((batch, n, n), dtype=np.uint16)
    for b in range(batch):
        rng = _rng(data_seed + b)
        u = _orthogonal(rng, n)
        v = _orthogonal(rng, n)
        sigma = 10.0 ** rng.uniform(-sigma_decades, 0.0, size=n)
        out[b] = to_bf16_bits((u * sigma[None, :]) @ v.T)
    return out


def c4_shampoo_spd(n=1024, batch=32, data_seed=1004):
    """fp32 SPD matrices Q diag(i^-1.5 + 1e-6) Q^T (condition number about 1e5)."""
    lam = np.arange(1, n + 1, dtype=np.float64) ** -1.5 + 1e-6
    out = np.empty((batch, n, n), dtype=np.float32)
    for b in range(batch):
        q = _orthogonal(_rng(data_seed + b), n)
        a = (q * lam[None, :]) @ q.T
        out[b] = (0.5 * (a + a.T)).astype(np.float32)
    return out


def c5_wishart_spd(n=8192, batch=4, data_seed=1005, ratio=2, ridge=1e-4):
    """fp32 SPD matrices W W^T / k + ridge I with Gaussian W (n x k, k = ratio n):
    Marchenko-Pastur spectrum."""
    k = ratio * n
    out = np.empty((batch, n, n), dtype=np.float32)
    for b in range(batch):
        w = _rng(data_seed + b).standard_normal((n, k)).astype(np.float32)
        a = (w @ w.T).astype(np.float64) / k
        a[np.diag_indices(n)] += ridge
        out[b] = a.astype(np.float32)
    return out


def sign_indefinite(n=512, batch=4, data_seed=1006, decades=3.0):
    """fp32 symmetric indefinite matrices Q diag(lambda) Q^T: |lambda| log-uniform in
    [10^-decades, 1], random signs.  Stands in for the paper's matrix-sign experiments
    (Gaussian and heavy-tailed spectra); the sign function is sign-pattern of lambda."""
    out = np.empty((batch, n, n), dtype=np.float32)
    for b in range(batch):
        rng = _rng(data_seed + b)
        q = _orthogonal(rng, n)
        lam = 10.0 ** rng.uniform(-decades, 0.0, size=n) * rng.choice([-1.0, 1.0], size=n)
        a = (q * lam[None, :]) @ q.T
        out[b] = (0.5 * (a + a.T)).astype(np.float32)
    return out


def sign_block(n_half=192, batch=2, data_seed=1007):
    """fp32 [[0, A], [I, 0]] with A symmetric positive definite (eigenvalues log-uniform in
    [1e-2, 1]): not symmetric, but its square is; sign gives A^(1/2) and A^(-1/2) in the
    off-diagonal blocks (the route from matrix sign to square roots, Section 5)."""
    n = n_half
    out = np.zeros((batch, 2 * n, 2 * n), dtype=np.float32)
    for b in range(batch):
        rng = _rng(data_seed + b)
        q = _orthogonal(rng, n)
        lam = 10.0 ** rng.uniform(-2.0, 0.0, size=n)
        a = (q * lam[None, :]) @ q.T
        out[b, :n, n:] = (0.5 * (a + a.T)).astype(np.float32)
        out[b, n:, :n] = np.eye(n, dtype=np.float32)
    return out


def inverse_general(n=512, batch=4, data_seed=1008, cond=30.0):
    """fp32 non-symmetric full-rank matrices U diag(sigma) V^T times a per-matrix scale, sigma
    log-uniform in [1/cond, 1]."""
    out = np.empty((batch, n, n), dtype=np.float32)
    for b in range(batch):
        rng = _rng(data_seed + b)
        u = _orthogonal(rng, n)
        v = _orthogonal(rng, n)
        sigma = np.exp(rng.uniform(-np.log(cond), 0.0, size=n))
        out[b] = ((u * sigma[None, :]) @ v.T * (1.0 + 2.0 * b)).astype(np.float32)
    return out


def spd_conditioned(n=384, batch=2, cond=1e4, data_seed=1009):
    """fp32 symmetric positive definite Q diag(lambda) Q^T, lambda log-uniform in [1/cond, 1]:
    ill-conditioned inputs for the square-root iterations (the paper's Shampoo preconditioners
    reach such condition numbers before the ridge is added)."""
    out = np.empty((batch, n, n), dtype=np.float32)
    for b in range(batch):
        rng = _rng(data_seed + b)
        q = _orthogonal(rng, n)
        lam = np.exp(rng.uniform(-np.log(cond), 0.0, size=n))
        a = (q * lam[None, :]) @ q.T
        out[b] = (0.5 * (a + a.T)).astype(np.float32)
    return out


def sign_nonnormal(n=256, batch=2, data_seed=1010, decades=1.5, skew=0.3):
    """fp32 S diag(lambda) S^-1 with S = I + skew * G / sqrt(n), G Gaussian: diagonalisable with
    real eigenvalues of both signs (|lambda| log-uniform in [10^-decades, 1]) but neither
    symmetric nor normal, and neither is its square."""
    out = np.empty((batch, n, n), dtype=np.float32)
    for b in range(batch):
        rng = _rng(data_seed + b)
        s = np.eye(n) + skew * rng.standard_normal((n, n)) / np.sqrt(n)
        lam = 10.0 ** rng.uniform(-decades, 0.0, size=n) * rng.choice([-1.0, 1.0], size=n)
        out[b] = np.linalg.solve(s.T, (s * lam[None, :]).T).T.astype(np.float32)
    return out
