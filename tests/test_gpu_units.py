"""Unit parity of single kernels against numpy / the oracle (GPU)."""
import numpy as np
import pytest
import torch

from oracle import gauss_sketch as gs
from paper_2601_22137_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def prism():
    from paper_2601_22137_amd import prism as P
    P.lib()
    return P


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


@pytest.mark.parametrize("a_km", [False, True])
@pytest.mark.parametrize("shape", [(128, 128, 64), (256, 128, 80), (128, 16, 128), (128, 32, 256), (256, 64, 128), (64, 64, 48)])
def test_gemm_f32(prism, a_km, shape):
    M, N, K = shape
    rng = np.random.default_rng(M + N + K)
    A = rng.standard_normal((3, M, K)).astype(np.float32)
    B = rng.standard_normal((3, K, N)).astype(np.float32)
    Ain = np.ascontiguousarray(A.transpose(0, 2, 1)) if a_km else A
    C = prism.gemm_f32(_dev(Ain), _dev(B), a_km=a_km).cpu().numpy()
    ref = A.astype(np.float64) @ B.astype(np.float64)
    assert np.linalg.norm(C - ref) / np.linalg.norm(ref) < 1e-6


@pytest.mark.parametrize("n,ld,batch", [(64, 16, 2), (192, 32, 2), (768, 16, 2), (1024, 32, 2), (4096, 32, 2),
                                        (1024, 16, 16), (2048, 32, 8), (1152, 32, 15), (768, 16, 12), (1088, 32, 16), (2048, 64, 2),
                                        # one and two chunks of 256 k (shorter than the kernel's ring), 128-row workgroups
                                        # with a ragged number of ring rounds
                                        (256, 16, 40), (512, 32, 20), (1280, 32, 13), (256, 32, 70)])
def test_chain_product_bf16(prism, n, ld, batch):
    """Off-diagonal entries from the bf16 copy, diagonal from the fp32 matrix; R = I - small, the
    case in which a rounded diagonal would be wrong by more than the whole off-diagonal part.
    Small batches take the 16-row kernel, (n / 64) * batch >= 128 the 64-row one (chunks of 256 k,
    with and without a ragged last ring round; V and the result also as bf16 planes); the widest sketch (ld = 64) and large batches of sizes
    that are no multiple of 256 are not taken (the library keeps to the fp32 matrix there)."""
    rng = np.random.default_rng(3 * n + ld)
    R = np.empty((batch, n, n), dtype=np.float32)
    for b in range(batch):
        g = rng.standard_normal((n, n)) / n
        R[b] = (np.eye(n) - 0.5 * (g + g.T)).astype(np.float32)
    V = rng.standard_normal((batch, n, ld)).astype(np.float32)
    Rb = W.to_bf16_bits(R)
    rb_dev = torch.from_numpy(Rb.view(np.int16)).cuda()
    small = ld <= 32 and (n // 64) * batch < 128
    if ld == 64 or (not small and n % 256):
        with pytest.raises(prism.PrismError, match="UNSUPPORTED"):
            prism.chain_product_bf16(rb_dev, _dev(R), _dev(V))
        return
    out, planes = prism.chain_product_bf16(rb_dev, _dev(R), _dev(V), return_planes=True)
    out = out.cpu().numpy()
    if not small:
        # the launch read V as three bf16 planes and wrote its result that way too: each is the exact
        # 8 + 8 + 8 bit split of the fp32 array, laid out [matrix][k / 256][plane][column][unit'][8 k] with
        # unit' = (unit & 16) | ((unit ^ column) & 15)
        pl = planes.cpu().numpy().view(np.uint16).reshape(2, batch, n // 256, 3, ld, 32, 8)
        unit = np.arange(32)[None, :]
        stored = (unit & 16) | ((unit ^ np.arange(ld)[:, None]) & 15)                # [column][unit] -> stored unit
        pl = np.take_along_axis(pl, stored[None, None, None, None, :, :, None], axis=5).reshape(2, batch, n // 256, 3, ld, 256)
        for which, arr in ((0, V), (1, out)):
            parts = W.from_bf16_bits(pl[which]).astype(np.float64)              # [batch][c][plane][col][k]
            total = parts.sum(axis=2).transpose(0, 1, 3, 2).reshape(batch, n, ld)
            assert np.array_equal(total.astype(np.float32), arr), which
            # pieces are truncations: each carries at most 8 significant bits of what the ones before left
            hi = parts[:, :, 0].transpose(0, 1, 3, 2).reshape(batch, n, ld)
            assert np.array_equal(hi.astype(np.float32).view(np.uint32), arr.view(np.uint32) & 0xFFFF0000), which
    idx = np.arange(n)
    for b in (0, batch - 1):
        exact = R[b].astype(np.float64) @ V[b].astype(np.float64)
        Rq = W.from_bf16_bits(Rb[b]).astype(np.float64)
        Rq[idx, idx] = R[b][idx, idx]
        ref = Rq @ V[b].astype(np.float64)
        assert np.linalg.norm(out[b] - ref) / np.linalg.norm(ref) < 2e-7 * np.sqrt(n)
        # the rounded off-diagonal part moves the product by far less than a rounded diagonal would
        assert np.linalg.norm(Rq @ V[b] - exact) / np.linalg.norm(exact) < 1e-3


@pytest.mark.parametrize("a_km", [False, True])
@pytest.mark.parametrize("n,K", [(128, 64), (384, 208), (64, 48)])
def test_gemm_f32_symmetric(prism, a_km, n, K):
    """A A^T (or A^T A) through the variant that computes the upper triangle of tiles only."""
    rng = np.random.default_rng(n + K)
    A = rng.standard_normal((3, n, K)).astype(np.float32)
    At = np.ascontiguousarray(A.transpose(0, 2, 1))
    C = prism.gemm_f32(_dev(At if a_km else A), _dev(At), a_km=a_km, sym=True).cpu().numpy()
    ref = A.astype(np.float64) @ At.astype(np.float64)
    assert np.linalg.norm(C - ref) / np.linalg.norm(ref) < 1e-6
    full = prism.gemm_f32(_dev(At if a_km else A), _dev(At), a_km=a_km).cpu().numpy()
    iu = np.triu_indices(n)
    assert np.array_equal(C[:, iu[0], iu[1]], full[:, iu[0], iu[1]])      # the computed half is unchanged
    assert np.array_equal(C, C.transpose(0, 2, 1))


@pytest.mark.parametrize("n,ld", [(64, 16), (192, 32), (768, 16), (1024, 64), (4096, 32)])
def test_chain_product(prism, n, ld):
    rng = np.random.default_rng(n + ld)
    R = (rng.standard_normal((2, n, n)) / np.sqrt(n)).astype(np.float32)
    V = rng.standard_normal((2, n, ld)).astype(np.float32)
    out = prism.chain_product(_dev(R), _dev(V)).cpu().numpy()
    ref = R.astype(np.float64) @ V.astype(np.float64)
    err = np.linalg.norm(out - ref) / np.linalg.norm(ref)
    assert err < 2e-7 * np.sqrt(n), err       # fp32 accumulation over n terms


def test_gemm_f64a(prism):
    rng = np.random.default_rng(7)
    A = rng.standard_normal((2, 128, 96)).astype(np.float32)
    B = rng.standard_normal((2, 96, 192))
    C = prism.gemm_f64a(_dev(A), _dev(B)).cpu().numpy()
    ref = A.astype(np.float64) @ B
    assert np.linalg.norm(C - ref) / np.linalg.norm(ref) < 1e-14


@pytest.mark.parametrize("tile,shape", [(128, (128, 256, 192)), (256, (512, 256, 128)), (128, (384, 128, 64)),
                                        # operands beyond half the Infinity Cache and a multiple of 256 tiles:
                                        # the tile order in which every XCD sweeps 4 x 8 blocks of its own
                                        (128, (2048, 2048, 8448)), (256, (1024, 16384, 2048))])
def test_gemm_bf16_nt(prism, tile, shape):
    M, N, K = shape
    rng = np.random.default_rng(M * 3 + N)
    A = W.to_bf16_bits(rng.standard_normal((2, M, K)))
    B = W.to_bf16_bits(rng.standard_normal((2, N, K)))
    C = prism.gemm_bf16_nt(_dev(A.view(np.int16)), _dev(B.view(np.int16)), tile).cpu().numpy()
    ref = W.from_bf16_bits(A).astype(np.float64) @ W.from_bf16_bits(B).astype(np.float64).transpose(0, 2, 1)
    assert np.linalg.norm(C - ref) / np.linalg.norm(ref) < 1e-6


@pytest.mark.parametrize("km", [2, 3])
@pytest.mark.parametrize("tile,shape", [(128, (128, 256, 192)), (128, (384, 128, 64)), (2561, (512, 384, 320)),
                                        (256, (512, 256, 128)), (2561, (2048, 2048, 4160)), (256, (1024, 4096, 2048))])
def test_gemm_bf16_operands_stored_k_major(prism, tile, shape, km):
    """The same product with B (km = 2) or both operands (km = 3) stored with K as the slow index,
    which the kernel reads from LDS with transposing reads."""
    M, N, K = shape
    rng = np.random.default_rng(M * 3 + N + km)
    A = W.to_bf16_bits(rng.standard_normal((2, M, K)))
    B = W.to_bf16_bits(rng.standard_normal((2, N, K)))
    ref = W.from_bf16_bits(A).astype(np.float64) @ W.from_bf16_bits(B).astype(np.float64).transpose(0, 2, 1)
    As = np.ascontiguousarray(A.transpose(0, 2, 1)) if km == 3 else A
    Bs = np.ascontiguousarray(B.transpose(0, 2, 1))
    C = prism.gemm_bf16_nt(_dev(As.view(np.int16)), _dev(Bs.view(np.int16)), tile, km).cpu().numpy()
    assert np.linalg.norm(C - ref) / np.linalg.norm(ref) < 1e-6


def test_gemm_bf16_256x128_tiles(prism):
    M, N, K = 768, 640, 448
    rng = np.random.default_rng(5)
    A = W.to_bf16_bits(rng.standard_normal((3, M, K)))
    B = W.to_bf16_bits(rng.standard_normal((3, N, K)))
    C = prism.gemm_bf16_nt(_dev(A.view(np.int16)), _dev(B.view(np.int16)), 2561).cpu().numpy()
    ref = W.from_bf16_bits(A).astype(np.float64) @ W.from_bf16_bits(B).astype(np.float64).transpose(0, 2, 1)
    assert np.linalg.norm(C - ref) / np.linalg.norm(ref) < 1e-6


@pytest.mark.parametrize("n,p_s,k,fn,seed", [(300, 8, 0, 1, 22137), (1000, 16, 3, 2, 5), (257, 6, 7, 3, 2 ** 40 + 17),
                                             (4096, 32, 11, 1, 22137), (512, 64, 1, 2, 2 ** 63 + 5)])
def test_sketch_bit_exact(prism, n, p_s, k, fn, seed):
    got = prism.sketch(n, p_s, seed, k, fn).cpu().numpy()
    want = gs.sketch(seed, k, fn, p_s, n).T
    assert got.dtype == np.float32
    assert np.array_equal(got.view(np.uint32), np.ascontiguousarray(want).view(np.uint32))


def test_box_muller_factors_exhaustive_bit_exact(prism):
    """All 2^24 radii and all 2^24 angles: the device arithmetic equals the oracle's bit for bit."""
    step = 1 << 22
    for first in range(0, 1 << 24, step):
        r, c, s = prism.gauss_parts(first, step)
        v = np.arange(first, first + step, dtype=np.int64)
        wr = gs.radius(v + 1)
        wc, ws = gs.cos_sin(v)
        assert np.array_equal(r.cpu().numpy().view(np.uint64), wr.view(np.uint64)), first
        assert np.array_equal(c.cpu().numpy().view(np.uint64), np.ascontiguousarray(wc).view(np.uint64)), first
        assert np.array_equal(s.cpu().numpy().view(np.uint64), np.ascontiguousarray(ws).view(np.uint64)), first
