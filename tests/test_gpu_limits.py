"""The documented size limits: the largest batch and a matrix close to the largest extent.  At these
sizes the oracle runs on a few matrices only; the rest is checked through what must hold at any size
(all matrices of a call share S_k, so equal inputs give bit-identical outputs wherever they sit in the
batch; the polar factor of a full-rank A is A (A^T A)^(-1/2))."""
import numpy as np
import pytest
import torch

from oracle import prism_ref as O
from paper_2601_22137_amd import workloads as W

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(600)]

SEED = W.SKETCH_SEED
MAX_BATCH = 65535
DISTINCT, COPIES = 255, 257          # 255 * 257 = 65535


@pytest.fixture(scope="module")
def prism():
    from paper_2601_22137_amd import prism as P
    P.lib()
    return P


def _rel(x, ref):
    return np.linalg.norm(np.asarray(x, dtype=np.float64) - ref) / np.linalg.norm(ref)


def _replicated(base):
    assert base.shape[0] == DISTINCT
    return base.repeat(COPIES, 1, 1).contiguous()


def _all_copies_equal(x):
    v = x.view(COPIES, DISTINCT, *x.shape[1:])
    if v.dtype == torch.bfloat16:
        v = v.view(torch.int16)
    return bool((v == v[0:1]).all())


def test_largest_batch_polar_fp32(prism):
    A = np.concatenate([W.c1_polar_small(data_seed=5000 + i) for i in range(DISTINCT)])      # 64 x 32 each
    x = _replicated(torch.from_numpy(A).cuda())
    assert x.shape[0] == MAX_BATCH
    info = prism.polar(x, 5, 30, 8, SEED, 1e-6).read()
    assert _all_copies_equal(x)
    it = info["iters"].reshape(COPIES, DISTINCT)
    assert np.all(it == it[0]) and np.all(info["status"] == prism.INFO_CONVERGED)
    out = x[:DISTINCT].cpu().numpy()
    for i in (0, 127, DISTINCT - 1):
        ref, oinfo = O.polar(A[i], 5, 30, 8, SEED, 1e-6)
        assert _rel(out[i], ref) <= 1e-5
        assert info[i]["iters"] == oinfo["iters"]
    last = x[-1].cpu().numpy()
    assert np.array_equal(last, out[DISTINCT - 1])


def test_largest_batch_polar_bf16(prism):
    A = np.concatenate([W.c1_polar_small(m=128, n=64, data_seed=5300 + i) for i in range(DISTINCT)])
    bits = W.to_bf16_bits(A)
    x = _replicated(torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16))
    info = prism.polar(x, 5, 5, 16, SEED, 0.0, flags=prism.FLAG_BF16_PLAIN_ITERATE).read()
    assert _all_copies_equal(x)
    assert np.all(info["iters"] == 5)
    out = W.from_bf16_bits(x[:DISTINCT].view(torch.int16).cpu().numpy().view(np.uint16))
    for i in (0, 200):
        ref, _ = O.polar(W.from_bf16_bits(bits[i]), 5, 5, 16, SEED, 0.0)
        assert _rel(out[i], ref) <= 2e-2


def test_largest_batch_inverse_root(prism):
    n = 64
    A = W.spd_conditioned(n, DISTINCT, 1e2, data_seed=5600)
    x = _replicated(torch.from_numpy(A).cuda())
    info = prism.inv_root(x, 2, 40, 8, SEED, 1e-5).read()
    assert _all_copies_equal(x)
    assert np.all(info["status"] == prism.INFO_CONVERGED)
    out = x[:DISTINCT].cpu().numpy()
    for i in (0, DISTINCT - 1):
        ref, oinfo = O.inv_root(A[i].astype(np.float64), 2, 40, 8, SEED, 1e-5)
        assert _rel(out[i], ref) <= 1e-5
        assert info[i]["iters"] == oinfo["iters"]


def test_batch_beyond_the_limit_is_refused(prism):
    x = torch.zeros((MAX_BATCH + 1, 8, 8), device="cuda")
    with pytest.raises(prism.PrismError):
        prism.polar(x, 5, 5, 8, SEED, 1e-6)
    assert not x.any()


def test_matrix_near_the_largest_extent(prism):
    """fp32 polar factor of one 4,190,000 x 500 matrix (2.095e9 entries, 2.145e9 with its sides
    rounded up to multiples of 128; the limit is 2^31 - 1 = 2.147e9).  Reference: A (A^T A)^(-1/2)
    with the Gram matrix accumulated in fp64 and its inverse square root by eigendecomposition."""
    m, n, chunk = 4_190_000, 500, 1 << 18
    gen = torch.Generator(device="cuda")
    gen.manual_seed(5900)
    a = torch.randn((1, m, n), device="cuda", generator=gen)
    scale = torch.exp(torch.linspace(np.log(1e-2), 0.0, n, device="cuda"))       # kappa ~ 1e2
    a *= scale
    gram = torch.zeros((n, n), dtype=torch.float64, device="cuda")
    for r0 in range(0, m, chunk):
        blk = a[0, r0:r0 + chunk].double()
        gram += blk.T @ blk
    lam, vec = np.linalg.eigh(gram.cpu().numpy())
    assert lam[0] > 0
    w = torch.from_numpy((vec / np.sqrt(lam)) @ vec.T).cuda()
    x = a.clone()
    info = prism.polar(x, 5, 30, 8, SEED, 1e-6).read()
    assert info[0]["status"] == prism.INFO_CONVERGED and 1 <= info[0]["iters"] <= 20
    err2 = ref2 = 0.0
    for r0 in range(0, m, chunk):
        ref = a[0, r0:r0 + chunk].double() @ w
        err2 += float(((x[0, r0:r0 + chunk].double() - ref) ** 2).sum())
        ref2 += float((ref ** 2).sum())
    assert np.sqrt(err2 / ref2) <= 1e-5
    assert abs(ref2 - n) <= 1e-6 * n            # the reference itself has orthonormal columns
    with pytest.raises(prism.PrismError):       # one tile row more crosses the limit
        prism.workspace_bytes(prism.FN_POLAR, 1, 4_194_400, 500, prism.F32, 5, 8)
