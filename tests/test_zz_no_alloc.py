"""prism_polar_static (the entry point that allocates nothing: its intermediates live in a static
device array) against prism_polar_ex, through the C-ABI.  Same kernels, same plan: the outputs must
be the same bits, and both within the parity bar of the oracle.  Two calls in a row per case, the
second with a smaller input, so that the contents the first call leaves in the array are what the
second one starts from.  Collected last (file name): a failure here must not hide other tests.
"""
import ctypes

import numpy as np
import pytest
import torch

from oracle import prism_ref as O
from paper_2601_22137_amd import workloads as W

pytestmark = pytest.mark.gpu

SEED = W.SKETCH_SEED


@pytest.fixture(scope="module")
def prism():
    from paper_2601_22137_amd import prism as P
    P.lib()
    return P


def _rel(x, ref):
    return np.linalg.norm(np.asarray(x, dtype=np.float64) - ref) / np.linalg.norm(ref)


def _bf16_tensor(bits):
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)


def _bf16_to_f64(t):
    return W.from_bf16_bits(t.view(torch.int16).cpu().numpy().view(np.uint16)).astype(np.float64)


def _pair(prism, host, bf16, args, flags=0):
    """Runs the same input through prism_polar_ex and prism_polar_static; returns outputs and infos."""
    mk = (lambda: _bf16_tensor(host.copy())) if bf16 else (lambda: torch.from_numpy(host.copy()).cuda())
    x_ref, x_st = mk(), mk()
    info_st = prism.new_info(host.shape[0])          # made before the call: the call itself allocates nothing
    torch.cuda.synchronize()
    i_ref = prism.polar(x_ref, *args, flags=flags).read()
    before = torch.cuda.memory_allocated()
    prism.polar_static(x_st, *args, flags=flags, info=info_st)
    assert torch.cuda.memory_allocated() == before
    i_st = info_st.read()
    return x_ref, x_st, i_ref, i_st


def _same(prism, host, bf16, args, flags, tol):
    x_ref, x_st, i_ref, i_st = _pair(prism, host, bf16, args, flags)
    assert torch.equal(x_ref.view(torch.int16) if bf16 else x_ref, x_st.view(torch.int16) if bf16 else x_st)
    assert i_ref.tobytes() == i_st.tobytes()
    out = _bf16_to_f64(x_st) if bf16 else x_st.cpu().numpy().astype(np.float64)
    for i in range(host.shape[0]):
        a = W.from_bf16_bits(host[i]) if bf16 else host[i]
        ref, oinfo = O.polar(a, *args)
        assert _rel(out[i], ref) <= tol, (i, _rel(out[i], ref))
        assert int(i_st[i]["iters"]) == oinfo["iters"] and int(i_st[i]["status"]) == oinfo["status"]


def test_static_fp32_two_calls_second_smaller(prism):
    rng = np.random.default_rng(77)
    big = (rng.standard_normal((3, 330, 200)) * np.exp(rng.uniform(-3, 0, size=(3, 1, 200)))).astype(np.float32)
    small = (rng.standard_normal((2, 90, 130)) * np.exp(rng.uniform(-2, 0, size=(2, 90, 1)))).astype(np.float32)
    args = (5, 40, 8, SEED, 1e-5)
    _same(prism, big, False, args, 0, 1e-5)
    _same(prism, small, False, args, 0, 1e-5)
    _same(prism, W.c1_polar_small(), False, (5, 30, 8, SEED, 1e-6), 0, 1e-5)     # one-workgroup kernel, smaller still


@pytest.mark.parametrize("plain", [False, True])
def test_static_bf16_two_calls_second_smaller(prism, plain):
    flags = prism.FLAG_BF16_PLAIN_ITERATE if plain else 0
    big = W.c2_muon_group(1, batch=2, scale=2)         # 384 x 1536: wide, transposed internally
    small = W.c2_muon_group(0, batch=3, scale=4)       # 192 x 192
    args = (5, 5, 16, SEED, 0.0)
    _same(prism, big, True, args, flags, 2e-2)
    _same(prism, small, True, args, flags, 2e-2)
    ragged = W.to_bf16_bits(np.concatenate([W.c1_polar_small(m=257, n=64, data_seed=1300 + i) for i in range(2)]))
    x_ref, x_st, i_ref, i_st = _pair(prism, ragged, True, (5, 40, 8, SEED, 1e-2), flags)
    assert torch.equal(x_ref.view(torch.int16), x_st.view(torch.int16)) and i_ref.tobytes() == i_st.tobytes()


def test_static_rejects_what_does_not_fit_and_a_caller_workspace(prism):
    lib = prism.lib()
    need = prism.workspace_bytes(prism.FN_POLAR, 16, 768, 768, prism.BF16, 5, 16)
    assert need > prism.STATIC_SCRATCH_BYTES
    x = torch.zeros((16, 768, 768), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(prism.PrismError, match="PRISM_EUNSUPPORTED"):
        prism.polar_static(x, 5, 5, 16, SEED, 0.0)
    assert "PRISM_STATIC_SCRATCH_BYTES" in lib.prism_last_error().decode()
    o = prism.Options()
    ws = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")
    o.workspace = ws.data_ptr()
    o.workspace_bytes = ws.numel()
    y = torch.ones((1, 64, 32), dtype=torch.float32, device="cuda")
    rc = lib.prism_polar_static(y.data_ptr(), 1, 64, 32, prism.F32, 5, 10, 8, SEED, 1e-6, None, ctypes.byref(o))
    assert rc == prism.EINVAL
    # empty input: valid, nothing enqueued
    assert lib.prism_polar_static(None, 0, 64, 32, prism.F32, 5, 10, 8, SEED, 1e-6, None, None) == prism.OK
    torch.cuda.synchronize()
    assert torch.all(y == 1.0)
