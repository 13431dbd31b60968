"""The grouped call (one library call over groups of different shapes, internal fork / join
streams): every group must come out exactly as from its own single-group call, and against the
oracle to the usual bars; the optimizer-side helpers are thin wrappers around it."""
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


def _bf16(bits):
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)


def test_grouped_polar_equals_single_calls_and_oracle(prism):
    """Muon-shaped groups at a quarter of the size (192x192, 192x768, 768x192, 192x576), six groups
    so that internal streams are reused, twice in a row."""
    bits = [W.c2_muon_group(i % 4, batch=3 + i, scale=4, data_seed=1002 + 10 * (i // 4)) for i in range(6)]
    single = []
    for b in bits:
        x = _bf16(b.copy())
        prism.polar(x, 5, 5, 16, SEED, 0.0, flags=prism.FLAG_BF16_PLAIN_ITERATE)
        single.append(x)
    for rep in range(3):   # the last one with every kernel on the caller's stream
        xs = [_bf16(b.copy()) for b in bits]
        flags = prism.FLAG_BF16_PLAIN_ITERATE | (prism.FLAG_SINGLE_STREAM if rep == 2 else 0)
        _, infos = prism.run_grouped(prism.FN_POLAR, xs, 5, 5, 16, SEED, 0.0, flags=flags)
        torch.cuda.synchronize()
        for g, (x, ref) in enumerate(zip(xs, single)):
            assert torch.equal(x.view(torch.int16), ref.view(torch.int16)), g
            rec = infos[g].read()
            assert np.all(rec["iters"] == 5)
    out0 = W.from_bf16_bits(xs[1][0].view(torch.int16).cpu().numpy().view(np.uint16))
    ref, _ = O.polar(W.from_bf16_bits(bits[1][0]), 5, 5, 16, SEED, 0.0)
    assert _rel(out0, ref) <= 2e-2


def test_grouped_polar_in_parts_on_internal_streams(prism):
    """Batches that are multiples of four: the one launch sequence over all shapes is issued per
    quarter of every group on internal streams (split iterate here, and a tolerance, so that the
    per-matrix stop flags matter).  Same bits as the single calls, reports in the caller's arrays."""
    bits = [W.c2_muon_group(i, batch=8, scale=4, data_seed=1500 + i) for i in range(4)]
    single, single_info = [], []
    for b in bits:
        x = _bf16(b.copy())
        single_info.append(prism.polar(x, 5, 30, 16, SEED, 2e-2).read())
        single.append(x)
    xs = [_bf16(b.copy()) for b in bits]
    _, infos = prism.run_grouped(prism.FN_POLAR, xs, 5, 30, 16, SEED, 2e-2)
    torch.cuda.synchronize()
    for g in range(4):
        assert torch.equal(xs[g].view(torch.int16), single[g].view(torch.int16)), g
        rec = infos[g].read()
        assert np.array_equal(rec["iters"], single_info[g]["iters"]) and np.array_equal(rec["alpha"], single_info[g]["alpha"])
        assert np.array_equal(rec["status"], single_info[g]["status"])
    out0 = W.from_bf16_bits(xs[2][5].view(torch.int16).cpu().numpy().view(np.uint16))
    ref, oinfo = O.polar(W.from_bf16_bits(bits[2][5]), 5, 30, 16, SEED, 2e-2)
    assert _rel(out0, ref) <= 2e-2 and infos[2].read()[5]["iters"] == oinfo["iters"]


def test_grouped_fp32_polar_with_small_and_general_groups(prism):
    """fp32 groups to tolerance: three whose padded iterate is 64 x 64 (they run in the one-workgroup
    kernel) beside one that takes the general path; same bits as the single calls, oracle parity."""
    shapes = [(5, 64, 32), (3, 200, 72), (2, 40, 24), (4, 48, 64)]
    As = [np.concatenate([W.c1_polar_small(m=m, n=n, data_seed=2100 + 10 * g + i) for i in range(b)])
          for g, (b, m, n) in enumerate(shapes)]
    single = []
    for A in As:
        x = torch.from_numpy(A.copy()).cuda()
        prism.polar(x, 5, 30, 8, SEED, 1e-6)
        single.append(x)
    xs = [torch.from_numpy(A.copy()).cuda() for A in As]
    _, infos = prism.run_grouped(prism.FN_POLAR, xs, 5, 30, 8, SEED, 1e-6)
    torch.cuda.synchronize()
    for g, (x, ref) in enumerate(zip(xs, single)):
        assert torch.equal(x, ref), g
        rec = infos[g].read()
        want, oinfo = O.polar(As[g][0], 5, 30, 8, SEED, 1e-6)
        assert _rel(x[0].cpu().numpy(), want) <= 1e-5
        assert rec[0]["iters"] == oinfo["iters"] and rec[0]["status"] == prism.INFO_CONVERGED


def test_grouped_call_replays_from_a_hip_graph(prism):
    """The fork onto the internal streams and the join back are event waits, so a grouped call
    captures from the caller's stream like a single one: every replay, with eager work and
    synchronisations in between, must give the bits of the eager call."""
    bits = [W.c2_muon_group(i, batch=4, scale=4) for i in range(4)]
    src = [_bf16(b.copy()) for b in bits]
    eager = [t.clone() for t in src]
    _, h = prism.run_grouped(prism.FN_POLAR, eager, 5, 5, 16, SEED, 0.0, flags=prism.FLAG_BF16_PLAIN_ITERATE)
    torch.cuda.synchronize()
    alpha_eager = [r.read()["alpha"].copy() for r in h]
    xs = [t.clone() for t in src]
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        prism.run_grouped(prism.FN_POLAR, xs, 5, 5, 16, SEED, 0.0, flags=prism.FLAG_BF16_PLAIN_ITERATE)   # warm-up
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            _, handles = prism.run_grouped(prism.FN_POLAR, xs, 5, 5, 16, SEED, 0.0, flags=prism.FLAG_BF16_PLAIN_ITERATE)
        for _ in range(3):
            for x, s0 in zip(xs, src):
                x.copy_(s0)                                      # eager work between the replays
            graph.replay()
            side.synchronize()
            for g in range(4):
                assert torch.equal(xs[g].view(torch.int16), eager[g].view(torch.int16)), g
                assert np.array_equal(handles[g].read()["alpha"], alpha_eager[g])


def test_grouped_inverse_root_and_sqrt(prism):
    A1, A2 = W.c4_shampoo_spd(n=128, batch=2), W.c4_shampoo_spd(n=200, batch=3, data_seed=77)
    xs = [torch.from_numpy(A1.copy()).cuda(), torch.from_numpy(A2.copy()).cuda()]
    _, infos = prism.run_grouped(prism.FN_INV_ROOT, xs, 3, 40, 16, SEED, 1e-5, root_p=4)
    for A, x, h in zip((A1, A2), xs, infos):
        rec = h.read()
        for i in range(A.shape[0]):
            ref, oinfo = O.inv_root(A[i], 4, 40, 16, SEED, 1e-5)
            assert _rel(x[i].cpu().numpy(), ref) <= 1e-5
            assert rec[i]["iters"] == oinfo["iters"]
    S1, S2 = W.c5_wishart_spd(n=128, batch=2), W.c5_wishart_spd(n=192, batch=1, data_seed=5)
    xs = [torch.from_numpy(S1.copy()).cuda(), torch.from_numpy(S2.copy()).cuda()]
    invs, infos = prism.run_grouped(prism.FN_SQRT_NEWTON, xs, 3, 30, 1, SEED, 1e-5)
    for S, x, inv in zip((S1, S2), xs, invs):
        rx, ry, _ = O.sqrt_db_newton(S[0], 30, 1e-5)
        assert _rel(x[0].cpu().numpy(), rx) <= 1e-5 and _rel(inv[0].cpu().numpy(), ry) <= 1e-5


def test_grouped_argument_errors(prism):
    x = torch.zeros((1, 16, 16), dtype=torch.float32, device="cuda")
    with pytest.raises(prism.PrismError):
        prism.run_grouped(prism.FN_POLAR, [x, torch.zeros((1, 8, 8), dtype=torch.float32, device="cuda")], 4, 3, 0, SEED, 0.0)


def test_optimizer_helpers(prism):
    from paper_2601_22137_amd import optim
    rng = np.random.default_rng(3)
    shapes = [(96, 64), (64, 96), (96, 64), (128, 128), (64, 96)]
    grads = [torch.from_numpy(rng.standard_normal(s).astype(np.float32)).cuda() for s in shapes]
    outs = optim.muon_orthogonalize(grads, degree=5, iters=8, sketch_dim=8)
    for g, o in zip(grads, outs):
        assert o.shape == g.shape
        ref, _ = O.polar(g.cpu().numpy(), 5, 8, 8, SEED, 0.0)
        assert _rel(o.cpu().numpy(), ref) <= 1e-5
    stats = [torch.from_numpy(W.c4_shampoo_spd(n=n, batch=1, data_seed=90 + n)[0]).cuda() for n in (64, 128, 64)]
    roots, iters = optim.shampoo_inverse_roots(stats, root_p=4)
    for s, r, it in zip(stats, roots, iters):
        ref, oinfo = O.inv_root(s.cpu().numpy(), 4, 40, 16, SEED, 1e-5)
        assert _rel(r.cpu().numpy(), ref) <= 1e-5 and it == oinfo["iters"]


def test_shared_gpu_flag_is_a_scheduling_hint(prism):
    """PRISM_FLAG_SHARED_GPU changes tile sizes only: at a size where it does (Gram dimension 768,
    a multiple of 256) a single call with the flag gives the bits of the grouped call, and both stay
    within the rounding of the unflagged call."""
    bits = [W.c2_muon_group(0, batch=2), W.c2_muon_group(3, batch=2)]
    plain = prism.FLAG_BF16_PLAIN_ITERATE
    xs = [_bf16(b.copy()) for b in bits]
    prism.run_grouped(prism.FN_POLAR, xs, 5, 5, 16, SEED, 0.0, flags=plain)
    torch.cuda.synchronize()
    for g, b in enumerate(bits):
        hinted = _bf16(b.copy())
        prism.polar(hinted, 5, 5, 16, SEED, 0.0, flags=plain | prism.FLAG_SHARED_GPU)
        assert torch.equal(hinted.view(torch.int16), xs[g].view(torch.int16))
        unhinted = _bf16(b.copy())
        prism.polar(unhinted, 5, 5, 16, SEED, 0.0, flags=plain)
        d = (unhinted.float() - hinted.float()).norm() / hinted.float().norm()
        assert float(d) <= 2e-2


def test_calls_from_two_host_threads(prism):
    """Two host threads, each with a stream of its own, issue calls of different shapes at the same
    time (ctypes releases the GIL during a call): workspaces are per stream and the shared state of
    the library is locked, so both get the bits of the same calls made one after the other."""
    import threading
    jobs = [(np.concatenate([W.c1_polar_small(m=200, n=72, data_seed=2500 + i) for i in range(3)]), 5),
            (np.concatenate([W.c1_polar_small(m=64, n=32, data_seed=2600 + i) for i in range(6)]), 3)]
    want = []
    for A, deg in jobs:
        x = torch.from_numpy(A.copy()).cuda()
        prism.polar(x, deg, 30, 8, SEED, 1e-6)
        want.append(x)
    torch.cuda.synchronize()
    got, errors = [None, None], []

    def work(j):
        try:
            A, deg = jobs[j]
            st = torch.cuda.Stream()
            with torch.cuda.stream(st):
                for _ in range(20):
                    x = torch.from_numpy(A.copy()).cuda()
                    prism.polar(x, deg, 30, 8, SEED, 1e-6)
                st.synchronize()
            got[j] = x
        except Exception as e:          # noqa: BLE001 - reported by the assertion below
            errors.append(e)

    threads = [threading.Thread(target=work, args=(j,)) for j in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors
    for j in range(2):
        assert torch.equal(got[j], want[j]), j
