#!/usr/bin/env python3
"""Benchmark of the PRISM hot path on one MI355X.

A step is one pass of the whole path (norm, Gram/residual, sketch chain, fit, polynomial build and
apply, every iteration to the budget or tolerance) over one batch of synthetic matrices that is
already resident in HBM.  Default workload: the Muon-shaped batch (64 bf16 matrices, 16 each of
768x768, 768x3072, 3072x768, 768x2304; degree 5, sketch 16, 5 iterations).  Prints one JSON line.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK = {"bf16": 2500.0, "f32": 157.3, "f64": 78.6}   # dense MFMA TFLOP/s, MI355X


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c2", choices=["c1", "c2", "c3", "c4", "c5", "sign", "inverse", "sqrt-newton"])
    ap.add_argument("--split", action="store_true", help="c2: carry the iterate as a bf16 high+low pair")
    ap.add_argument("--batch", type=int, default=0, help="override the batch size (c3/c4/c5)")
    ap.add_argument("--streams", type=int, default=0,
                    help="HIP streams the calls of one step are spread over (default: one per shape group, i.e. 4 for c2)")
    ap.add_argument("--sub-batches", type=int, default=1,
                    help="split every group's batch into this many calls (spread over the streams)")
    ap.add_argument("--no-grouped", dest="grouped", action="store_false",
                    help="c2: four calls on --streams streams per step instead of one prism_run_grouped call (the default, in "
                         "which the library forks to its internal streams)")
    ap.add_argument("--graph", dest="graph", action="store_true", default=None,
                    help="capture every step's calls in a HIP graph beforehand and time the replays (one stream); "
                         "the default for c2 with the grouped call")
    ap.add_argument("--no-graph", dest="graph", action="store_false")
    ap.add_argument("--only-group", type=int, default=-1, help="c2: run a single shape group (profiling aid)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle leg")
    ap.add_argument("--no-profile", action="store_true", help="skip the per-kernel event pass")
    ap.add_argument("--copy-probe", action="store_true",
                    help="only copy 1 GiB device to device three times (calibrates the FETCH_SIZE / WRITE_SIZE counters)")
    return ap.parse_args()


class Workload:
    """name, groups of device tensors, how to call the library, flop model."""


def make_workload(args, torch, prism, W):
    wl = Workload()
    name = args.workload
    wl.name = name
    wl.seed = W.SKETCH_SEED
    if name == "c2":
        wl.desc = "muon-shaped: 64 bf16 matrices = 16 x {768x768, 768x3072, 3072x768, 768x2304}, degree 5, sketch 16, 5 iterations" + \
                  (", split-bf16 iterate" if args.split else ", plain bf16 iterate")
        wl.dtype = "bf16"
        wl.host = [W.c2_muon_group(i) for i in range(4) if args.only_group < 0 or i == args.only_group]
        wl.flags = 0 if args.split else prism.FLAG_BF16_PLAIN_ITERATE
        # single calls (profile pass, --no-grouped) carry the hint that the grouped call gives its groups,
        # so that the same kernels are timed
        wl.call = lambda x: prism.polar(x, 5, 5, 16, wl.seed, 0.0, flags=wl.flags | prism.FLAG_SHARED_GPU)
        wl.split = args.split
    elif name == "c3":
        b = args.batch or 8
        wl.desc = "polar of %d x 4096x4096 bf16, sigma log-uniform [1e-4,1], degree 5, sketch 32, tol 1e-2, split-bf16 iterate" % b
        wl.dtype = "bf16"
        wl.host = [W.c3_polar_large(batch=b)]
        wl.call = lambda x: prism.polar(x, 5, 40, 32, wl.seed, 1e-2)
        wl.split = True
    elif name == "c4":
        b = args.batch or 32
        wl.desc = "inverse 4th root of %d x 1024x1024 fp32 SPD (power-law spectrum), sketch 16, tol 1e-5" % b
        wl.dtype = "f32"
        wl.host = [W.c4_shampoo_spd(batch=b)]
        wl.call = lambda x: prism.inv_root(x, 4, 40, 16, wl.seed, 1e-5)
    elif name == "c5":
        b = args.batch or 4
        wl.desc = "sqrt + inverse sqrt of %d x 8192x8192 fp32 SPD (Wishart), degree 5, sketch 64, tol 1e-5" % b
        wl.dtype = "f32"
        wl.host = [W.c5_wishart_spd(batch=b)]
        wl.call = lambda x: prism.sqrt(x, 5, 40, 64, wl.seed, 1e-5)[1]
    elif name == "sqrt-newton":
        b = args.batch or 4
        wl.desc = "sqrt + inverse sqrt of %d x 8192x8192 fp32 SPD (Wishart, the config-5 inputs) by PRISM DB Newton, tol 1e-5, at most 12 iterations" % b
        wl.dtype = "f32"
        wl.host = [W.c5_wishart_spd(batch=b)]
        wl.call = lambda x: prism.sqrt_newton(x, 12, 1e-5)[1]
    elif name == "sign":
        b = args.batch or 8
        wl.desc = "matrix sign of %d x 2048x2048 fp32 symmetric indefinite (|lambda| over 2 decades), degree 5, sketch 32, tol 1e-5" % b
        wl.dtype = "f32"
        wl.host = [W.sign_indefinite(n=2048, batch=b, decades=2.0)]
        wl.call = lambda x: prism.sign(x, 5, 40, 32, wl.seed, 1e-5)
    elif name == "inverse":
        b = args.batch or 8
        wl.desc = "Chebyshev inverse of %d x 2048x2048 fp32 non-symmetric (cond 30), sketch 32, tol 1e-5" % b
        wl.dtype = "f32"
        wl.host = [W.inverse_general(n=2048, batch=b, cond=30.0)]
        wl.call = lambda x: prism.inverse(x, 40, 32, wl.seed, 1e-5)
    else:
        wl.desc = "polar of one 64x32 fp32 matrix, cond 1e3, degree 5, sketch 8, tol 1e-6"
        wl.dtype = "f32"
        wl.host = [W.c1_polar_small()]
        wl.call = lambda x: prism.polar(x, 5, 30, 8, wl.seed, 1e-6)
    wl.n_matrices = sum(h.shape[0] for h in wl.host)
    return wl


def to_device(h, torch):
    if h.dtype == np.uint16:
        return torch.from_numpy(h.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(h).cuda()


def flops_per_iteration(name, m, n, split):
    """(algorithmic, executed) GEMM flops of one iteration for one matrix (dense, no symmetry savings)."""
    S, L = min(m, n), max(m, n)
    if name in ("c1", "c2", "c3"):
        algo = 4.0 * L * S * S + 2.0 * S ** 3
        return algo, algo + (2.0 * L * S * S if split else 0.0)
    if name == "c5":
        return 8.0 * n ** 3, 8.0 * n ** 3
    if name == "sqrt-newton":           # block Gauss-Jordan inverse (2 n^3) and the two updates
        return 6.0 * n ** 3, 6.0 * n ** 3
    if name in ("sign", "inverse"):      # residual product, R^2, update
        return 6.0 * n ** 3, 6.0 * n ** 3
    return 8.0 * n ** 3, 8.0 * n ** 3      # c4, p = 4: X R, T^2, T^4, T^4 M


def oracle_call(name, host_matrix, W, O, seed):
    if name == "c2":
        return O.polar(W.from_bf16_bits(host_matrix), 5, 5, 16, seed, 0.0)
    if name == "c3":
        return O.polar(W.from_bf16_bits(host_matrix), 5, 40, 32, seed, 1e-2)
    if name == "c4":
        return O.inv_root(host_matrix, 4, 40, 16, seed, 1e-5)
    if name == "c5":
        r, _, info = O.sqrt(host_matrix, 5, 40, 64, seed, 1e-5)
        return r, info
    if name == "sqrt-newton":
        r, _, info = O.sqrt_db_newton(host_matrix, 12, 1e-5)
        return r, info
    if name == "sign":
        return O.sign(host_matrix, 5, 40, 32, seed, 1e-5)
    if name == "inverse":
        return O.inverse(host_matrix, 40, 32, seed, 1e-5)
    return O.polar(host_matrix, 5, 30, 8, seed, 1e-6)


KERNEL_OF_KIND = {"bf16_gram": r"gemm_bf16_kernel<\d+, 1,", "bf16_polyq": r"gemm_bf16_kernel<\d+, 2,",
                  "bf16_apply": r"gemm_bf16_kernel<\d+, 3,"}


def recorded_traffic(workload, kind):
    """HBM bytes per launch (fetch + write) of the dominant kernel, from the rocprofv3 --pmc summary
    committed under profiles/ for this workload (counters scaled by a copy of known size); None
    when no such summary exists.  It is a recorded measurement, not taken during this run."""
    import re
    path = os.path.join(ROOT, "profiles", "%s_hbm_traffic.md" % workload)
    pat = KERNEL_OF_KIND.get(kind)
    if pat is None or not os.path.exists(path):
        return None
    tot, n = {"FETCH_SIZE": 0.0, "WRITE_SIZE": 0.0}, {"FETCH_SIZE": 0, "WRITE_SIZE": 0}
    for line in open(path):
        cells = [c.strip() for c in line.split("|")]
        if len(cells) >= 6 and re.search(pat, cells[1]) and cells[2] in tot and cells[5]:
            d = int(cells[3])
            tot[cells[2]] += float(cells[5]) * d
            n[cells[2]] += d
    if not n["FETCH_SIZE"] or not n["WRITE_SIZE"]:
        return None
    return round(tot["FETCH_SIZE"] / n["FETCH_SIZE"] + tot["WRITE_SIZE"] / n["WRITE_SIZE"])


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); --gpus %d is not supported" % args.gpus,
              file=sys.stderr)
        sys.exit(2)
    import torch
    if args.copy_probe:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")     # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_probe_bytes": src.numel() * 4, "copies": 3}))
        return
    from paper_2601_22137_amd import prism, workloads as W
    prism.lib()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    wl = make_workload(args, torch, prism, W)
    K, Wm = args.steps, args.warmup

    # one pristine device copy per step: the calls work in place and nothing is re-uploaded in the timed region
    pristine = [to_device(h, torch) for h in wl.host]
    bytes_per_copy = sum(p.numel() * p.element_size() for p in pristine)
    n_copies = K + Wm
    copies = [[p.clone() for p in pristine] for _ in range(n_copies)]

    # The calls of one step (one per shape group) are independent: each goes to a stream of its own
    # (default priority), so that the small latency-bound kernels of one call run beside the GEMMs
    # of another.  Consecutive steps queue up behind each other on the same streams.
    nsub = max(1, args.sub_batches)
    if args.streams or args.sub_batches > 1 or wl.name != "c2":
        args.grouped = False
    if args.graph is None:
        args.graph = bool(args.grouped)
    nstreams = 1 if args.grouped else (args.streams or len(wl.host) * nsub)
    side = [torch.cuda.Stream() for _ in range(nstreams)] if nstreams > 1 else None

    def parts(x):
        if nsub == 1:
            return [x]
        per = (x.shape[0] + nsub - 1) // nsub
        return [x[j:j + per] for j in range(0, x.shape[0], per)]

    class Joined:      # the info records of the sub-batch calls of one group, in matrix order
        def __init__(self, hs):
            self.hs = hs

        def read(self):
            return np.concatenate([h.read() for h in self.hs])

    def step(i, use_streams=True):
        if args.grouped and use_streams and wl.name == "c2":
            return prism.run_grouped(prism.FN_POLAR, copies[i], 5, 5, 16, wl.seed, 0.0, flags=wl.flags)[1]
        hs, slot = [], 0
        for x in copies[i]:
            sub = []
            for xp in parts(x):
                if side is None or not use_streams:
                    sub.append(wl.call(xp))
                else:
                    with torch.cuda.stream(side[slot % nstreams]):
                        sub.append(wl.call(xp))
                slot += 1
            hs.append(Joined(sub))
        return hs

    graphs = None
    if args.graph:
        # the calls allocate nothing once their workspace exists, so a step can be captured as is;
        # a graph holds fixed pointers, hence one graph per resident copy
        side = None
        cap = torch.cuda.Stream()
        with torch.cuda.stream(cap):
            step(0)                      # creates the workspace of this stream
            cap.synchronize()
            for dst, src in zip(copies[0], pristine):
                dst.copy_(src)
            graphs = []
            for i in range(n_copies):
                gr = torch.cuda.CUDAGraph()
                with torch.cuda.graph(gr, stream=cap):
                    hs = step(i)
                graphs.append((gr, hs))
        torch.cuda.synchronize()

        def run_step(i):
            graphs[i][0].replay()
            return graphs[i][1]
    else:
        run_step = step

    for i in range(Wm):
        run_step(i)
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record()
    handles = None
    for i in range(K):
        handles = run_step(Wm + i)
    if side is not None:
        for st in side:
            torch.cuda.current_stream().wait_stream(st)
    ev1.record()
    torch.cuda.synchronize()
    ms_total = ev0.elapsed_time(ev1)
    ms_per_step = ms_total / K
    value = wl.n_matrices / (ms_per_step * 1e-3)

    # iteration counts of the last step -> flops
    infos = []
    for h in handles:
        infos.append(h.read())
    algo = execd = 0.0
    iters_all = []
    for h, inf in zip(wl.host, infos):
        m, n = h.shape[1], h.shape[2]
        fa, fe = flops_per_iteration(wl.name, m, n, getattr(wl, "split", False))
        for rec in inf:
            algo += fa * rec["iters"]
            execd += fe * rec["iters"]
            if getattr(wl, "split", False):
                # the low half of the iterate is multiplied only until the fitted alpha first leaves the
                # upper end of its interval (from that update on the library reads the high half alone)
                al = rec["alpha"][:rec["iters"]]
                below = np.nonzero(al < 1.4499)[0]
                n_split = int(below[0]) if len(below) else int(rec["iters"])
                execd -= (fe - fa) * (rec["iters"] - n_split)
            iters_all.append(int(rec["iters"]))
    tflops_algo = algo / (ms_per_step * 1e-3) / 1e12
    tflops_exec = execd / (ms_per_step * 1e-3) / 1e12

    # CPU oracle on a bounded sample of the same workload
    cpu = None
    parity = None
    if not args.no_cpu:
        from oracle import prism_ref as O
        try:
            from threadpoolctl import threadpool_info
            threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            threads = len(os.sched_getaffinity(0))
        # sample sized to 10-30 s of host work where one matrix takes long; config 2 is cheap enough for the whole batch
        per_group = {"c1": 1, "c2": 16, "c3": 1, "c4": 8, "c5": 1, "sign": 2, "inverse": 2, "sqrt-newton": 1}[wl.name]
        if wl.name in ("c3", "c5") and wl.host[0].shape[1] > 2048:
            per_group = 1
        t_cpu, n_cpu, worst = 0.0, 0, 0.0
        last = [x for x in copies[Wm + K - 1]]
        for g, h in enumerate(wl.host):
            out = last[g]
            if out.dtype == torch.bfloat16:
                out_h = W.from_bf16_bits(out.view(torch.int16).cpu().numpy().view(np.uint16))
            else:
                out_h = out.cpu().numpy()
            for i in range(min(per_group, h.shape[0])):
                t0 = time.perf_counter()
                ref, oinfo = oracle_call(wl.name, h[i], W, O, wl.seed)
                t_cpu += time.perf_counter() - t0
                n_cpu += 1
                rel = float(np.linalg.norm(out_h[i].astype(np.float64) - ref) / np.linalg.norm(ref))
                worst = max(worst, rel)
                if oinfo["iters"] != int(infos[g][i]["iters"]):
                    worst = float("inf")
        cpu = {"value": round(n_cpu / t_cpu, 4), "unit": "matrices/s", "cores": int(threads), "kind": "oracle",
               "sample": "%d matrices (%d per shape group) of the same workload, numpy fp64" % (n_cpu, per_group)}
        parity = {"max_rel_fro_err_vs_oracle": worst, "matrices_checked": n_cpu}

    # per-kernel durations (HIP events around each launch) over a repeat of the timed steps
    roofline = None
    kernel_ms = {}
    if not args.no_profile:
        for i in range(n_copies):
            for dst, src in zip(copies[i], pristine):
                dst.copy_(src)
        torch.cuda.synchronize()
        nprof = min(K, 3)
        prism.profile_enable(True)
        for i in range(nprof):
            step(Wm + i, use_streams=False)     # one stream: every kernel is timed running alone
        torch.cuda.synchronize()
        prof = prism.profile_collect()
        prism.profile_enable(False)
        kernel_ms = {k: round(v[0] / nprof, 4) for k, v in prof.items() if v[1]}
        gemm_kinds = [k for k in prof if prof[k][1] and (k.startswith("bf16_") or k.startswith("f32_") or k.startswith("f64_")
                                                          or k == "spd_inverse")]
        dom = max(gemm_kinds, key=lambda k: prof[k][0])
        # algorithmic flops of all launches of that kind in the profiled steps
        fl = 0.0
        for h, inf in zip(wl.host, infos):
            m, n = h.shape[1], h.shape[2]
            S, L = min(m, n), max(m, n)
            per_iter = {"bf16_apply": 2.0 * L * S * S, "bf16_gram": 2.0 * L * S * S, "bf16_polyq": 2.0 * S ** 3,
                        "f32_resid": 2.0 * L * S * S, "f32_polyq": 2.0 * S ** 3,
                        "f32_apply": (4.0 if wl.name in ("c5", "sqrt-newton") else 2.0) * L * S * S,
                        "f32_store": 4.0 * S ** 3, "f64_mnext": 2.0 * S ** 3, "spd_inverse": 2.0 * S ** 3,
                        # one launch runs every iteration: Gram, R^2 and the update
                        "f32_small_polar": 4.0 * L * S * S + 2.0 * S ** 3}[dom]
            for rec in inf:
                nit = rec["iters"] + (1 if dom in ("bf16_gram", "f32_resid") and rec["status"] == prism.INFO_CONVERGED else 0)
                fl += per_iter * nit
        fl *= nprof
        dur_s = prof[dom][0] * 1e-3
        dt_peak = "f64" if dom.startswith("f64") else ("bf16" if dom.startswith("bf16") else "f32")
        achieved = fl / dur_s / 1e12
        roofline = {"bound": "mfma", "kernel": dom, "achieved": round(achieved, 2), "peak": PEAK[dt_peak], "unit": "TFLOP/s",
                    "frac": round(achieved / PEAK[dt_peak], 4), "traffic": recorded_traffic(wl.name, dom),
                    "launches": int(prof[dom][1]), "avg_launch_ms": round(prof[dom][0] / prof[dom][1], 4)}

    out = {
        "metric": "matrices_per_s", "value": round(value, 3), "unit": "matrices/s", "n_gpus": 1, "steps": K, "warmup": Wm,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": wl.name + ": " + wl.desc, "matrices_per_step": wl.n_matrices,
                   "input_bytes_per_step": bytes_per_copy, "streams": nstreams,
                   "calls_per_step": 1 if args.grouped else len(wl.host) * nsub, "hip_graph": bool(args.graph), "grouped_call": bool(args.grouped)},
        "tflops_algorithmic": round(tflops_algo, 2), "tflops_executed": round(tflops_exec, 2),
        "frac_of_mfma_peak": round(tflops_exec / PEAK[wl.dtype], 4),
        "iterations": {"min": min(iters_all), "max": max(iters_all)},
        "kernel_ms_per_step": kernel_ms,
        "roofline": roofline, "cpu_baseline": cpu, "parity": parity,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
