#!/usr/bin/env python3
"""Benchmark of the PRISM hot path on one MI355X.

A step is one pass of the whole path (norm, Gram/residual, sketch chain, fit, polynomial build and
apply, every iteration to the budget or tolerance) over one batch of synthetic matrices that is
already resident in HBM.

Default run: the headline is the large polar configuration (8 x 4096 x 4096 bf16, degree 5, sketch
32, tol 1e-2: the configuration the matrix-core target is stated on); the other four configurations
are measured in the same run with fewer steps and reported under "configs" of the same JSON line.
`--workload X` measures X alone (no "configs").  Prints ONE JSON line on stdout; progress goes to
stderr.
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
HBM_PEAK_GBS = 8000.0
TOL = {"c1": 1e-6, "c3": 1e-2, "c4": 1e-5, "c5": 1e-5, "sign": 1e-5, "inverse": 1e-5, "sqrt-newton": 1e-5}
# steps / warm-up of the configurations measured beside the headline
SIDE_STEPS = {"c1": (20, 3), "c2": (10, 3), "c3": (5, 2), "c4": (5, 2), "c5": (2, 1)}


def log(msg):
    print("[bench %6.1fs] %s" % (time.perf_counter() - T0, msg), file=sys.stderr, flush=True)


T0 = time.perf_counter()


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default=None,
                    choices=["c1", "c2", "c3", "c4", "c5", "sign", "inverse", "sqrt-newton"],
                    help="measure this workload alone (default: c3 as the headline plus c1, c2, c4, c5 under 'configs')")
    ap.add_argument("--split", action="store_true", help="c2: carry the iterate as a bf16 high+low pair")
    ap.add_argument("--batch", type=int, default=0, help="override the batch size (c3/c4/c5)")
    ap.add_argument("--no-grouped", dest="grouped", action="store_false",
                    help="c2: four calls per step instead of one prism_run_grouped call")
    ap.add_argument("--no-graph", dest="graph", action="store_false",
                    help="c2: launch the grouped call eagerly instead of replaying a captured HIP graph")
    ap.add_argument("--only-group", type=int, default=-1, help="c2: run a single shape group (profiling aid)")
    ap.add_argument("--input-cache", default=None, metavar="DIR",
                    help="keep the generated inputs of c3 / c5 (a minute of host work each) as .npy files in DIR and reuse them")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle legs")
    ap.add_argument("--no-profile", action="store_true", help="skip the per-kernel event pass")
    ap.add_argument("--single-stream", action="store_true",
                    help="keep every kernel on one stream (PRISM_FLAG_SINGLE_STREAM; no HIP graph): the launch configuration "
                         "of the per-kernel pass, for profiler runs in which no kernel is stretched by a neighbour")
    ap.add_argument("--gemm-probe", type=int, default=0, metavar="TILE",
                    help="only run the bare bf16 product 8 x 4096^3 (no epilogue work beyond the fp32 store) ten times with "
                         "tile 256, 2561 (256 x 128) or 128 (+ 10000: both operands stored [K][M] / [K][N], + 20000: the second "
                         "only), and print its rate: the kernel under the profiler's counters")
    ap.add_argument("--copy-probe", action="store_true",
                    help="only copy 1 GiB device to device three times (calibrates the FETCH_SIZE / WRITE_SIZE counters)")
    return ap.parse_args()


class Workload:
    """name, groups of host arrays, how to call the library, flop model."""


def cached(args, key, make):
    """make() or its copy kept in --input-cache (the generators are seeded: same bits either way)."""
    if not args.input_cache:
        return make()
    os.makedirs(args.input_cache, exist_ok=True)
    path = os.path.join(args.input_cache, key + ".npy")
    if os.path.exists(path):
        return np.load(path)
    arr = make()
    np.save(path, arr)
    return arr


def make_workload(name, args, prism, W):
    wl = Workload()
    wl.name = name
    wl.seed = W.SKETCH_SEED
    wl.split = False
    wl.p_s, wl.nv = 0, 0           # sketch width (padded) and products per chain, for the HBM-bound kernels
    ss = prism.FLAG_SINGLE_STREAM if args.single_stream else 0
    if name == "c2":
        wl.desc = "muon-shaped: 64 bf16 matrices = 16 x {768x768, 768x3072, 3072x768, 768x2304}, degree 5, sketch 16, 5 iterations" + \
                  (", split-bf16 iterate" if args.split else ", plain bf16 iterate")
        wl.dtype = "bf16"
        wl.host = [W.c2_muon_group(i) for i in range(4) if args.only_group < 0 or i == args.only_group]
        wl.flags = 0 if args.split else prism.FLAG_BF16_PLAIN_ITERATE
        # single calls (profile pass, --no-grouped) carry the hint that the grouped call gives its groups,
        # so that the same kernels are timed
        wl.call = lambda x: prism.polar(x, 5, 5, 16, wl.seed, 0.0, flags=wl.flags | prism.FLAG_SHARED_GPU | ss)
        wl.split = args.split
        wl.ld, wl.nv, wl.r_bytes = 16, 5, 2
    elif name == "c3":
        b = args.batch or 8
        wl.desc = "polar of %d x 4096x4096 bf16, sigma log-uniform [1e-4,1], degree 5, sketch 32, tol 1e-2, split-bf16 iterate" % b
        wl.dtype = "bf16"
        wl.host = [cached(args, "c3_b%d" % b, lambda: W.c3_polar_large(batch=b))]
        wl.call = lambda x: prism.polar(x, 5, 40, 32, wl.seed, 1e-2, flags=ss)
        wl.split = True
        wl.ld, wl.nv, wl.r_bytes = 32, 5, 2
    elif name == "c4":
        b = args.batch or 32
        wl.desc = "inverse 4th root of %d x 1024x1024 fp32 SPD (power-law spectrum), sketch 16, tol 1e-5" % b
        wl.dtype = "f32"
        wl.host = [W.c4_shampoo_spd(batch=b)]
        wl.call = lambda x: prism.inv_root(x, 4, 40, 16, wl.seed, 1e-5, flags=ss)
        wl.ld, wl.nv, wl.r_bytes = 16, 5, 4
    elif name == "c5":
        b = args.batch or 4
        wl.desc = "sqrt + inverse sqrt of %d x 8192x8192 fp32 SPD (Wishart), degree 5, sketch 64, tol 1e-5" % b
        wl.dtype = "f32"
        wl.host = [cached(args, "c5_b%d" % b, lambda: W.c5_wishart_spd(batch=b))]
        wl.call = lambda x: prism.sqrt(x, 5, 40, 64, wl.seed, 1e-5, flags=ss)[1]
        wl.ld, wl.nv, wl.r_bytes = 64, 5, 4
    elif name == "sqrt-newton":
        b = args.batch or 4
        wl.desc = "sqrt + inverse sqrt of %d x 8192x8192 fp32 SPD (Wishart, the config-5 inputs) by PRISM DB Newton, tol 1e-5, at most 12 iterations" % b
        wl.dtype = "f32"
        wl.host = [W.c5_wishart_spd(batch=b)]
        wl.call = lambda x: prism.sqrt_newton(x, 12, 1e-5)[1]
        wl.ld, wl.nv, wl.r_bytes = 0, 0, 4
    elif name == "sign":
        b = args.batch or 8
        wl.desc = "matrix sign of %d x 2048x2048 fp32 symmetric indefinite (|lambda| over 2 decades), degree 5, sketch 32, tol 1e-5" % b
        wl.dtype = "f32"
        wl.host = [W.sign_indefinite(n=2048, batch=b, decades=2.0)]
        wl.call = lambda x: prism.sign(x, 5, 40, 32, wl.seed, 1e-5)
        wl.ld, wl.nv, wl.r_bytes = 32, 5, 4
    elif name == "inverse":
        b = args.batch or 8
        wl.desc = "Chebyshev inverse of %d x 2048x2048 fp32 non-symmetric (cond 30), sketch 32, tol 1e-5" % b
        wl.dtype = "f32"
        wl.host = [W.inverse_general(n=2048, batch=b, cond=30.0)]
        wl.call = lambda x: prism.inverse(x, 40, 32, wl.seed, 1e-5)
        wl.ld, wl.nv, wl.r_bytes = 32, 3, 4
    else:
        wl.desc = "polar of one 64x32 fp32 matrix, cond 1e3, degree 5, sketch 8, tol 1e-6"
        wl.dtype = "f32"
        wl.host = [W.c1_polar_small()]
        wl.call = lambda x: prism.polar(x, 5, 30, 8, wl.seed, 1e-6)
        wl.ld, wl.nv, wl.r_bytes = 16, 5, 4
    wl.n_matrices = sum(h.shape[0] for h in wl.host)
    return wl


def to_device(h, torch):
    if h.dtype == np.uint16:
        return torch.from_numpy(h.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(h).cuda()


def flops_per_iteration(name, m, n, split):
    """(algorithmic, executed) GEMM flops of one iteration for one matrix.  Algorithmic: the dense
    products the method defines.  Executed: what the matrix cores run, i.e. half of the symmetric
    products of the polar iteration (Gram matrix and R^2: upper triangle of tiles only)."""
    S, L = min(m, n), max(m, n)
    if name in ("c1", "c2", "c3"):
        algo = 4.0 * L * S * S + 2.0 * S ** 3
        return algo, algo - (L * S * S + S ** 3) * (1.0 if name != "c1" else 0.0)
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


# kernel name as rocprofv3 prints it: gemm_bf16_kernel<tile rows, tile columns, epilogue, ...>
KERNEL_OF_KIND = {"bf16_gram": r"gemm_bf16\w*<\d+, \d+, 1,", "bf16_polyq": r"gemm_bf16\w*<\d+, \d+, 2,",
                  "bf16_apply": r"gemm_bf16\w*<\d+, \d+, 3,"}


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


def blas_threads():
    try:
        from threadpoolctl import threadpool_info
        return int(max([p.get("num_threads", 1) for p in threadpool_info()] or [1]))
    except Exception:
        return len(os.sched_getaffinity(0))


def run_config(name, K, Wm, args, torch, prism, W):
    """Measures one workload; returns its record (a dict)."""
    log("%s: generating inputs" % name)
    wl = make_workload(name, args, prism, W)
    log("%s: %s" % (name, wl.desc))

    # one pristine device copy per step: the calls work in place and nothing is re-uploaded in the timed region
    pristine = [to_device(h, torch) for h in wl.host]
    bytes_per_copy = sum(p.numel() * p.element_size() for p in pristine)
    n_copies = K + Wm
    copies = [[p.clone() for p in pristine] for _ in range(n_copies)]

    grouped = bool(args.grouped) and name == "c2" and len(wl.host) > 1
    graph = grouped and bool(args.graph) and not args.single_stream
    ss = prism.FLAG_SINGLE_STREAM if args.single_stream else 0

    def step(i, extra_flags=0):
        if grouped:
            return prism.run_grouped(prism.FN_POLAR, copies[i], 5, 5, 16, wl.seed, 0.0, flags=wl.flags | extra_flags | ss)[1]
        return [wl.call(x) for x in copies[i]]

    graphs = None
    if graph:
        # the calls allocate nothing once their workspace exists, so a step can be captured as is;
        # a graph holds fixed pointers, hence one graph per resident copy
        cap = torch.cuda.Stream()
        with torch.cuda.stream(cap):
            step(0)                      # creates the workspaces
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
    # one event before every step and one after the last: the steps queue back to back on the
    # stream, so consecutive events give each call's duration and first-to-last the whole region
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(K + 1)]
    handles = None
    for i in range(K):
        evs[i].record()
        handles = run_step(Wm + i)
    evs[K].record()
    torch.cuda.synchronize()
    ms_total = evs[0].elapsed_time(evs[K])
    per_call = np.array([evs[i].elapsed_time(evs[i + 1]) for i in range(K)])
    ms_per_step = ms_total / K
    value = wl.n_matrices / (ms_per_step * 1e-3)
    log("%s: %.3f ms per step (median %.3f, min %.3f)" % (name, ms_per_step, float(np.median(per_call)), float(per_call.min())))

    # iteration counts of the last step -> flops; res/tol at the stopping iteration and the one before
    infos = [h.read() for h in handles]
    algo = execd = 0.0
    iters_all, at_stop, before_stop = [], [], []
    for h, inf in zip(wl.host, infos):
        m, n = h.shape[1], h.shape[2]
        fa, fe = flops_per_iteration(wl.name, m, n, wl.split)
        for rec in inf:
            k = int(rec["iters"])
            algo += fa * k
            execd += fe * k
            iters_all.append(k)
            if name in TOL and rec["status"] == prism.INFO_CONVERGED:
                at_stop.append(float(rec["residual"][k]) / TOL[name])
                if k > 0:
                    before_stop.append(float(rec["residual"][k - 1]) / TOL[name])
    tflops_algo = algo / (ms_per_step * 1e-3) / 1e12
    tflops_exec = execd / (ms_per_step * 1e-3) / 1e12
    margin = None
    if at_stop:
        margin = {"res_over_tol_at_stop": [round(min(at_stop), 4), round(max(at_stop), 4)],
                  "res_over_tol_one_before": [round(min(before_stop), 3), round(max(before_stop), 3)] if before_stop else None}

    # CPU oracle on a bounded sample of the same workload, compared with the last step's output
    cpu = parity = None
    if not args.no_cpu:
        from oracle import prism_ref as O
        # sample sized to seconds of host work: all 64 of config 2, one matrix where one takes long
        per_group = {"c1": 1, "c2": 16, "c3": 1, "c4": 8, "c5": 1, "sign": 2, "inverse": 2, "sqrt-newton": 1}[wl.name]
        t_cpu, n_cpu, worst, counts_equal = 0.0, 0, 0.0, True
        last = copies[Wm + K - 1]
        for g, h in enumerate(wl.host):
            out = last[g][:per_group]
            if out.dtype == torch.bfloat16:
                out_h = W.from_bf16_bits(out.view(torch.int16).cpu().numpy().view(np.uint16))
            else:
                out_h = out.cpu().numpy()
            for i in range(min(per_group, h.shape[0])):
                t0 = time.perf_counter()
                ref, oinfo = oracle_call(wl.name, h[i], W, O, wl.seed)
                t_cpu += time.perf_counter() - t0
                n_cpu += 1
                worst = max(worst, float(np.linalg.norm(out_h[i].astype(np.float64) - ref) / np.linalg.norm(ref)))
                if oinfo["iters"] != int(infos[g][i]["iters"]) or oinfo["status"] != int(infos[g][i]["status"]):
                    counts_equal = False
        cpu = {"value": round(n_cpu / t_cpu, 4), "unit": "matrices/s", "cores": blas_threads(), "kind": "oracle",
               "sample": "%d of the %d matrices of the workload (the first %d of each shape group), numpy fp64"
                         % (n_cpu, wl.n_matrices, per_group)}
        if name == "c1":
            from threadpoolctl import threadpool_limits
            with threadpool_limits(limits=1):
                t0 = time.perf_counter()
                for _ in range(20):
                    oracle_call(wl.name, wl.host[0][0], W, O, wl.seed)
                cpu["single_thread_value"] = round(20.0 / (time.perf_counter() - t0), 2)
        parity = {"max_rel_fro_err_vs_oracle": worst, "iteration_counts_and_status_equal": counts_equal,
                  "matrices_checked": n_cpu, "bar": 2e-2 if wl.dtype == "bf16" else 1e-5}
        log("%s: oracle %.3f matrices/s, worst rel err %.2e, counts equal: %s" % (name, cpu["value"], worst, counts_equal))

    # per-kernel durations (HIP events around each launch) over a repeat of the timed steps
    roofline = None
    kernel_ms = {}
    hbm = {}
    if not args.no_profile:
        for i in range(n_copies):
            for dst, src in zip(copies[i], pristine):
                dst.copy_(src)
        torch.cuda.synchronize()
        nprof = min(K, 3)
        prism.profile_enable(True)
        for i in range(nprof):
            step(Wm + i, prism.FLAG_SINGLE_STREAM)     # every kernel on one stream: each is timed running alone
        torch.cuda.synchronize()
        prof = prism.profile_collect()
        prism.profile_enable(False)
        kernel_ms = {k: round(v[0] / nprof, 4) for k, v in prof.items() if v[1]}
        gemm_kinds = [k for k in prof if prof[k][1] and (k.startswith("bf16_") or k.startswith("f32_") or k.startswith("f64_")
                                                          or k == "spd_inverse")]
        dom = max(gemm_kinds, key=lambda k: prof[k][0])
        # algorithmic flops of all launches of that kind in the profiled steps
        fl = chain_bytes = moment_bytes = prep_bytes = 0.0
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
                k = int(rec["iters"])
                nit = k + (1 if dom in ("bf16_gram", "f32_resid") and rec["status"] == prism.INFO_CONVERGED else 0)
                fl += per_iter * nit
                # HBM-bound kernels: the chain reads R once per product, the moments read the chain
                # vectors once, pre-scaling reads the input once and writes the iterate once
                chain_bytes += k * wl.nv * float(S) * S * wl.r_bytes
                moment_bytes += k * wl.nv * float(S) * wl.ld * 4
                prep_bytes += 2.0 * m * n * h.dtype.itemsize
        fl *= nprof
        dur_s = prof[dom][0] * 1e-3
        dt_peak = "f64" if dom.startswith("f64") else ("bf16" if dom.startswith("bf16") else "f32")
        achieved = fl / dur_s / 1e12
        roofline = {"bound": "mfma", "kernel": dom, "achieved": round(achieved, 2), "peak": PEAK[dt_peak], "unit": "TFLOP/s",
                    "frac": round(achieved / PEAK[dt_peak], 4), "traffic": recorded_traffic(wl.name, dom),
                    "launches": int(prof[dom][1]), "avg_launch_ms": round(prof[dom][0] / prof[dom][1], 4)}
        for kind, nbytes in (("prep", prep_bytes), ("chain", chain_bytes), ("moments", moment_bytes)):
            if name != "c1" and kind in prof and prof[kind][1] and nbytes > 0:   # config 1 is one launch, bound by latency
                gbs = nbytes * nprof / (prof[kind][0] * 1e-3) / 1e9
                hbm[kind] = {"achieved_GBps": round(gbs, 1), "frac_of_hbm_peak": round(gbs / HBM_PEAK_GBS, 4),
                             "launches": int(prof[kind][1]), "avg_launch_ms": round(prof[kind][0] / prof[kind][1], 4)}

    rec = {
        "workload": wl.name + ": " + wl.desc, "dtype": wl.dtype, "steps": K, "warmup": Wm,
        "matrices_per_step": wl.n_matrices, "matrices_per_s": round(value, 3),
        "ms_per_step": round(ms_per_step, 4), "ms_per_step_median": round(float(np.median(per_call)), 4),
        "ms_per_step_min": round(float(per_call.min()), 4),
        "tflops_algorithmic": round(tflops_algo, 2), "tflops_executed": round(tflops_exec, 2),
        "frac_of_mfma_peak": round(tflops_exec / PEAK[wl.dtype], 4),
        "frac_of_mfma_peak_algorithmic": round(tflops_algo / PEAK[wl.dtype], 4),
        "iterations": {"min": min(iters_all), "max": max(iters_all)},
        "stop_margin": margin, "kernel_ms_per_step": kernel_ms,
        "roofline": roofline, "hbm_bound_kernels": hbm, "cpu_baseline": cpu, "parity": parity,
        "launch": {"input_bytes_per_step": bytes_per_copy, "calls_per_step": 1 if grouped or len(wl.host) == 1 else len(wl.host),
                   "hip_graph": graph, "grouped_call": grouped},
    }
    del copies, pristine, graphs, handles
    torch.cuda.empty_cache()
    return rec


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
    if args.gemm_probe:
        gen = torch.Generator(device="cuda").manual_seed(1)
        a = torch.randn(8, 4096, 4096, device="cuda", generator=gen).to(torch.bfloat16)
        b = torch.randn(8, 4096, 4096, device="cuda", generator=gen).to(torch.bfloat16)
        # + 10000: both operands stored with K as the slow index, + 20000: the second one only
        km = 3 if 10000 <= args.gemm_probe < 20000 else (2 if args.gemm_probe >= 20000 else 0)
        tile = args.gemm_probe % 10000
        prism.gemm_bf16_nt(a, b, tile, km)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(10):
            prism.gemm_bf16_nt(a, b, tile, km)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / 10
        print(json.dumps({"gemm_probe": "8 x 4096^3 bf16, tile %d" % args.gemm_probe, "ms": round(ms, 4),
                          "tflops": round(2 * 8 * 4096.0 ** 3 / ms / 1e9, 1)}))
        return

    head_name = args.workload or "c3"
    head = run_config(head_name, args.steps, args.warmup, args, torch, prism, W)
    out = {
        "metric": "matrices_per_s", "value": head["matrices_per_s"], "unit": "matrices/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["ms_per_step"],
        "ms_per_step_median": head["ms_per_step_median"], "ms_per_step_min": head["ms_per_step_min"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": head["dtype"], "data": "synthetic",
        "config": dict({"workload": head["workload"], "matrices_per_step": head["matrices_per_step"]}, **head["launch"]),
        "tflops_algorithmic": head["tflops_algorithmic"], "tflops_executed": head["tflops_executed"],
        "frac_of_mfma_peak": head["frac_of_mfma_peak"], "frac_of_mfma_peak_algorithmic": head["frac_of_mfma_peak_algorithmic"],
        "iterations": head["iterations"], "stop_margin": head["stop_margin"],
        "kernel_ms_per_step": head["kernel_ms_per_step"],
        "roofline": head["roofline"], "hbm_bound_kernels": head["hbm_bound_kernels"],
        "cpu_baseline": head["cpu_baseline"], "parity": head["parity"],
    }
    if args.workload is None:
        others = {}
        for name in ("c1", "c2", "c4", "c5"):
            k, w = SIDE_STEPS[name]
            others[name] = run_config(name, k, w, args, torch, prism, W)
        out["configs"] = others
    log("done")
    print(json.dumps(out))


if __name__ == "__main__":
    main()
