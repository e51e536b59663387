#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X.

One step = one full Gram-matrix evaluation (`mgk_gram`) of the large-batch
configuration: 2000 molecule-like graphs of 20-60 vertices, all 2 001 000
unordered pairs, fp32, q = 0.05, PCG to a relative residual of 1e-6.  The
graphs are loaded, reordered and packed once (outside the timed region, as
the paper argues for its own measurements: reordering is done once, the Gram
matrix is evaluated many times); launch -> values on the device is timed.

Prints ONE JSON line with the throughput in graph pairs/s, the matvec
element-pair rate, the ALU roofline of the solver kernels (timed with HIP events
on the launch stream) and the CPU oracle timed on a bounded sample.  The
`roofline` object says which kernels ran (from the library's launch record),
whether they keep the matrix entries in registers, and gives three fractions of
the fp32 vector peak: `frac` (algorithmic flops of the paper's cost model),
`frac_executed` (flops the product really executes: 2 per element pair and
iteration when the entries are cached) and `frac_executed_counters` (all fp32
vector flops, from the committed rocprofv3 counter summary of this command),
the same step with the entries regenerated in every product (`on_the_fly`),
and the HBM traffic from the committed FETCH_SIZE / WRITE_SIZE summary.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

FP32_VECTOR_PEAK_TFLOPS = 157.3   # MI355X published fp32 vector peak (packed FMA)
FLOPS_PER_ELEMENT_PAIR = 8        # SE-labeled element pair: 3 + kappa_e (sub, square, scale, exp, mul)


def _is_named_workload(workload, args):
    return (args.graphs == 2000 and args.product_cache == 1 and not args.waves and args.edge_kernel == "se"
            and args.reorder == 1 and args.tile_path == 0)


def hbm_traffic(workload, args):
    """HBM bytes per step from the committed counter summary (two rocprofv3 --pmc
    runs of this very command, FETCH_SIZE and WRITE_SIZE, each scaled by what the
    counter reads for a copy of known size).  Counters cannot be read from inside this
    process, so the figure is only given for the exact workloads and default settings it
    was measured on (profiles/hbm_traffic.json names the command of every entry)."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if not _is_named_workload(workload, args) or not os.path.exists(path):
        return None
    with open(path) as fh:
        entry = json.load(fh).get(workload)
    return entry["bytes_per_step"] if entry else None


def counted_flops(workload, args):
    """fp32 flops per step executed by the vector ALUs, from the committed rocprofv3 counter
    summary of this command (SQ_INSTS_VALU_ADD_F32 + MUL_F32 + 2 FMA_F32 + TRANS_F32 wave
    instructions x 64 lanes); same restriction as hbm_traffic."""
    path = os.path.join(ROOT, "profiles", "valu_flops.json")
    if not _is_named_workload(workload, args) or not os.path.exists(path):
        return None
    with open(path) as fh:
        entry = json.load(fh).get(workload)
    return entry["flops_per_step"] if entry else None


def _time_steps(torch, step, steps):
    step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def ablation(args, torch, W, M) -> int:
    """The paper's incremental study (Section VI, time to solution per optimisation level)
    mapped onto this library's switches, on the paper's two synthetic sets and on the
    benchmark workload, then Gram time and few-pair latency against the workgroup size.
    Levels, each keeping everything of the one before:
      tiles        non-empty octiles only, dense tile-pair product, vectors in global memory,
                   graphs in the given vertex order            (paper: Sparse)
      +reorder     PBR vertex order                            (paper: +Reorder)
      +adaptive    dense or sparse product chosen per pair     (paper: +Adaptive)
      +block       whole solve in one workgroup, both graphs and p, y shared in LDS,
                   jobs in the given order                     (paper: +Block)
      +dynsched    most expensive pairs first                  (paper: +DynSched)
      +registers   off-diagonal entries of small pairs kept in registers (not in the paper)
    The compact octile format (paper: +Compact) is the only storage format built, so it is
    part of every level; the paper's naive dense level is not built."""
    levels = [
        ("tiles", dict(reorder=0, onchip=0, tile_path=2, sched=0, cache=0)),
        ("+reorder", dict(reorder=1, onchip=0, tile_path=2, sched=0, cache=0)),
        ("+adaptive", dict(reorder=1, onchip=0, tile_path=0, sched=0, cache=0)),
        ("+block", dict(reorder=1, onchip=16384, tile_path=0, sched=0, cache=0)),
        ("+dynsched", dict(reorder=1, onchip=16384, tile_path=0, sched=1, cache=0)),
        ("+registers", dict(reorder=1, onchip=16384, tile_path=0, sched=1, cache=1)),
    ]
    solver = M.Solver(0)
    for name in ("nws", "ba", "config4"):
        wb = W.paper_synthetic(name) if name != "config4" else W.config4(args.graphs)
        G = wb.n_graphs
        K = torch.zeros((G, G), dtype=torch.float32, device="cuda")
        solver.configure(wb.params)
        solver.set_solver(1e-6, 0)
        solver.set_launch(0)
        batches = {}
        for label, lv in levels:
            if name == "config4" and lv["onchip"] == 0:
                continue   # two million pairs with vectors in global memory do not fit
            if lv["reorder"] not in batches:
                batches[lv["reorder"]] = solver.load_batch(wb, reorder=lv["reorder"])
            B = batches[lv["reorder"]]
            solver.set_onchip_limit(lv["onchip"])
            solver.set_tile_path(lv["tile_path"])
            solver.set_schedule(bool(lv["sched"]))
            solver.set_product_cache(bool(lv["cache"]))
            ms = _time_steps(torch, lambda: solver.gram(B, K), args.steps)
            print(json.dumps({"study": "levels", "workload": name, "level": label, "ms_per_gram": ms,
                              "pairs_per_s": G * (G + 1) / 2 / (ms * 1e-3)}), flush=True)
        for b in batches.values():
            b.free()
    # workgroup size against throughput (whole Gram) and latency (4 pairs alone), streaming
    # on-chip kernel, graphs of 10-40 vertices (a size every workgroup size can hold; a
    # pair too large for the requested size gets the next larger one)
    wb = W.config1()
    solver.configure(wb.params)
    solver.set_product_cache(False)
    B = solver.load_batch(wb)
    K = torch.zeros((100, 100), dtype=torch.float32, device="cuda")
    order = np.argsort(-wb.sizes())[:8].astype(np.int32)   # the four largest pairs
    K4 = torch.zeros(4, dtype=torch.float32, device="cuda")
    for waves in (1, 2, 4, 8, 16):
        solver.set_launch(waves)
        ms_g = _time_steps(torch, lambda: solver.gram(B, K), 20)
        ms_p = _time_steps(torch, lambda: solver.pairs(B, B, order[:4], order[4:], K4), 50)
        print(json.dumps({"study": "workgroup size", "workload": "config1", "waves_per_pair": waves,
                          "ms_per_gram": ms_g, "ms_4_largest_pairs": ms_p}), flush=True)
    solver.set_launch(0)
    solver.set_product_cache(True)
    ms_g = _time_steps(torch, lambda: solver.gram(B, K), 20)
    ms_p = _time_steps(torch, lambda: solver.pairs(B, B, order[:4], order[4:], K4), 50)
    print(json.dumps({"study": "workgroup size", "workload": "config1", "waves_per_pair": "auto, registers",
                      "ms_per_gram": ms_g, "ms_4_largest_pairs": ms_p}), flush=True)
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--graphs", type=int, default=2000, help="graphs in the batch (2000 = the named workload)")
    ap.add_argument("--workload", default="config4",
                    help="config4 (default, the benchmark line), config0, config1, config2:<density>, "
                         "mixed:<density>:<density>, config3, nws, ba")
    ap.add_argument("--waves", type=int, default=0, help="wavefronts per pair (0 = library default)")
    ap.add_argument("--reorder", type=int, default=1, help="0 none, 1 PBR, 2 RCM")
    ap.add_argument("--tile-path", type=int, default=0, help="global-memory solver: 0 auto, 1 sparse, 2 dense, 3 sparse with p gathered from global memory")
    ap.add_argument("--product-cache", type=int, default=1,
                    help="on-chip solver: 1 keep the matrix entries of small pairs in registers, 0 regenerate them")
    ap.add_argument("--edge-kernel", default="se",
                    help="se (default, the benchmark line), poly (Wendland (1-r)^4(4r+1), radius 0.25), "
                         "kron_se (3 attributes), rconv_se (3 parts): the other edge base kernels, on the "
                         "Gram workloads")
    ap.add_argument("--ablation", action="store_true",
                    help="instead of the benchmark line: time the optimisation levels of the paper's "
                         "incremental study and a workgroup-size sweep, one JSON line each")
    ap.add_argument("--on-the-fly", type=int, default=1,
                    help="1: after the timed steps also time the step with the entries regenerated in "
                         "every product and report it beside the default (0 for counter runs)")
    ap.add_argument("--cpu-sample", type=int, default=64, help="pairs timed on the CPU oracle (0 = skip)")
    ap.add_argument("--calibrate-copy-mib", type=int, default=0,
                    help="also run one device-to-device copy of this many MiB before the timed region; "
                         "under `rocprofv3 --pmc FETCH_SIZE` / `WRITE_SIZE` it calibrates the counters")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: the pair list shards trivially across GPUs, but this "
              "build and its test boxes have a single MI355X; run with --gpus 1", file=sys.stderr)
        return 2

    import torch
    import mgk_workloads as W
    import paper_1910_06310_amd as M

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2

    if args.ablation:
        return ablation(args, torch, W, M)

    wl = args.workload
    pair_list = None
    if wl == "config4":
        wb = W.config4(args.graphs)
        wl_name = "config4: Gram of %d molecule-like graphs (20-60 vertices)" % wb.n_graphs
    elif wl == "config0":
        wb = W.config0()
        wl_name = "config0: Gram of 4 random graphs of 6-10 vertices"
    elif wl == "config1":
        wb = W.config1()
        wl_name = "config1: Gram of 100 molecule-like graphs (10-40 vertices)"
    elif wl.startswith("config2"):
        rho = float(wl.split(":")[1]) if ":" in wl else 0.05
        wb = W.config2(rho)
        pair_list = (np.arange(0, 128, 2, dtype=np.int32), np.arange(1, 128, 2, dtype=np.int32))
        wl_name = "config2: 64 pairs of ER graphs, n=256, edge density %g" % rho
    elif wl.startswith("mixed:"):
        # 64 pairs of one graph of each of two densities (n = 256): the cross-density study of
        # the tile-pair primitives (Section IV-B)
        _, da, db = wl.split(":")
        wb = W.concat_batches([W.config2(float(da), 64), W.config2(float(db), 64)],
                              name="mixed[%s x %s]" % (da, db))
        pair_list = (np.arange(0, 64, dtype=np.int32), np.arange(64, 128, dtype=np.int32))
        wl_name = "64 pairs of ER graphs, n=256, edge densities %s against %s" % (da, db)
    elif wl in ("nws", "ba"):
        wb = W.paper_synthetic(wl)
        wl_name = "paper synthetic set %s: Gram of 160 graphs of 96 nodes" % wl.upper()
    elif wl == "config3":
        wb = W.config3()
        pair_list = (np.arange(0, 32, 2, dtype=np.int32), np.arange(1, 32, 2, dtype=np.int32))
        wl_name = "config3: 16 pairs of 3-D geometric graphs, n=2048, mean degree 12"
    else:
        print("unknown workload " + wl, file=sys.stderr)
        return 2
    flops_per_element_pair = FLOPS_PER_ELEMENT_PAIR
    if args.edge_kernel != "se":
        import dataclasses
        ek = args.edge_kernel
        if ek == "poly":
            wb.params = dataclasses.replace(wb.params, edge_kernel="poly", poly_rho=0.25,
                                            poly_coef=(1.0, 0.0, -10.0, 20.0, -15.0, 4.0))
            flops_per_element_pair = 3 + 1 + 2 * 5       # difference, Horner of degree 5
        elif ek in ("kron_se", "rconv_se"):
            dim = 3
            prm = dataclasses.replace(wb.params, edge_kernel=ek, label_dim=dim,
                                      length_scales=(0.15, 0.4, 0.25) if ek == "kron_se" else (0.3,))
            wb = W.with_label_attributes(wb, np.random.default_rng(7), dim, 0.3, prm)
            # per attribute (pair of parts): difference, square, accumulate; one (dim^2) exponentials
            flops_per_element_pair = 3 + (3 * dim + 2 if ek == "kron_se" else 5 * dim * dim)
        else:
            print("unknown edge kernel " + ek, file=sys.stderr)
            return 2
        wl_name += ", edge kernel " + ek
    G = wb.n_graphs
    solver = M.Solver(0)
    solver.configure(wb.params)
    solver.set_solver(1e-6, 0)
    solver.set_launch(args.waves)
    solver.set_tile_path(args.tile_path)
    solver.set_product_cache(int(args.product_cache))
    t0 = time.perf_counter()
    B = solver.load_batch(wb, reorder=args.reorder)
    load_s = time.perf_counter() - t0
    stats = B.stats()

    if pair_list is None:
        K = torch.zeros((G, G), dtype=torch.float32, device="cuda")
        iters = torch.zeros((G, G), dtype=torch.int32, device="cuda")
        flags = torch.zeros((G, G), dtype=torch.int32, device="cuda")

        def step():
            solver.gram(B, K, iters, flags)
    else:
        K = torch.zeros(len(pair_list[0]), dtype=torch.float32, device="cuda")
        iters = torch.zeros(len(pair_list[0]), dtype=torch.int32, device="cuda")
        flags = torch.zeros(len(pair_list[0]), dtype=torch.int32, device="cuda")

        def step():
            solver.pairs(B, B, pair_list[0], pair_list[1], K, iters, flags)

    if args.calibrate_copy_mib > 0:
        src = torch.ones(args.calibrate_copy_mib * 262144, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    t0 = time.perf_counter()
    step()                                   # first call also builds the job list
    torch.cuda.synchronize()
    first_s = time.perf_counter() - t0
    for _ in range(max(args.warmup - 1, 0)):
        step()
    torch.cuda.synchronize()

    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
          for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for a, b in ev:
        a.record()
        step()
        b.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    kernel_ms = [a.elapsed_time(b) for a, b in ev]

    if pair_list is None:
        pi, pj = W.gram_pairs(G)
    else:
        pi, pj = pair_list
    n_pairs = len(pi)
    ms_per_step = wall * 1e3 / args.steps
    pairs_per_s = n_pairs / (wall / args.steps)

    # exact work from the returned iteration counts: sum over pairs of
    # iterations * nnz(A) * nnz(A')
    it_all = iters.cpu().numpy().astype(np.float64)
    fl_all = flags.cpu().numpy()
    it = it_all[pi, pj] if pair_list is None else it_all
    out_iter_range = [int(it.min()), int(it.max())] if len(it) else [0, 0]
    z = wb.nnz().astype(np.float64)
    element_pairs = float((it * z[pi] * z[pj]).sum())
    pair_iterations = float(it.sum())
    not_converged = int((fl_all[pi, pj] if pair_list is None else fl_all).sum())
    kernel_s = float(np.mean(kernel_ms)) * 1e-3
    alg_flops = flops_per_element_pair * element_pairs
    achieved_tflops = alg_flops / kernel_s / 1e12

    out = {
        "metric": "graph pairs/sec (marginalized graph kernel, PCG to 1e-6, on-the-fly matvec)",
        "value": pairs_per_s,
        "unit": "pairs/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {
            "workload": "%s, %d pairs" % (wl_name, n_pairs),
            "q": wb.params.q, "h": wb.params.h, "length_scale": wb.params.length_scale,
            "rtol": 1e-6, "reorder": {0: "none", 1: "pbr", 2: "rcm"}[args.reorder],
            "waves_per_pair": args.waves or "auto",
            "tile_path": {0: "auto", 1: "sparse", 2: "dense", 3: "sparse, global gathers"}[args.tile_path],
            "product_cache": int(args.product_cache),
        },
        "matvec_element_pairs_per_s": element_pairs / kernel_s,
        "mean_iterations": pair_iterations / n_pairs,
        "iterations_min_max": out_iter_range,
        "not_converged": not_converged,
        "tiles": stats["n_tiles"], "offdiag_tiles": stats["n_offdiag_tiles"], "nnz": stats["nnz"],
        "load_and_pack_s": load_s, "first_call_s": first_s,
        "roofline": None,
    }
    # which kernels ran: from the library's own record of the launches of the last step
    launches = [ln for ln in solver.launch_log().splitlines() if ln.strip()]

    def _pairs_of(ln):
        for tok in ln.split():
            if tok.startswith("pairs="):
                return int(tok[6:])
        return 0

    dominant = max(launches, key=_pairs_of).split(" pairs=")[0] if launches else "none"
    families = sorted({ln.split("<")[0].split(" ")[0] for ln in launches})
    cached_pairs = sum(_pairs_of(ln) for ln in launches if "entries_cached=1" in ln)
    entries_cached = cached_pairs > 0
    # Executed flops of the product.  Entries regenerated (Alg. 2 as printed): the algorithmic
    # count per element pair and iteration.  Entries cached in registers: one multiply-add
    # (2 flop) per element pair and iteration, plus the one-off generation of each entry.
    zz = float((z[pi] * z[pj]).sum())
    # (A few pairs of a cached launch may not fit the entry-keeping kernel; they are counted
    # by their share of the pairs.)
    cached_share = cached_pairs / n_pairs if n_pairs else 0.0
    executed_per_pair_iter = 2 * cached_share + flops_per_element_pair * (1.0 - cached_share)
    executed_flops = (executed_per_pair_iter * element_pairs
                      + cached_share * (flops_per_element_pair - 2) * zz)
    traffic = hbm_traffic(wl, args)
    cflops = counted_flops(wl, args)
    out["roofline"] = {
        "bound": "alu",
        "kernel": dominant,
        "kernel_families": families,
        "launch_shapes": len(launches),
        "entries_cached": entries_cached,
        "entries_cached_share_of_pairs": cached_share,
        "achieved": achieved_tflops,
        "peak": FP32_VECTOR_PEAK_TFLOPS,
        "unit": "TFLOP/s",
        "frac": achieved_tflops / FP32_VECTOR_PEAK_TFLOPS,
        "frac_is": "algorithmic: %d flop per element pair and iteration (the paper's cost model for "
                   "this edge kernel) x element pairs / kernel time / peak" % flops_per_element_pair,
        "flops_per_element_pair": flops_per_element_pair,
        "executed_flops_per_element_pair": executed_per_pair_iter,
        "frac_executed": (executed_flops / kernel_s / 1e12 / FP32_VECTOR_PEAK_TFLOPS
                          if executed_flops is not None else None),
        "frac_executed_counters": (cflops / kernel_s / 1e12 / FP32_VECTOR_PEAK_TFLOPS
                                   if cflops is not None else None),
        "traffic": traffic,
        "hbm_GBps": traffic / kernel_s / 1e9 if traffic is not None else None,
        "element_pairs_per_step": element_pairs,
        "kernel_ms_per_step": kernel_s * 1e3,
    }

    # The same step with the entries regenerated in every product (Alg. 2 as printed), so that
    # the rate of flops actually executed by the on-the-fly product stands beside the default.
    if entries_cached and pair_list is None and args.product_cache == 1 and args.on_the_fly:
        solver.set_product_cache(0)
        step()
        torch.cuda.synchronize()
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(2)]
        for a, b in evs:
            a.record()
            step()
            b.record()
        torch.cuda.synchronize()
        otf_s = float(np.mean([a.elapsed_time(b) for a, b in evs])) * 1e-3
        it2 = iters.cpu().numpy().astype(np.float64)[pi, pj]
        ep2 = float((it2 * z[pi] * z[pj]).sum())
        out["roofline"]["on_the_fly"] = {
            "kernel_ms_per_step": otf_s * 1e3,
            "pairs_per_s": n_pairs / otf_s,
            "frac": flops_per_element_pair * ep2 / otf_s / 1e12 / FP32_VECTOR_PEAK_TFLOPS,
            "note": "mgk_set_product_cache(0): every entry regenerated in every product, "
                    "%d flop per element pair executed" % flops_per_element_pair,
        }
        solver.set_product_cache(1)
        step()   # leave K, iters, flags as the default path wrote them
        torch.cuda.synchronize()

    if args.cpu_sample > 0:
        from oracle import c_oracle as C
        if pair_list is None and int(wb.sizes().max()) ** 2 <= 4096:
            sel = np.random.default_rng(0).choice(len(pi), min(args.cpu_sample, len(pi)), replace=False)
            C.pairs(wb, pi[sel[:1]], pj[sel[:1]], tier=0)   # build + load outside the clock
            t0 = time.perf_counter()
            ref = C.pairs(wb, pi[sel], pj[sel], tier=0)
            cpu_s = time.perf_counter() - t0
            got = K.cpu().numpy().astype(np.float64)[pi[sel], pj[sel]]
            t0 = time.perf_counter()
            C.pairs(wb, pi[sel], pj[sel], tier=1)
            cpu_mf_s = time.perf_counter() - t0
            out["cpu_baseline"] = {
                "value": len(sel) / cpu_s,
                "unit": "pairs/s",
                "cores": C.threads(),
                "kind": "oracle",
                "sample": "%d of %d pairs drawn uniformly (seed 0), dense fp64 assemble + Cholesky, "
                          "one pair per thread; rate extrapolates to the whole Gram" % (len(sel), n_pairs),
                "matrix_free_tier_pairs_per_s": len(sel) / cpu_mf_s,
                "max_rel_err_gpu_vs_oracle": float(np.max(np.abs(got - ref) / ref)),
            }
        else:
            # pairs too large for the dense tier: matrix-free fp64 CG on the first pairs of the list
            m = min(args.cpu_sample, n_pairs)
            t0 = time.perf_counter()
            ref = C.pairs(wb, pi[:m], pj[:m], tier=1)
            cpu_s = time.perf_counter() - t0
            Kh = K.cpu().numpy().astype(np.float64)
            got = Kh[pi[:m], pj[:m]] if pair_list is None else Kh[:m]
            out["cpu_baseline"] = {
                "value": m / cpu_s,
                "unit": "pairs/s",
                "cores": C.threads(),
                "kind": "oracle",
                "sample": "first %d of %d pairs, matrix-free fp64 conjugate gradients to 1e-13 "
                          "(rows of the first graph in parallel)" % (m, n_pairs),
                "max_rel_err_gpu_vs_oracle": float(np.max(np.abs(got - ref) / ref)),
            }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
