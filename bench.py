#!/usr/bin/env python3
"""Benchmark of the PCSR SpMM hot path on one MI355X.

A step is one C = A*B over the whole synthetic workload (PCSR traversal, B gather + FMA,
write-back), with the PCSR arrays, B and C already resident in HBM.  PCSR generation and
feature extraction are one-off per graph (the paper amortises them over training
iterations) and are reported in separate fields, outside the timed region.

Prints ONE JSON line: metric/value (GFLOP/s = 2*nnz*K / t), the HBM roofline of the SpMM
kernel measured live with device events, and the CPU oracle timed on this machine's cores.
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

import numpy as np

HBM_PEAK_GBS = 8000.0
# HBM bytes per SpMM launch measured with rocprofv3 --pmc (FETCH_SIZE and WRITE_SIZE runs,
# each scaled by what the counter reads for a plain copy kernel of known size); the
# summaries with the commands are under profiles/.  Keyed by workload, K, the kernel instance
# that was profiled, the item size SG and the item schedule: a run that launches another
# instance, or the same instance over another PCSR layout, reports null.
PROFILED_TRAFFIC = {
    ("poisson-full", 32, "spmm_kernel<1, false, 8, 4, 1>", 0, "index"): 3503085,
    ("road-full", 128, "spmm_kernel<2, false, 32, 4, 1>", 0, "index"): 2121481179,
    ("rmat20-full", 64, "spmm_kernel<1, true, 16, 4, 1>", 32, "column"): 2050060690,
    ("sbm-full", 256, "spmm_window_kernel<1, 16, 4, 1>", 0, "index"): 2230701604,
    ("sbm_shuffled-full", 256, "spmm_kernel<1, true, 16, 4, 1>", 32, "column"): 10018994230,
    ("rmat22-full", 16, "spmm_kernel<1, true, 16, 1, 1>", 32, "column"): 6858113234,
    ("rmat22-full", 32, "spmm_kernel<1, true, 8, 4, 1>", 32, "column"): 9844466834,
    ("rmat22-full", 64, "spmm_kernel<1, true, 16, 4, 1>", 32, "column"): 17907130971,
    ("rmat22-full", 128, "spmm_kernel<1, true, 16, 4, 1>", 32, "column"): 36026222500,
    ("rmat22-full", 256, "spmm_kernel<1, true, 16, 4, 1>", 32, "column"): 75014491538,
    ("rmat22-full", 512, "spmm_kernel<1, true, 16, 4, 1>", 32, "column"): 155942151679,
}


def kernel_instance(V: int, S: int, launch: dict) -> str:
    """Name of the SpMM kernel instance as rocprofv3 prints it."""
    shape = f"{launch['lanes_per_row']}, {launch['vec']}, {launch['rep']}"
    if launch["lds_bytes"]:
        return f"spmm_window_kernel<{V}, {shape}>"
    if launch["items_per_group"] > 1:
        return f"spmm_batched_kernel<{V}, {shape}, {launch['items_per_group']}>"
    return f"spmm_kernel<{V}, {'true' if S else 'false'}, {shape}>"


def algorithmic_bytes(g, K: int) -> int:
    """Minimum HBM traffic of one SpMM: colidx + val once, rowptr once, every referenced
    B row once, C once."""
    n_refcols = int(np.unique(g.colidx).shape[0])
    return g.nnz * 8 + (g.n_rows + 1) * 4 + n_refcols * K * 4 + g.n_rows * K * 4


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="rmat22",
                    help="rmat22 (default: the largest benchmark configuration) | road | rmat20 | sbm | "
                         "sbm_shuffled | poisson")
    ap.add_argument("--K", type=int, default=0,
                    help="0 = the workload's benchmark width (the widest one, 512, for rmat22's K sweep)")
    ap.add_argument("--size", default="full", choices=["full", "small"])
    ap.add_argument("--V", type=int, default=-1, help="-1 = library selector")
    ap.add_argument("--S", type=int, default=-1)
    ap.add_argument("--SG", type=int, default=0)
    ap.add_argument("--lanes-per-row", type=int, default=0)
    ap.add_argument("--vec", type=int, default=0)
    ap.add_argument("--rep", type=int, default=0)
    ap.add_argument("--waves", type=int, default=0)
    ap.add_argument("--items-per-group", type=int, default=0)
    ap.add_argument("--col-window", type=int, default=-1, help="-1 = library selector")
    ap.add_argument("--gpu-build", action="store_true", help="generate the PCSR arrays with GPU kernels")
    ap.add_argument("--reorder", nargs="?", const="cluster", default=None, choices=["cluster", "degree"],
                    help="apply one of the library's relabellings first (A' = P A P^T, B' = P B): 'cluster' = "
                         "label propagation (pcsr_reorder), 'degree' = descending in-degree "
                         "(pcsr_reorder_by_degree); the timed SpMM runs on the relabelled problem and its "
                         "result is checked as C = P^T C'")
    ap.add_argument("--no-xcd-remap", action="store_true")
    ap.add_argument("--index-order", action="store_true",
                    help="S = 1: run the work items in index order even where the selector asks for the "
                         "column-ordered schedule")
    ap.add_argument("--atomic-split", action="store_true",
                    help="S = 1: accumulate split panels with fp32 atomics instead of the two-pass write-back")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-check", action="store_true")
    ap.add_argument("--graph-batch", type=int, default=-1,
                    help="also capture this many SpMMs in one HIP graph and report the replay time per SpMM "
                         "beside the launch floor (-1 = 64 when one launch takes under 50 us, else off)")
    ap.add_argument("--no-hipsparse", action="store_true", help="skip the hipSPARSE SpMM comparison leg")
    ap.add_argument("--no-stream", action="store_true",
                    help="skip the copy-kernel measurement of the achievable HBM stream rate")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 1 GiB elementwise copy kernel (reads 1 GiB, writes 1 GiB) so a "
                         "rocprofv3 --pmc run of this command holds a dispatch of known traffic")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build is single-GPU; run with --gpus 1 (no sharded path exists)",
              file=sys.stderr)
        return 2

    import torch

    import paper_2605_15695_amd as pc
    import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)

    t0 = time.time()
    g = synth.workload(args.workload, args.size)
    spec = synth.WORKLOADS[args.workload]
    K = args.K or max(spec["K"])
    B = synth.dense_operand(g.n_cols, K, spec["B"], 2)
    gen_s = time.time() - t0

    perm, reorder_ms = None, None
    g_orig, B_orig = g, B
    if args.reorder:
        t0 = time.time()
        if args.reorder == "degree":
            perm = pc.pcsr_reorder_by_degree(g.n_rows, g.rowptr, g.colidx)
        else:
            perm, n_clusters = pc.pcsr_reorder(g.n_rows, g.rowptr, g.colidx)
        rp, ci, va = pc.pcsr_permute_csr(g.n_rows, g.rowptr, g.colidx, g.vals, perm)
        reorder_ms = (time.time() - t0) * 1e3
        g = synth.Graph(g.name + "_reordered", g.n_rows, g.n_cols, rp, ci, va)
        B = np.empty_like(B_orig)
        B[perm] = B_orig

    t0 = time.time()
    feats = pc.pcsr_features(g.n_rows, g.n_cols, g.rowptr, g.colidx)
    sel = pc.pcsr_select(feats, K)
    feat_ms = (time.time() - t0) * 1e3
    # the library's own pick, with any field overridden from the command line
    V = sel.V if args.V < 0 else args.V
    S = sel.S if args.S < 0 else args.S
    params = pc.make_params(
        V=V, S=S, SG=args.SG or (sel.SG if S == sel.S else 0),
        lanes_per_row=args.lanes_per_row or sel.lanes_per_row, vec=args.vec or sel.vec,
        rep=args.rep or sel.rep, waves_per_wg=args.waves or sel.waves_per_wg,
        items_per_group=args.items_per_group or sel.items_per_group,
        col_window=sel.col_window if args.col_window < 0 else args.col_window,
        flags=(sel.flags if S == sel.S and not args.index_order else 0)
        | (pc.PCSR_FLAG_NO_XCD_REMAP if args.no_xcd_remap else 0)
        | (pc.PCSR_FLAG_GPU_BUILD if args.gpu_build else 0)
        | (pc.PCSR_FLAG_ATOMIC_SPLIT if args.atomic_split else 0))
    t0 = time.time()
    h = pc.pcsr_build(g.n_rows, g.n_cols, g.rowptr, g.colidx, g.vals, params)
    build_ms = (time.time() - t0) * 1e3
    launch = pc.pcsr_query_launch(h, K)
    instance = kernel_instance(V, S, launch)
    schedule = "column" if (int(params.flags) & pc.PCSR_FLAG_COLUMN_ORDER) and S else "index"
    workload_name = f"{args.workload}-{args.size}" + (f"+reorder({args.reorder})" if args.reorder else "")
    pc.pcsr_reserve_workspace(h, K)

    Bd = torch.from_numpy(B).cuda()
    Cd = torch.empty((g.n_rows, K), dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream()

    for _ in range(args.warmup):
        pc.pcsr_spmm(h, Bd, Cd, K, stream)
    torch.cuda.synchronize()

    # timed region: exactly `steps` SpMMs, each bracketed by events on the launch stream
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
           for _ in range(args.steps)]
    torch.cuda.synchronize()
    wall0 = time.perf_counter()
    for a, b in evs:
        a.record(stream)
        pc.pcsr_spmm(h, Bd, Cd, K, stream)
        b.record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - wall0
    per_launch_ms = [a.elapsed_time(b) for a, b in evs]
    ms_per_step = wall * 1e3 / args.steps
    kern_ms = statistics.fmean(per_launch_ms)

    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.mul(src, 1.0, out=dst)
        torch.cuda.synchronize()
        del src, dst

    flops = 2.0 * g.nnz * K
    bytes_min = algorithmic_bytes(g, K)
    achieved = bytes_min / (kern_ms * 1e-3) / 1e9

    # What a plain copy reaches on this machine (1 GiB read + 1 GiB written per launch): the
    # practical ceiling beside the 8 TB/s of the data sheet.
    stream_gbs = None
    if not args.no_stream:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.mul(src, 1.0, out=dst)
        cev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(10)]
        for a, b in cev:
            a.record(stream)
            torch.mul(src, 1.0, out=dst)   # an elementwise kernel; copy_() may go through the DMA engines
            b.record(stream)
        torch.cuda.synchronize()
        stream_gbs = 2.0 * src.numel() * 4 / (statistics.median(a.elapsed_time(b) for a, b in cev) * 1e-3) / 1e9
        del src, dst

    out = {
        "metric": "SpMM GFLOP/s (2*nnz*K)",
        "value": flops / (ms_per_step * 1e-3) / 1e9,
        "unit": "GFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": workload_name, "graph": g.name, "n": g.n_rows,
                   "nnz": g.nnz, "K": K, "V": V, "S": S, "SG": int(params.SG), "schedule": schedule,
                   **launch, "kernel": instance,
                   "workspace_bytes": pc.pcsr_workspace_bytes(h, K)},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS,
                     "copy_kernel_gbs": stream_gbs,
                     "frac_of_copy_kernel": achieved / stream_gbs if stream_gbs else None,
                     "traffic": PROFILED_TRAFFIC.get((workload_name, K, instance, int(params.SG), schedule)),
                     "kernel_ms_mean": kern_ms, "kernel_ms_median": statistics.median(per_launch_ms),
                     "kernel_ms_min": min(per_launch_ms), "algorithmic_bytes": bytes_min},
        "setup": {"generate_s": gen_s, "features_select_ms": feat_ms, "pcsr_build_ms": build_ms,
                  "reorder_ms": reorder_ms},
    }

    gb = args.graph_batch if args.graph_batch >= 0 else (64 if kern_ms < 0.05 else 0)
    if gb > 0:
        # launch-bound regime: N SpMMs replayed from one captured graph, and the same graph
        # shape filled with a one-element kernel as the floor of what a launch costs
        side = torch.cuda.Stream()
        tiny = torch.zeros(64, device="cuda")

        def captured(fn):
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                fn(side)
            side.synchronize()
            gr = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gr, stream=side):
                for _ in range(gb):
                    fn(torch.cuda.current_stream())
            for _ in range(3):
                gr.replay()
            torch.cuda.synchronize()
            ts = []
            for _ in range(20):
                t0 = time.perf_counter()
                gr.replay()
                torch.cuda.synchronize()
                ts.append((time.perf_counter() - t0) * 1e6 / gb)
            return statistics.median(ts)

        us_spmm = captured(lambda st: pc.pcsr_spmm(h, Bd, Cd, K, st))
        us_floor = captured(lambda st: tiny.add_(1.0))
        out["launch_bound"] = {"graph_batch": gb, "us_per_spmm_in_graph": us_spmm,
                               "us_per_empty_kernel_in_graph": us_floor,
                               "us_per_spmm_eager_events": kern_ms * 1e3,
                               "us_per_step_eager_wall": ms_per_step * 1e3}

    # ---- the CPU oracle as it stands, on this machine's host cores, on a bounded sample of rows
    rows = ref = bound = None
    if not args.no_check or not args.no_cpu_baseline:
        import oracle

        if g.nnz * K <= 2.5e9:
            sample, reps = "full workload, best of 3", 3
        else:
            n_s = max(1, int(g.n_rows * 2.5e9 / (g.nnz * K)))
            rows = np.sort(np.random.default_rng(0).choice(g.n_rows, n_s, replace=False)).astype(np.int64)
            sample, reps = f"{n_s} random rows of {g.n_rows}, 1 run", 1

        def run_oracle(sel, n_threads=0):
            t0 = time.perf_counter()
            if sel is None:
                r, b = oracle.spmm(g_orig.rowptr, g_orig.colidx, g_orig.vals, B_orig, n_threads=n_threads)
            else:
                r, b = oracle.spmm_rows(g_orig.rowptr, g_orig.colidx, g_orig.vals, B_orig, sel,
                                        n_threads=n_threads)
            return r, b, time.perf_counter() - t0

        deg_orig = np.diff(g_orig.rowptr.astype(np.int64))
        ncores = oracle.max_threads()            # read before the one-thread run lowers the setting
        # one thread first (an eighth of the sample), then all cores
        one_rows = (rows if rows is not None else np.arange(g.n_rows, dtype=np.int64))[::8]
        _, _, t_one = run_oracle(one_rows, n_threads=1)
        one_flops = 2.0 * float(deg_orig[one_rows].sum()) * K
        best = float("inf")
        for _ in range(reps):
            ref, bound, t = run_oracle(rows, n_threads=ncores)
            best = min(best, t)
        cpu_flops = flops if rows is None else 2.0 * float(deg_orig[rows].sum()) * K
        out["cpu_baseline"] = {"value": cpu_flops / best / 1e9, "unit": "GFLOP/s",
                               "cores": ncores, "kind": "oracle", "sample": sample,
                               "single_thread_value": one_flops / t_one / 1e9,
                               "single_thread_sample": f"every 8th row of that sample ({one_rows.shape[0]} rows)"}

    def sampled(Cx, relabelled):
        """Rows of a device result that the oracle sample covers, in the oracle's row order."""
        if rows is None:
            got = Cx.cpu().numpy()
            return got[perm] if (relabelled and perm is not None) else got
        sel_rows = rows if (perm is None or not relabelled) else perm[rows].astype(np.int64)
        return Cx[torch.from_numpy(sel_rows).cuda()].cpu().numpy()

    if not args.no_hipsparse:
        # vendor baseline on the same arrays (best of its CSR algorithms), outside the timed region
        import ctypes

        from paper_2605_15695_amd import sweep as sw

        lib = sw._baseline_lib()
        d_csr = [torch.from_numpy(x).cuda() for x in (g.rowptr, g.colidx, g.vals)]
        Ch = torch.empty_like(Cd)
        best_h, hs_ok = None, True
        for name, alg in sw.HIPSPARSE_ALGS.items():
            ctx = ctypes.c_void_p()
            rc = lib.hsp_spmm_create(g.n_rows, g.n_cols, g.nnz, d_csr[0].data_ptr(), d_csr[1].data_ptr(),
                                     d_csr[2].data_ptr(), Bd.data_ptr(), Ch.data_ptr(), K, alg,
                                     stream.cuda_stream, ctypes.byref(ctx))
            if rc != 0:
                continue
            med, _ = sw.time_launches(lambda: lib.hsp_spmm_run(ctx), stream, torch, 3, 10)
            lib.hsp_spmm_destroy(ctx)
            if ref is not None:
                # hipSPARSE works on the (possibly relabelled) arrays the PCSR handle was built from
                ok_h, _ = oracle.within_tolerance(sampled(Ch, True), ref, bound)
                hs_ok = hs_ok and ok_h
            if best_h is None or med < best_h[1]:
                best_h = (name, med)
        if best_h:
            out["hipsparse"] = {"alg": best_h[0], "ms": best_h[1], "gflops": flops / best_h[1] / 1e6,
                                "pcsr_speedup": best_h[1] / kern_ms,
                                "max_abs_diff_vs_pcsr": float((Ch - Cd).abs().max().item()),
                                "within_oracle_tolerance": bool(hs_ok) if ref is not None else None}
        del Ch, d_csr

    if ref is not None:
        ok, worst = oracle.within_tolerance(sampled(Cd, True), ref, bound)
        out["parity"] = {"ok": bool(ok), "worst_err_over_limit": worst}
        if not ok:
            print(json.dumps(out))
            print("bench.py: GPU result is outside tolerance", file=sys.stderr)
            return 1
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
