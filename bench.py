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
# summaries with the commands are under profiles/.  Keyed by (workload, K).
PROFILED_TRAFFIC = {
    ("road-full", 128): 2_121_501_891,      # profiles/spmm_road_K128.md
    ("sbm-full", 256): 1_867_418_528,       # profiles/spmm_sbm_K256.md
    ("rmat20-full", 64): 2_996_129_152,     # profiles/spmm_rmat20_K64.md
    ("rmat22-full", 64): 29_434_107_301,    # profiles/spmm_rmat22_K64.md
}


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
    ap.add_argument("--workload", default="road", help="road | rmat20 | sbm | sbm_shuffled | poisson | rmat22")
    ap.add_argument("--K", type=int, default=0, help="0 = the workload's benchmark width")
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
    ap.add_argument("--reorder", action="store_true",
                    help="apply the library's locality reordering first (A' = P A P^T, B' = P B); the timed "
                         "SpMM runs on the relabelled problem and its result is checked as C = P^T C'")
    ap.add_argument("--no-xcd-remap", action="store_true")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-check", action="store_true")
    ap.add_argument("--graph-batch", type=int, default=-1,
                    help="also capture this many SpMMs in one HIP graph and report the replay time per SpMM "
                         "beside the launch floor (-1 = 64 when one launch takes under 50 us, else off)")
    ap.add_argument("--no-hipsparse", action="store_true", help="skip the hipSPARSE SpMM comparison leg")
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
    from paper_2605_15695_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)

    t0 = time.time()
    g = synth.workload(args.workload, args.size)
    spec = synth.WORKLOADS[args.workload]
    K = args.K or spec["K"][0]
    B = synth.dense_operand(g.n_cols, K, spec["B"], 2)
    gen_s = time.time() - t0

    perm, reorder_ms = None, None
    g_orig, B_orig = g, B
    if args.reorder:
        t0 = time.time()
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
        flags=(pc.PCSR_FLAG_NO_XCD_REMAP if args.no_xcd_remap else 0)
        | (pc.PCSR_FLAG_GPU_BUILD if args.gpu_build else 0))
    t0 = time.time()
    h = pc.pcsr_build(g.n_rows, g.n_cols, g.rowptr, g.colidx, g.vals, params)
    build_ms = (time.time() - t0) * 1e3
    launch = pc.pcsr_query_launch(h, K)

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
        "config": {"workload": f"{args.workload}-{args.size}" + ("+reorder" if args.reorder else ""),
                   "graph": g.name, "n": g.n_rows,
                   "nnz": g.nnz, "K": K, "V": V, "S": S, **launch},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS,
                     "traffic": PROFILED_TRAFFIC.get((f"{args.workload}-{args.size}", K)),
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

    if not args.no_hipsparse:
        # vendor baseline on the same arrays (best of its CSR algorithms), outside the timed region
        import ctypes

        from paper_2605_15695_amd import sweep as sw

        lib = sw._baseline_lib()
        d_csr = [torch.from_numpy(x).cuda() for x in (g.rowptr, g.colidx, g.vals)]
        Ch = torch.empty_like(Cd)
        best_h = None
        for name, alg in sw.HIPSPARSE_ALGS.items():
            ctx = ctypes.c_void_p()
            rc = lib.hsp_spmm_create(g.n_rows, g.n_cols, g.nnz, d_csr[0].data_ptr(), d_csr[1].data_ptr(),
                                     d_csr[2].data_ptr(), Bd.data_ptr(), Ch.data_ptr(), K, alg,
                                     stream.cuda_stream, ctypes.byref(ctx))
            if rc != 0:
                continue
            med, _ = sw.time_launches(lambda: lib.hsp_spmm_run(ctx), stream, torch, 3, 10)
            lib.hsp_spmm_destroy(ctx)
            if best_h is None or med < best_h[1]:
                best_h = (name, med)
        if best_h:
            out["hipsparse"] = {"alg": best_h[0], "ms": best_h[1], "gflops": flops / best_h[1] / 1e6,
                                "pcsr_speedup": best_h[1] / kern_ms,
                                "max_abs_diff_vs_pcsr": float((Ch - Cd).abs().max().item())}
        del Ch, d_csr

    if not args.no_check or not args.no_cpu_baseline:
        import oracle

        # the oracle as it stands, on this machine's host cores
        if g.nnz * K <= 2.5e9:
            rows, sample = None, "full workload, best of 3"
            reps = 3
        else:
            n_s = max(1, int(g.n_rows * 2.5e9 / (g.nnz * K)))
            rows = np.sort(np.random.default_rng(0).choice(g.n_rows, n_s, replace=False)).astype(np.int64)
            sample, reps = f"{n_s} random rows of {g.n_rows}, 1 run", 1
        best = float("inf")
        for _ in range(reps):
            t0 = time.perf_counter()
            if rows is None:
                ref, bound = oracle.spmm(g_orig.rowptr, g_orig.colidx, g_orig.vals, B_orig)
            else:
                ref, bound = oracle.spmm_rows(g_orig.rowptr, g_orig.colidx, g_orig.vals, B_orig, rows)
            best = min(best, time.perf_counter() - t0)
        # row i of the original problem is row perm[i] of the relabelled one
        if rows is None:
            cpu_flops = flops
            got = Cd.cpu().numpy()
            if perm is not None:
                got = got[perm]
        else:
            cpu_flops = 2.0 * float(np.diff(g_orig.rowptr.astype(np.int64))[rows].sum()) * K
            sel_rows = rows if perm is None else perm[rows].astype(np.int64)
            got = Cd[torch.from_numpy(sel_rows).cuda()].cpu().numpy()
        ok, worst = oracle.within_tolerance(got, ref, bound)
        out["cpu_baseline"] = {"value": cpu_flops / best / 1e9, "unit": "GFLOP/s",
                               "cores": oracle.max_threads(), "kind": "oracle", "sample": sample}
        out["parity"] = {"ok": bool(ok), "worst_err_over_limit": worst}
        if not ok:
            print(json.dumps(out))
            print("bench.py: GPU result is outside tolerance", file=sys.stderr)
            return 1
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
