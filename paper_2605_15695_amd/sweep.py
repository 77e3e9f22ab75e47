"""Exhaustive configuration sweep on one MI355X: every PCSR format tuple (V, S, SG) times
every kernel launch shape (lanes_per_row, vec, rep, waves_per_wg, XCD remap) for one
workload and width K, timed with device events, beside hipSPARSE SpMM on the same
arrays.  One JSON line per timing goes to --out; the recorded sweeps are the data the
library's selection rule (pcsr_select) is distilled from, in the role the paper gives
the training set of its SpMM-decider (Section 5.2).

Outputs of all tuples are compared on the GPU with the first tuple's output (max
|difference| relative to max |C|) as a consistency diagnostic; parity against the
CPU oracle is the job of the tests and of bench.py.

    python -m paper_2605_15695_amd.sweep --workload rmat20 --K 64 --out sweeps/rmat20.jsonl
"""
from __future__ import annotations

import argparse
import ctypes
import itertools
import json
import pathlib
import statistics
import sys
import time

import numpy as np

from . import binding as pc
import synth

HBM_PEAK_GBS = 8000.0
HIPSPARSE_ALGS = {"default": 0, "csr_alg1": 4, "csr_alg2": 6, "csr_alg3": 12}


def algorithmic_bytes(g, K: int) -> int:
    n_refcols = int(np.unique(g.colidx).shape[0])
    return g.nnz * 8 + (g.n_rows + 1) * 4 + n_refcols * K * 4 + g.n_rows * K * 4


def kernel_shapes(K: int, quick: bool):
    """(lanes_per_row, vec, rep) with a tile of lanes*vec*rep columns that covers K in one
    or two grid.y slices without a fully idle repeat."""
    shapes = []
    for vec in (4, 2, 1):
        if K % vec:
            continue
        # quick: only the widest vector load, except for K <= 32, where narrower loads
        # (fewer rows per wavefront) win on some inputs
        widest = 4 if K % 4 == 0 else (2 if K % 2 == 0 else 1)
        if quick and K > 32 and vec != widest:
            # ... and the two 64-column slices built from narrow loads
            if 64 * 8 >= K and K % 2 == 0 and vec == 2:
                shapes.append((32, 2, 1))
            elif 64 * 8 >= K and vec == 1:
                shapes.append((64, 1, 1))
            continue
        for lpr in (4, 8, 16, 32, 64):
            for rep in (1, 2, 4):
                tile = lpr * vec * rep
                if tile * 8 < K or tile < 32 and tile < K:
                    continue                      # too many slices: A re-read too often
                if lpr * vec * (rep - 1) >= K:
                    continue                      # a whole repeat would be idle
                if lpr * vec >= 2 * K and lpr > 4:
                    continue                      # half of the lanes idle
                shapes.append((lpr, vec, rep))
    return shapes


def time_launches(fn, stream, torch, warmup: int, reps: int):
    for _ in range(warmup):
        fn()
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
           for _ in range(reps)]
    torch.cuda.synchronize()
    for a, b in evs:
        a.record(stream)
        fn()
        b.record(stream)
    torch.cuda.synchronize()
    ts = [a.elapsed_time(b) for a, b in evs]
    return statistics.median(ts), min(ts)


def _baseline_lib():
    path = pathlib.Path(__file__).resolve().parent / "libpcsr_baseline.so"
    lib = ctypes.CDLL(str(path))
    i64, i32, vp = ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p
    lib.hsp_spmm_create.argtypes = [i64, i64, i64, vp, vp, vp, vp, vp, i32, i32, vp, ctypes.POINTER(vp)]
    lib.hsp_spmm_run.argtypes = [vp]
    lib.hsp_spmm_destroy.argtypes = [vp]
    lib.hsp_spmm_buffer_bytes.argtypes = [vp]
    lib.hsp_spmm_buffer_bytes.restype = i64
    lib.alg1_spmm.argtypes = [i64, vp, vp, vp, vp, vp, i32, i32, vp]
    return lib


def main(argv=None) -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", required=True)
    ap.add_argument("--size", default="full")
    ap.add_argument("--K", type=int, nargs="*", default=None)
    ap.add_argument("--out", required=True)
    ap.add_argument("--quick", action="store_true", help="widest vector only (all widths for K <= 32), waves in {2,4}")
    ap.add_argument("--reps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--formats", default="all",
                    help="all | comma list of V:S:SG[:col_window[:flags]], e.g. 1:0:0,1:1:64,1:1:64:0:64 "
                         "(flags: PCSR_FLAG_* bits given to pcsr_build, 64 = column-ordered schedule)")
    ap.add_argument("--no-hipsparse", action="store_true")
    ap.add_argument("--reorder", nargs="?", const="cluster", default=None, choices=["cluster", "degree"],
                    help="sweep the matrix after one of the library's relabellings: 'cluster' (pcsr_reorder) "
                         "or 'degree' (pcsr_reorder_by_degree)")
    ap.add_argument("--shapes", default=None,
                    help="explicit launch shapes instead of the enumeration: comma list of "
                         "lanes:vec:rep:waves:items_per_group")
    args = ap.parse_args(argv)

    import torch

    if not torch.cuda.is_available():
        print("sweep: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    stream = torch.cuda.current_stream()
    out = open(args.out, "a")

    def emit(rec):
        out.write(json.dumps(rec) + "\n")
        out.flush()

    t0 = time.time()
    g = synth.workload(args.workload, args.size)
    spec = synth.WORKLOADS[args.workload]
    Ks = args.K or spec["K"]
    print(f"[sweep] {args.workload}-{args.size}: n={g.n_rows} nnz={g.nnz} generated in {time.time()-t0:.1f}s",
          flush=True)
    if args.reorder:
        t0 = time.time()
        if args.reorder == "degree":
            perm, ncl = pc.pcsr_reorder_by_degree(g.n_rows, g.rowptr, g.colidx), 0
        else:
            perm, ncl = pc.pcsr_reorder(g.n_rows, g.rowptr, g.colidx)
        rp, ci, va = pc.pcsr_permute_csr(g.n_rows, g.rowptr, g.colidx, g.vals, perm)
        g = synth.Graph(g.name + "_reordered", g.n_rows, g.n_cols, rp, ci, va)
        print(f"[sweep] reordered into {ncl} clusters in {time.time()-t0:.2f}s", flush=True)
    feats = pc.pcsr_features(g.n_rows, g.n_cols, g.rowptr, g.colidx)
    emit({"kind": "graph", "workload": args.workload, "size": args.size, "n": g.n_rows, "nnz": g.nnz,
          "features": dict(zip(pc.FEATURE_NAMES, map(float, feats)))})

    if args.formats == "all":
        sg_eq3 = 0
        co = pc.PCSR_FLAG_COLUMN_ORDER
        formats = [(1, 0, 0), (2, 0, 0), (1, 1, sg_eq3), (2, 1, sg_eq3), (1, 1, 256), (1, 1, 1024), (2, 1, 1024),
                   (1, 1, 32, 0, co), (1, 1, 64, 0, co), (2, 1, 64, 0, co), (1, 0, 0, 512), (1, 0, 0, 1024)]
    else:
        formats = [tuple(int(x) for x in f.split(":")) for f in args.formats.split(",")]
    formats = [f + (0,) * (5 - len(f)) for f in formats]             # (V, S, SG, col_window, build flags)

    d_rowptr = torch.from_numpy(g.rowptr).cuda()
    d_colidx = torch.from_numpy(g.colidx).cuda()
    d_vals = torch.from_numpy(g.vals).cuda()

    handles = {}
    for fmt in formats:
        V, S, SG, CW, FL = fmt
        t0 = time.time()
        handles[fmt] = pc.pcsr_build(g.n_rows, g.n_cols, g.rowptr, g.colidx, g.vals,
                                     pc.make_params(V=V, S=S, SG=SG, col_window=CW,
                                                    flags=pc.PCSR_FLAG_NO_VALIDATE | FL))
        hit = pc.pcsr_window_stats(handles[fmt])["hit_fraction"]
        print(f"[sweep] built V={V} S={S} SG={SG} CW={CW} flags={FL} (window hit {hit:.3f}) in "
              f"{time.time()-t0:.2f}s", flush=True)

    for K in Ks:
        B = synth.dense_operand(g.n_cols, K, spec["B"], 2)
        Bd = torch.from_numpy(B).cuda()
        del B
        Cd = torch.empty((g.n_rows, K), dtype=torch.float32, device="cuda")
        Cref = None
        flops = 2.0 * g.nnz * K
        bytes_min = algorithmic_bytes(g, K)
        base = {"workload": args.workload + (f"+reorder({args.reorder})" if args.reorder else ""), "size": args.size, "K": K, "nnz": g.nnz, "n": g.n_rows,
                "bytes_min": bytes_min}
        best = (float("inf"), None)
        for fmt in formats:
            V, S, SG, CW, FL = fmt
            h = handles[fmt]
            waves_list = (2, 4) if args.quick else (1, 2, 4, 8)
            ipg_list = (1, 2, 4) if not S else (1,)
            if CW:
                if pc.pcsr_window_stats(h)["hit_fraction"] < 0.05:
                    continue                      # no block has a window worth staging
                waves_list, ipg_list = (8, 16), (1,)
            if args.shapes:
                combos = [(tuple(int(x) for x in sh.split(":")[:3]), int(sh.split(":")[3]), 1,
                           int(sh.split(":")[4])) for sh in args.shapes.split(",")]
            else:
                combos = itertools.product(kernel_shapes(K, args.quick), waves_list, (1, 0), ipg_list)
            for (lpr, vec, rep), waves, remap, ipg in combos:
                if args.quick and not remap:
                    continue
                if ipg > 1 and S:
                    continue
                pc.pcsr_set_kernel_params(h, lpr, vec, rep, waves, ipg,
                                          0 if remap else pc.PCSR_FLAG_NO_XCD_REMAP)
                try:
                    q = pc.pcsr_query_launch(h, K)
                except pc.PcsrError:
                    continue
                Cd.fill_(float("nan"))
                med, mn = time_launches(lambda: pc.pcsr_spmm(h, Bd, Cd, K, stream), stream, torch,
                                        args.warmup, args.reps)
                if Cref is None:
                    Cref = Cd.clone()
                    scale = float(Cref.abs().max().item()) or 1.0
                    dev = 0.0
                else:
                    dev = float((Cd - Cref).abs().max().item()) / scale
                rec = dict(base, kind="pcsr", V=V, S=S, SG=SG, col_window=CW, build_flags=FL, lanes_per_row=lpr, vec=vec, rep=rep,
                           waves_per_wg=waves, items_per_group=ipg, xcd_remap=remap, grid_x=q["grid_x"], grid_y=q["grid_y"],
                           ms_median=med, ms_min=mn, gflops=flops / med / 1e6,
                           roofline_frac=bytes_min / (med * 1e-3) / 1e9 / HBM_PEAK_GBS, max_rel_dev=dev)
                emit(rec)
                if med < best[0]:
                    best = (med, rec)
            print(f"[sweep] K={K} V={V} S={S} SG={SG} CW={CW} flags={FL} done; best so far {best[0]:.4f} ms",
                  flush=True)

        hs_best = (float("inf"), None)
        if not args.no_hipsparse:
            lib = _baseline_lib()
            for name, alg in HIPSPARSE_ALGS.items():
                ctx = ctypes.c_void_p()
                t0 = time.time()
                rc = lib.hsp_spmm_create(g.n_rows, g.n_cols, g.nnz, d_rowptr.data_ptr(), d_colidx.data_ptr(),
                                         d_vals.data_ptr(), Bd.data_ptr(), Cd.data_ptr(), K, alg,
                                         stream.cuda_stream, ctypes.byref(ctx))
                torch.cuda.synchronize()
                prep = time.time() - t0
                if rc != 0:
                    emit(dict(base, kind="hipsparse", alg=name, error=rc))
                    continue
                Cd.fill_(float("nan"))
                med, mn = time_launches(lambda: lib.hsp_spmm_run(ctx), stream, torch, args.warmup, args.reps)
                dev = float((Cd - Cref).abs().max().item()) / scale if Cref is not None else None
                rec = dict(base, kind="hipsparse", alg=name, ms_median=med, ms_min=mn,
                           gflops=flops / med / 1e6, preprocess_s=prep,
                           buffer_bytes=int(lib.hsp_spmm_buffer_bytes(ctx)),
                           roofline_frac=bytes_min / (med * 1e-3) / 1e9 / HBM_PEAK_GBS, max_rel_dev=dev)
                emit(rec)
                lib.hsp_spmm_destroy(ctx)
                if med < hs_best[0]:
                    hs_best = (med, rec)
                print(f"[sweep] K={K} hipsparse {name}: {med:.4f} ms", flush=True)
        # the library's own pick (pcsr_select) for this input, timed like the others
        sel = pc.pcsr_select(feats, K)
        hsel = pc.pcsr_build(g.n_rows, g.n_cols, g.rowptr, g.colidx, g.vals, sel)
        qs = pc.pcsr_query_launch(hsel, K)
        Cd.fill_(float("nan"))
        med, mn = time_launches(lambda: pc.pcsr_spmm(hsel, Bd, Cd, K, stream), stream, torch,
                                args.warmup, args.reps)
        dev = float((Cd - Cref).abs().max().item()) / scale if Cref is not None else None
        # time the sweep's best tuple again, back to back with the pick, so that the ratio
        # compares two measurements taken under the same conditions
        best_again = None
        if best[1]:
            b = best[1]
            hb = handles[(b["V"], b["S"], b["SG"], b["col_window"], b.get("build_flags", 0))]
            pc.pcsr_set_kernel_params(hb, b["lanes_per_row"], b["vec"], b["rep"], b["waves_per_wg"],
                                      b["items_per_group"], 0 if b["xcd_remap"] else pc.PCSR_FLAG_NO_XCD_REMAP)
            best_again, _ = time_launches(lambda: pc.pcsr_spmm(hb, Bd, Cd, K, stream), stream, torch,
                                          args.warmup, args.reps)
        selrec = dict(base, kind="selected", V=sel.V, S=sel.S, SG=sel.SG, **qs, ms_median=med, ms_min=mn,
                      gflops=flops / med / 1e6, roofline_frac=bytes_min / (med * 1e-3) / 1e9 / HBM_PEAK_GBS,
                      max_rel_dev=dev, best_retimed_ms=best_again,
                      vs_sweep_best=(best_again / med) if best_again else None)
        emit(selrec)
        hsel.close()
        print(f"[sweep] K={K} SELECTED V={sel.V} S={sel.S} SG={sel.SG} lpr={qs['lanes_per_row']} vec={qs['vec']} "
              f"rep={qs['rep']} gy={qs['grid_y']} waves={qs['waves_per_wg']}: {med:.4f} ms "
              f"({100 * (best_again or best[0]) / med:.1f}% of the sweep's best tuple re-timed)", flush=True)
        if not args.no_hipsparse:
            # plain CSR baseline: the basic scheme of Algorithm 1 (one wavefront per row, one column per lane)
            lib = _baseline_lib()
            a1_best = None
            for W in (1, 2, 4, 8):
                Cd.fill_(float("nan"))
                med, mn = time_launches(
                    lambda: lib.alg1_spmm(g.n_rows, d_rowptr.data_ptr(), d_colidx.data_ptr(), d_vals.data_ptr(),
                                          Bd.data_ptr(), Cd.data_ptr(), K, W, stream.cuda_stream),
                    stream, torch, args.warmup, min(args.reps, 5))
                dev = float((Cd - Cref).abs().max().item()) / scale if Cref is not None else None
                emit(dict(base, kind="alg1", W=W, ms_median=med, ms_min=mn, gflops=flops / med / 1e6,
                          max_rel_dev=dev))
                a1_best = med if a1_best is None else min(a1_best, med)
            print(f"[sweep] K={K} Algorithm 1 baseline: {a1_best:.4f} ms", flush=True)
        summary = dict(base, kind="summary", selected=selrec, pcsr_best=best[1], hipsparse_best=hs_best[1],
                       speedup_vs_hipsparse=(hs_best[0] / best[0]) if hs_best[1] and best[1] else None)
        emit(summary)
        b = best[1]
        print(f"[sweep] K={K} BEST {b['ms_median']:.4f} ms {b['gflops']:.0f} GFLOP/s roofline {b['roofline_frac']:.3f} "
              f"V={b['V']} S={b['S']} SG={b['SG']} CW={b['col_window']} flags={b.get('build_flags', 0)} lpr={b['lanes_per_row']} vec={b['vec']} rep={b['rep']} "
              f"waves={b['waves_per_wg']} ipg={b['items_per_group']} remap={b['xcd_remap']} | hipsparse best "
              f"{hs_best[0]:.4f} ms ({hs_best[1]['alg'] if hs_best[1] else '-'})", flush=True)
        del Bd, Cd, Cref
        torch.cuda.empty_cache()
    for h in handles.values():
        h.close()
    out.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
