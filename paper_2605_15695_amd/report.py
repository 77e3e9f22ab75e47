"""Turns sweep records (JSON lines written by paper_2605_15695_amd.sweep) into a markdown
table: per workload and K the best PCSR tuple, its time, GFLOP/s (2*nnz*K), fraction of
the HBM minimum-traffic roofline, cache-level gather rate, the library's own pick and
hipSPARSE's best algorithm, then the geometric-mean speed-up over hipSPARSE.

    python -m paper_2605_15695_amd.report sweeps/*.jsonl > sweep_summary.md
"""
from __future__ import annotations

import json
import math
import sys


def main(argv=None) -> int:
    paths = (argv or sys.argv[1:])
    recs = []
    for p in paths:
        with open(p) as f:
            recs += [json.loads(line) for line in f if line.strip()]
    keys = sorted({(r["workload"], r["K"]) for r in recs if r.get("kind") == "pcsr"})
    print("| workload | K | n | nnz | best tuple (V,S,SG / lanes,vec,rep,waves,items) | ms | GFLOP/s | roofline frac "
          "| gather TB/s | selected ms (% of best) | hipSPARSE best ms | speed-up | Alg. 1 ms |")
    print("|---|---|---|---|---|---|---|---|---|---|---|---|---|")
    ratios, sel_ratios, rnd_ratios, at_half = [], [], [], 0
    for w, K in keys:
        rs = [r for r in recs if r.get("kind") == "pcsr" and r["workload"] == w and r["K"] == K]
        b = min(rs, key=lambda r: r["ms_median"])
        hs = [r for r in recs if r.get("kind") == "hipsparse" and r["workload"] == w and r["K"] == K
              and "ms_median" in r]
        sel = [r for r in recs if r.get("kind") == "selected" and r["workload"] == w and r["K"] == K]
        h = min(hs, key=lambda r: r["ms_median"]) if hs else None
        a1 = [r["ms_median"] for r in recs if r.get("kind") == "alg1" and r["workload"] == w and r["K"] == K]
        a1_txt = f"{min(a1):.4f}" if a1 else "-"
        s = min(sel, key=lambda r: r["ms_median"]) if sel else None
        tup = (f'{b["V"]},{b["S"]},{b["SG"]} / {b["lanes_per_row"]},{b["vec"]},{b["rep"]},'
               f'{b["waves_per_wg"]},{b.get("items_per_group", 1)}')
        gather = b["nnz"] * K * 4 / (b["ms_median"] * 1e-3) / 1e12
        # ratio against the best tuple re-timed next to the pick when the sweep recorded it
        sref = (s.get("best_retimed_ms") or b["ms_median"]) if s else None
        sel_txt = f'{s["ms_median"]:.4f} ({100 * sref / s["ms_median"]:.0f}%)' if s else "-"
        hs_txt = f'{h["ms_median"]:.4f} ({h["alg"]})' if h else "-"
        sp = h["ms_median"] / b["ms_median"] if h else float("nan")
        if h:
            ratios.append(sp)
        if s:
            sel_ratios.append(sref / s["ms_median"])
        # expected normalised performance of a tuple drawn at random from the swept set (the
        # "rnd" column of the paper's Table 5)
        rnd_ratios.append(sum(b["ms_median"] / r["ms_median"] for r in rs) / len(rs))
        at_half += b["roofline_frac"] >= 0.5
        print(f'| {w} | {K} | {b["n"]} | {b["nnz"]} | {tup} | {b["ms_median"]:.4f} | {b["gflops"]:.0f} | '
              f'{b["roofline_frac"]:.3f} | {gather:.2f} | {sel_txt} | {hs_txt} | {sp:.2f}x | {a1_txt} |')
    if ratios:
        gm = math.exp(sum(map(math.log, ratios)) / len(ratios))
        print(f"\nGeometric mean of hipSPARSE best / PCSR best over {len(ratios)} inputs: **{gm:.2f}x**; "
              f"inputs at >= 50 % of the HBM minimum-traffic roofline: {at_half} of {len(keys)}.")
    if sel_ratios:
        gm = math.exp(sum(map(math.log, sel_ratios)) / len(sel_ratios))
        print(f"Library pick (pcsr_select) vs sweep best, geometric mean over {len(sel_ratios)} inputs: "
              f"**{100 * gm:.1f} %** of the best tuple's speed.")
    if rnd_ratios:
        print(f"A tuple drawn at random from the swept set reaches on average "
              f"**{100 * sum(rnd_ratios) / len(rnd_ratios):.1f} %** of the best tuple's speed "
              f"(per input: {100 * min(rnd_ratios):.0f}-{100 * max(rnd_ratios):.0f} %).")
    return 0


if __name__ == "__main__":
    sys.exit(main())
