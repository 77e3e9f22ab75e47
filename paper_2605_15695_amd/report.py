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


def records_table(recs, top: int = 6) -> None:
    """Compact view of the recorded sweep: per input, the best median time of every format tuple
    (over launch shapes) and of every launch shape (over formats), relative to the input's best."""
    keys = sorted({(r["workload"], r["K"]) for r in recs if r.get("kind") == "pcsr"})
    fmt_name = lambda r: (f'V{r["V"]} S{r["S"]} SG{r["SG"]}' + (" col-order" if r.get("build_flags", 0) & 64 else "")
                          + (f' window{r["col_window"]}' if r.get("col_window") else ""))
    shape_name = lambda r: (f'{r["lanes_per_row"]}x{r["vec"]}x{r["rep"]} w{r["waves_per_wg"]}'
                            + (f' i{r["items_per_group"]}' if r.get("items_per_group", 1) > 1 else ""))
    for w, K in keys:
        rs = [r for r in recs if r.get("kind") == "pcsr" and r["workload"] == w and r["K"] == K]
        best = min(r["ms_median"] for r in rs)
        print(f"\n### {w}, K={K}: best {best:.4f} ms over {len(rs)} timed tuples\n")
        for title, name in (("format (V, S, SG)", fmt_name), ("launch shape (lanes x vec x rep, waves)", shape_name)):
            by = {}
            for r in rs:
                k = name(r)
                if k not in by or r["ms_median"] < by[k]["ms_median"]:
                    by[k] = r
            rows = sorted(by.items(), key=lambda kv: kv[1]["ms_median"])[:top]
            print(f"| {title} | best ms | % of input's best | reached with |")
            print("|---|---|---|---|")
            for k, r in rows:
                other = shape_name(r) if name is fmt_name else fmt_name(r)
                print(f'| {k} | {r["ms_median"]:.4f} | {100 * best / r["ms_median"]:.0f} | {other} |')
            print()


def main(argv=None) -> int:
    paths = list(argv or sys.argv[1:])
    records = "--records" in paths
    if records:
        paths.remove("--records")
    top = 6
    for p in list(paths):
        if p.startswith("--top="):
            top = int(p.split("=", 1)[1])
            paths.remove(p)
    recs = []
    for p in paths:
        with open(p) as f:
            recs += [json.loads(line) for line in f if line.strip()]
    if records:
        records_table(recs, top)
        return 0
    keys = sorted({(r["workload"], r["K"]) for r in recs if r.get("kind") == "pcsr"})
    print("| workload | K | n | nnz | best tuple (V,S,SG[c = column-ordered] / lanes,vec,rep,waves,items) | ms | GFLOP/s | roofline frac "
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
        tup = (f'{b["V"]},{b["S"]},{b["SG"]}{"c" if b.get("build_flags", 0) & 64 else ""} / '
               f'{b["lanes_per_row"]},{b["vec"]},{b["rep"]},{b["waves_per_wg"]},{b.get("items_per_group", 1)}')
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
