"""Times the one-off set-up calls on one MI355X: pcsr_build with the host builder, with the
GPU builder from host CSR arrays (upload included) and from CSR arrays already in device
memory, for several format tuples, and pcsr_features on the host and on the device.
The paper amortises these over the training iterations (Section 5.1) and never times them.

    python -m paper_2605_15695_amd.build_bench --workload rmat22
"""
from __future__ import annotations

import argparse
import json
import sys
import time


def main(argv=None) -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="rmat22")
    ap.add_argument("--size", default="full")
    ap.add_argument("--reps", type=int, default=3)
    args = ap.parse_args(argv)

    import torch

    import synth
    from . import binding as pc

    if not torch.cuda.is_available():
        print("build_bench: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    g = synth.workload(args.workload, args.size)
    d = [torch.from_numpy(x).cuda() for x in (g.rowptr, g.colidx, g.vals)]
    torch.cuda.synchronize()
    co = pc.PCSR_FLAG_COLUMN_ORDER
    out = {"workload": f"{args.workload}-{args.size}", "n": g.n_rows, "nnz": g.nnz, "build_ms": [], "features_ms": {}}
    for V, S, SG, fl in [(1, 0, 0, 0), (2, 0, 0, 0), (1, 1, 1024, 0), (1, 1, 64, co), (2, 1, 64, co)]:
        row = {"V": V, "S": S, "SG": SG, "column_order": bool(fl)}
        for mode in ("host", "gpu_from_host_csr", "gpu_from_device_csr"):
            best = float("inf")
            for _ in range(args.reps):
                t0 = time.perf_counter()
                if mode == "host":
                    h = pc.pcsr_build(g.n_rows, g.n_cols, g.rowptr, g.colidx, g.vals,
                                      pc.make_params(V=V, S=S, SG=SG, flags=fl))
                elif mode == "gpu_from_host_csr":
                    h = pc.pcsr_build(g.n_rows, g.n_cols, g.rowptr, g.colidx, g.vals,
                                      pc.make_params(V=V, S=S, SG=SG, flags=fl | pc.PCSR_FLAG_GPU_BUILD))
                else:
                    h = pc.pcsr_build(g.n_rows, g.n_cols, *d, pc.make_params(V=V, S=S, SG=SG, flags=fl))
                torch.cuda.synchronize()
                best = min(best, time.perf_counter() - t0)
                h.close()
            row[mode] = round(best * 1e3, 2)
        out["build_ms"].append(row)
        print(f"[build_bench] {row}", flush=True)
    for mode in ("host", "device"):
        best = float("inf")
        for _ in range(args.reps):
            t0 = time.perf_counter()
            if mode == "host":
                pc.pcsr_features(g.n_rows, g.n_cols, g.rowptr, g.colidx)
            else:
                pc.pcsr_features(g.n_rows, g.n_cols, d[0], d[1])
            best = min(best, time.perf_counter() - t0)
        out["features_ms"][mode] = round(best * 1e3, 2)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
