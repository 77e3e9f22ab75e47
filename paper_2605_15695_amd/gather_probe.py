"""Measures the random-row gather ceiling of the GPU: rows of 64 B .. 1 KiB pulled from a
dense fp32 matrix of a given footprint at uniformly random indices, with a kernel that
does nothing else.  SpMM on scattered inputs cannot gather faster than this, whatever
its format or launch shape; the figures go beside the kernels' cache-level gather rate.

    python -m paper_2605_15695_amd.gather_probe
"""
from __future__ import annotations

import ctypes
import json
import pathlib
import statistics
import sys


def main(argv=None) -> int:
    import argparse

    import torch

    ap = argparse.ArgumentParser()
    ap.add_argument("--footprints-mb", type=float, nargs="*", default=[16, 256, 1024, 8192])
    args = ap.parse_args(argv)

    if not torch.cuda.is_available():
        print("gather_probe: no GPU visible", file=sys.stderr)
        return 2
    lib = ctypes.CDLL(str(pathlib.Path(__file__).resolve().parent / "libpcsr_baseline.so"))
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
    lib.probe_gather.argtypes = [vp, i32, vp, i64, vp, i32, vp]
    stream = torch.cuda.current_stream()
    blocks = 256 * 32
    out = torch.empty(blocks * 256, dtype=torch.float32, device="cuda")
    n_idx = 1 << 25
    results = []
    for footprint_mb in args.footprints_mb:
        for row_floats in (16, 32, 64, 128, 256):
            n_rows = int(footprint_mb * (1 << 20)) // (row_floats * 4)
            B = torch.ones((n_rows, row_floats), dtype=torch.float32, device="cuda")
            idx = torch.randint(0, n_rows, (n_idx,), dtype=torch.int32, device="cuda")

            def run():
                rc = lib.probe_gather(B.data_ptr(), row_floats, idx.data_ptr(), n_idx, out.data_ptr(),
                                      blocks, stream.cuda_stream)
                assert rc == 0, rc

            for _ in range(2):
                run()
            evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
                   for _ in range(5)]
            torch.cuda.synchronize()
            for a, b in evs:
                a.record(stream)
                run()
                b.record(stream)
            torch.cuda.synchronize()
            ms = statistics.median(a.elapsed_time(b) for a, b in evs)
            rec = {"footprint_MB": footprint_mb, "row_bytes": row_floats * 4, "gathers": n_idx, "ms": ms,
                   "gather_TBps": n_idx * row_floats * 4 / (ms * 1e-3) / 1e12,
                   "rows_per_us": n_idx / (ms * 1e3)}
            results.append(rec)
            print(json.dumps(rec), flush=True)
            del B, idx
            torch.cuda.empty_cache()
    return 0


if __name__ == "__main__":
    sys.exit(main())
