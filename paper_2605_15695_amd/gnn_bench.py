"""Times one GCN / GIN training step (forward, backward, Adam update) with every sparse
product going through pcsr_spmm, beside the same model on torch.sparse (rocSPARSE CSR).
Shape follows the paper's Section 6.5: 5 layers, 16 input and output features, hidden
size 32 / 64 / 128.  Synthetic graphs and random features stand in for the OGB graphs.

    python -m paper_2605_15695_amd.gnn_bench --workload road --model gcn --hidden 64
"""
from __future__ import annotations

import argparse
import json
import statistics
import sys
import time


def main(argv=None) -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="road")
    ap.add_argument("--size", default="full")
    ap.add_argument("--model", default="gcn", choices=["gcn", "gin"])
    ap.add_argument("--hidden", type=int, default=64)
    ap.add_argument("--layers", type=int, default=5)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-torch-sparse", action="store_true")
    args = ap.parse_args(argv)

    import torch

    import synth
    from .gnn import PcsrOperator, make_model

    if not torch.cuda.is_available():
        print("gnn_bench: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    g = synth.workload(args.workload, args.size)
    symmetric = args.workload in ("road", "rmat22")
    X = torch.from_numpy(synth.dense_operand(g.n_rows, 16, "normal", 5)).cuda()
    Y = torch.from_numpy(synth.dense_operand(g.n_rows, 16, "normal", 6)).cuda()

    def run(op, label):
        torch.manual_seed(0)
        model = make_model(args.model, op, 16, args.hidden, 16, args.layers).cuda()
        opt = torch.optim.Adam(model.parameters(), lr=1e-3)

        def step():
            opt.zero_grad(set_to_none=True)
            loss = torch.nn.functional.mse_loss(model(X), Y)
            loss.backward()
            opt.step()
            return loss

        for _ in range(args.warmup):
            step()
        torch.cuda.synchronize()
        ts = []
        for _ in range(args.steps):
            t0 = time.perf_counter()
            loss = step()
            torch.cuda.synchronize()
            ts.append((time.perf_counter() - t0) * 1e3)
        return {"impl": label, "ms_per_step_median": statistics.median(ts), "ms_per_step_min": min(ts),
                "final_loss": float(loss)}

    t0 = time.time()
    op = PcsrOperator(g.n_rows, g.n_cols, g.rowptr, g.colidx, g.vals, symmetric=symmetric, K_hint=args.hidden)
    build_s = time.time() - t0
    res = [run(op, "pcsr")]
    if not args.no_torch_sparse:
        A = torch.sparse_csr_tensor(torch.from_numpy(g.rowptr).cuda(), torch.from_numpy(g.colidx).cuda(),
                                    torch.from_numpy(g.vals).cuda(), size=(g.n_rows, g.n_cols))

        class TorchSparseOp:
            def __call__(self, H):
                return torch.sparse.mm(A, H)

        try:
            res.append(run(TorchSparseOp(), "torch.sparse"))
        except Exception as e:  # noqa: BLE001
            res.append({"impl": "torch.sparse", "error": repr(e)[:200]})
    out = {"workload": f"{args.workload}-{args.size}", "n": g.n_rows, "nnz": g.nnz, "model": args.model,
           "layers": args.layers, "hidden": args.hidden, "operator_build_s": build_s, "results": res}
    if len(res) == 2 and "ms_per_step_median" in res[1]:
        out["speedup_vs_torch_sparse"] = res[1]["ms_per_step_median"] / res[0]["ms_per_step_median"]
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
