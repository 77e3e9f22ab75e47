"""GNN integration of the PCSR SpMM (the paper embeds its kernel in GCN / GIN training,
Section 6.5): an autograd function whose forward is C = A*B and whose backward is
dB = A^T * dC, both through pcsr_spmm, plus minimal GCN / GIN layers built on it.

torch supplies tensors, streams, the dense weight GEMMs and the optimiser; every sparse
product runs in the library's kernels.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as pc


class PcsrOperator:
    """A fixed sparse matrix A ready for forward (A*B) and backward (A^T*dC) products.

    ``symmetric=True`` states that A equals its transpose (GCN-normalised undirected
    graphs), so one handle serves both directions.  Otherwise the transpose is built once
    with pcsr_transpose_csr.  Parameters are picked by pcsr_select for width ``K_hint``
    unless ``params`` is given.
    """

    def __init__(self, n_rows, n_cols, rowptr, colidx, vals, symmetric=False, K_hint=64, params=None):
        self.n_rows, self.n_cols = int(n_rows), int(n_cols)

        def build(nr, nc, rp, ci, va):
            p = params
            if p is None:
                p = pc.pcsr_select(pc.pcsr_features(nr, nc, rp, ci), K_hint)
                # launch shape stays on auto so one handle serves every layer width
                p.lanes_per_row = p.vec = p.rep = 0
            else:
                p = pc.make_params(**{f: getattr(params, f) for f, _ in pc.pcsr_params_t._fields_
                                      if f != "reserved"})
            return pc.pcsr_build(nr, nc, rp, ci, va, p)

        self.fwd = build(self.n_rows, self.n_cols, rowptr, colidx, vals)
        if symmetric:
            if n_rows != n_cols:
                raise ValueError("a symmetric operator must be square")
            self.bwd = self.fwd
        else:
            trp, tci, tva = pc.pcsr_transpose_csr(self.n_rows, self.n_cols, rowptr, colidx, vals)
            self.bwd = build(self.n_cols, self.n_rows, trp, tci, tva)

    def apply(self, B: torch.Tensor) -> torch.Tensor:
        return SpMMFunction.apply(B, self)

    __call__ = apply

    def _run(self, handle, n_out, X: torch.Tensor) -> torch.Tensor:
        if X.dtype != torch.float32 or not X.is_cuda or X.dim() != 2:
            raise ValueError("operand must be a 2-D float32 CUDA tensor")
        X = X.contiguous()
        K = X.shape[1]
        out = torch.empty((n_out, K), dtype=torch.float32, device=X.device)
        pc.pcsr_spmm(handle, X, out, K, torch.cuda.current_stream(X.device))
        return out


class SpMMFunction(torch.autograd.Function):
    @staticmethod
    def forward(ctx, B, op: PcsrOperator):
        ctx.op = op
        return op._run(op.fwd, op.n_rows, B)

    @staticmethod
    def backward(ctx, dC):
        op = ctx.op
        return op._run(op.bwd, op.n_cols, dC), None


class GCNLayer(torch.nn.Module):
    """H' = A_hat (H W) + b, the graph convolution of Kipf & Welling with a pre-normalised
    adjacency operator; the dense product comes first when it narrows the features."""

    def __init__(self, op: PcsrOperator, d_in: int, d_out: int, bias: bool = True):
        super().__init__()
        self.op = op
        self.lin = torch.nn.Linear(d_in, d_out, bias=False)
        self.bias = torch.nn.Parameter(torch.zeros(d_out)) if bias else None

    def forward(self, H):
        if self.lin.in_features >= self.lin.out_features:
            out = self.op(self.lin(H))
        else:
            out = self.lin(self.op(H))
        return out if self.bias is None else out + self.bias


class GINLayer(torch.nn.Module):
    """H' = MLP((1 + eps) H + A H), sum aggregation (Xu et al.)."""

    def __init__(self, op: PcsrOperator, d_in: int, d_out: int, eps: float = 0.0):
        super().__init__()
        self.op = op
        self.eps = torch.nn.Parameter(torch.tensor(float(eps)))
        self.mlp = torch.nn.Sequential(torch.nn.Linear(d_in, d_out), torch.nn.ReLU(),
                                       torch.nn.Linear(d_out, d_out))

    def forward(self, H):
        return self.mlp((1.0 + self.eps) * H + self.op(H))


def make_model(kind: str, op: PcsrOperator, d_in: int, hidden: int, d_out: int, n_layers: int = 5):
    """n_layers graph layers with ReLU between them (the paper trains 5-layer GCN / GIN
    models with hidden sizes 32, 64, 128 and 16 input / output features)."""
    dims = [d_in] + [hidden] * (n_layers - 1) + [d_out]
    layer = {"gcn": GCNLayer, "gin": GINLayer}[kind]
    mods = []
    for i in range(n_layers):
        mods.append(layer(op, dims[i], dims[i + 1]))
        if i + 1 < n_layers:
            mods.append(torch.nn.ReLU())
    return torch.nn.Sequential(*mods)
