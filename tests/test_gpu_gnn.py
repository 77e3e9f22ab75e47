"""Autograd wrapper and GNN layers on the GPU: forward against the CPU oracle, backward
(dB = A^T dC) against the oracle applied to the transposed CSR."""
import numpy as np
import pytest

import oracle
import paper_2605_15695_amd as pc
import synth

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def _transpose_scipy(g):
    import scipy.sparse as sp
    At = sp.csr_matrix((g.vals, g.colidx, g.rowptr), shape=(g.n_rows, g.n_cols)).T.tocsr()
    At.sort_indices()
    return At.indptr.astype(np.int32), At.indices.astype(np.int32), At.data.astype(np.float32)


@pytest.mark.parametrize("name,symmetric", [("rmat20", False), ("road", True), ("sbm", False)])
def test_forward_and_backward_match_oracle(name, symmetric):
    from paper_2605_15695_amd.gnn import PcsrOperator

    g = synth.workload(name, "small")
    K = 32
    op = PcsrOperator(g.n_rows, g.n_cols, g.rowptr, g.colidx, g.vals, symmetric=symmetric, K_hint=K)
    B = synth.dense_operand(g.n_cols, K, "normal", 3)
    dC = synth.dense_operand(g.n_rows, K, "normal", 4)
    Bd = torch.from_numpy(B).cuda().requires_grad_(True)
    C = op(Bd)
    C.backward(torch.from_numpy(dC).cuda())
    ref, bound = oracle.spmm(g.rowptr, g.colidx, g.vals, B)
    ok, worst = oracle.within_tolerance(C.detach().cpu().numpy(), ref, bound)
    assert ok, worst
    trp, tci, tva = _transpose_scipy(g)
    gref, gbound = oracle.spmm(trp, tci, tva, dC)
    ok, worst = oracle.within_tolerance(Bd.grad.cpu().numpy(), gref, gbound)
    assert ok, worst


def test_transpose_export_matches_scipy():
    g = synth.workload("rmat20", "small")
    trp, tci, tva = pc.pcsr_transpose_csr(g.n_rows, g.n_cols, g.rowptr, g.colidx, g.vals)
    rp, ci, va = _transpose_scipy(g)
    assert np.array_equal(trp, rp) and np.array_equal(tci, ci)
    assert np.array_equal(tva.view(np.uint32), va.view(np.uint32))


@pytest.mark.parametrize("kind", ["gcn", "gin"])
def test_five_layer_model_trains_one_step(kind):
    """Section 6.5 shape: 5 layers, 16 input / output features, hidden 32.  The sparse
    products inside must agree with a dense-adjacency reference of the same model."""
    from paper_2605_15695_amd.gnn import PcsrOperator, make_model

    g = synth.workload("poisson", "small")
    op = PcsrOperator(g.n_rows, g.n_cols, g.rowptr, g.colidx, g.vals, symmetric=False, K_hint=32)
    torch.manual_seed(0)
    model = make_model(kind, op, 16, 32, 16).cuda()
    X = torch.from_numpy(synth.dense_operand(g.n_rows, 16, "normal", 9)).cuda()
    out = model(X)
    loss = out.square().mean()
    loss.backward()
    grads = [p.grad.clone() for p in model.parameters()]

    # dense reference: same parameters, A as a dense fp64 matrix
    import scipy.sparse as sp
    A = torch.from_numpy(sp.csr_matrix((g.vals, g.colidx, g.rowptr), shape=(g.n_rows, g.n_cols))
                         .toarray().astype(np.float64))

    class DenseOp:
        def __call__(self, H):
            return A @ H

    torch.manual_seed(0)
    ref_model = make_model(kind, DenseOp(), 16, 32, 16).double()
    ref_model.load_state_dict({k: v.double().cpu() for k, v in model.state_dict().items()})
    ref_out = ref_model(X.double().cpu())
    ref_loss = ref_out.square().mean()
    ref_loss.backward()
    assert torch.allclose(out.double().cpu(), ref_out, rtol=1e-3, atol=1e-4)
    for gd, p in zip(grads, ref_model.parameters()):
        assert torch.allclose(gd.double().cpu(), p.grad, rtol=5e-3, atol=1e-5)
