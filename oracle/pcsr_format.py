"""CPU reference of the Parameterized CSR (PCSR) format and of the scalar quantities
the paper defines on it.  TEST INFRASTRUCTURE: only tests/, the smoke check and the
bench's cpu_baseline leg may import this; the product path never does.

What is followed (paper sections, own words):

* Section 4.2, "Data Representation" and "PCSR Generation": A is cut into row panels
  of V consecutive rows; inside a panel every column that holds at least one nonzero
  becomes one V x 1 "nonzero vector" with one column index and V value slots, missing
  slots padded with zero, values flattened V per vector.  rowPtr delimits the vectors
  of each work item.  With balancing (S) rowPtr is rewritten so that no work item
  exceeds SG vectors and TRow records, per work item, the panel whose C rows receive
  its partial sums.  Without balancing TRow is empty.
* Eq. (1): MAC-job gap.   Eq. (2): padding ratio PR_V.   Eq. (3): split granularity SG.
  Eq. (4): split ratio SR.   Table 3: the feature list.

Readings where the text is silent (each also listed in the design notes):
  - vectors inside a panel are ordered by ascending column; slot k of a vector
    belongs to row panel*V + k; rows past the end of A are padding (+0.0f).
  - the average panel length in Eq. (3) is nnz_V / (number of non-empty panels), the
    V-analogue of the hatted degree of Table 3; SG = ceil(that / omega) * omega, which
    in exact arithmetic is ceildiv(nnz_V, nonempty * omega) * omega; SG = omega when
    there is no vector at all.
  - a panel with l vectors becomes max(1, ceil(l / SG)) consecutive work items, all
    full except the last; an empty panel keeps one empty item (so SR >= 1 as Eq. (4)
    requires).
  - SR = (number of work items) / (number of panels).
  - Eq. (1) printed literally gives gap = tn when dim is a multiple of F*omega, but
    Table 2 prints 0 there, so gap = 0 when the remainder is 0.
  - CV uses the population standard deviation; the bandwidth of a row is last minus
    first column (0 for rows with fewer than two nonzeros); b averages over all rows.
"""
from __future__ import annotations

import numpy as np


def ceildiv(a, b):
    return -(-a // b)


# ----------------------------------------------------------------- Section 4.2
def vectorized_blocking(n_rows, rowptr, colidx, vals, V):
    """Panels of V rows -> (rowPtr int32[P+1], colIdx int32[nnz_V], val fp32[nnz_V*V])."""
    rowptr = np.asarray(rowptr, dtype=np.int64)
    colidx = np.asarray(colidx, dtype=np.int64)
    vals = np.asarray(vals, dtype=np.float32)
    P = ceildiv(n_rows, V)
    row_of = np.repeat(np.arange(n_rows, dtype=np.int64), np.diff(rowptr))
    panel_of = row_of // V
    slot_of = row_of % V
    # one vector per distinct (panel, column), ascending column inside a panel
    n_cols_key = int(colidx.max()) + 1 if colidx.size else 1
    key = panel_of * n_cols_key + colidx
    uniq, vec_of = np.unique(key, return_inverse=True)
    nnz_v = uniq.shape[0]
    vec_panel = uniq // n_cols_key
    vec_col = uniq - vec_panel * n_cols_key
    val = np.zeros(nnz_v * V, dtype=np.float32)          # +0.0f padding
    val[vec_of * V + slot_of] = vals
    new_rowptr = np.zeros(P + 1, dtype=np.int64)
    np.cumsum(np.bincount(vec_panel, minlength=P), out=new_rowptr[1:])
    return new_rowptr.astype(np.int32), vec_col.astype(np.int32), val


def split_granularity(panel_rowptr, omega):
    """Eq. (3) with the hatted average taken over non-empty panels."""
    lengths = np.diff(np.asarray(panel_rowptr, dtype=np.int64))
    nnz_v = int(lengths.sum())
    nonempty = int(np.count_nonzero(lengths))
    if nnz_v == 0:
        return int(omega)
    return int(ceildiv(nnz_v, nonempty * omega) * omega)


def workload_split(panel_rowptr, SG):
    """Rewrite rowPtr so every work item has at most SG vectors; emit TRow.
    Returns (rowPtr int32[M+1], TRow int32[M])."""
    panel_rowptr = np.asarray(panel_rowptr, dtype=np.int64)
    P = panel_rowptr.shape[0] - 1
    lengths = np.diff(panel_rowptr)
    items = np.maximum(1, ceildiv(lengths, SG))
    M = int(items.sum())
    trow = np.repeat(np.arange(P, dtype=np.int64), items)
    first_item = np.zeros(P, dtype=np.int64)
    np.cumsum(items[:-1], out=first_item[1:])
    within = np.arange(M, dtype=np.int64) - first_item[trow]
    new_rowptr = np.empty(M + 1, dtype=np.int64)
    new_rowptr[:M] = panel_rowptr[trow] + within * SG
    new_rowptr[M] = panel_rowptr[P]
    return new_rowptr.astype(np.int32), trow.astype(np.int32)


def pcsr_ref(n_rows, rowptr, colidx, vals, V, S, SG=0, omega=64):
    """Full PCSR under (V, S).  SG = 0 means Eq. (3) with the given omega.
    Returns dict(P, M, nnz_v, V, SG, rowptr, colidx, val, trow)."""
    prow, pcol, pval = vectorized_blocking(n_rows, rowptr, colidx, vals, V)
    P = prow.shape[0] - 1
    sg = int(SG) if SG else split_granularity(prow, omega)
    if S:
        new_rowptr, trow = workload_split(prow, sg)
    else:
        new_rowptr, trow = prow, np.zeros(0, dtype=np.int32)
    return dict(P=P, M=new_rowptr.shape[0] - 1, nnz_v=pcol.shape[0], V=V, SG=sg,
                rowptr=new_rowptr, colidx=pcol, val=pval, trow=trow)


def pcsr_to_coo(n_rows, pc):
    """Expand PCSR back to (row, col, val) triples including padding slots of rows < n_rows."""
    V = pc["V"]
    M = pc["M"]
    lengths = np.diff(pc["rowptr"].astype(np.int64))
    item_of_vec = np.repeat(np.arange(M, dtype=np.int64), lengths)
    panel_of_vec = pc["trow"].astype(np.int64)[item_of_vec] if pc["trow"].size else item_of_vec
    rows = (panel_of_vec[:, None] * V + np.arange(V)[None, :]).ravel()
    cols = np.repeat(pc["colidx"].astype(np.int64), V)
    vals = pc["val"]
    keep = rows < n_rows
    return rows[keep], cols[keep], vals[keep]


# ------------------------------------------------------------------ Eqs. (1)-(4)
def mac_job_gap(dim, F, omega=32):
    tn = min(dim, F * omega)
    tr = dim % (F * omega)
    return 0 if tr == 0 else tn - tr


def padding_ratio(nnz, nnz_v, V):
    return 0.0 if nnz_v == 0 else 1.0 - nnz / (nnz_v * V)


def split_ratio(M, P):
    return 1.0 if P == 0 else M / P


# ---------------------------------------------------------------------- Table 3
FEATURE_NAMES = ("n", "n_hat", "nnz", "delta", "d", "d_hat", "d_max", "CV", "CV_hat",
                 "SR_1", "SR_2", "rho", "b", "b_max", "PR_1", "PR_2")


def features(n_rows, n_cols, rowptr, colidx, omega=64):
    rowptr = np.asarray(rowptr, dtype=np.int64)
    colidx = np.asarray(colidx, dtype=np.int64)
    deg = np.diff(rowptr).astype(np.float64)
    nnz = int(rowptr[-1]) if rowptr.size else 0
    nonempty = deg > 0
    n_hat = int(np.count_nonzero(nonempty))
    d = nnz / n_rows if n_rows else 0.0
    d_hat = nnz / n_hat if n_hat else 0.0
    cv = float(np.std(deg) / d) if d > 0 else 0.0
    cv_hat = float(np.std(deg[nonempty]) / d_hat) if n_hat else 0.0
    bw = np.zeros(n_rows, dtype=np.float64)
    idx = np.nonzero(nonempty)[0]
    bw[idx] = colidx[rowptr[idx + 1] - 1] - colidx[rowptr[idx]]
    ones = np.ones(nnz, dtype=np.float32)
    out = {}
    for V in (1, 2):
        pc = pcsr_ref(n_rows, rowptr, colidx, ones, V, True, 0, omega)
        out[f"SR_{V}"] = split_ratio(pc["M"], pc["P"])
        out[f"PR_{V}"] = padding_ratio(nnz, pc["nnz_v"], V)
    vals = [n_rows, n_hat, nnz, n_hat / n_rows if n_rows else 0.0, d, d_hat,
            float(deg.max()) if n_rows else 0.0, cv, cv_hat, out["SR_1"], out["SR_2"],
            nnz / (n_rows * n_cols) if n_rows and n_cols else 0.0,
            float(bw.mean()) if n_rows else 0.0, float(bw.max()) if n_rows else 0.0,
            out["PR_1"], out["PR_2"]]
    return np.array(vals, dtype=np.float64)
