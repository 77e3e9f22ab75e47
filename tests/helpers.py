"""Small input builders shared by the tests (no method arithmetic)."""
import numpy as np


def random_csr(rng, n_rows, n_cols, density, empty_rows=(), full_rows=()):
    """Random pattern with sorted unique columns; values in +-[0.5, 1.5] (never zero)."""
    mask = rng.random((n_rows, n_cols)) < density
    for r in empty_rows:
        mask[r] = False
    for r in full_rows:
        mask[r] = True
    dense = np.where(mask, rng.uniform(0.5, 1.5, mask.shape) * rng.choice([-1.0, 1.0], mask.shape), 0.0)
    dense = dense.astype(np.float32)
    return dense_to_csr(dense) + (dense,)


def dense_to_csr(dense):
    n_rows = dense.shape[0]
    rowptr = np.zeros(n_rows + 1, dtype=np.int32)
    cols, vals = [], []
    for i in range(n_rows):
        nz = np.nonzero(dense[i])[0]
        cols.append(nz.astype(np.int32))
        vals.append(dense[i, nz].astype(np.float32))
        rowptr[i + 1] = rowptr[i] + nz.shape[0]
    colidx = np.concatenate(cols) if cols else np.zeros(0, np.int32)
    v = np.concatenate(vals) if vals else np.zeros(0, np.float32)
    return rowptr, colidx.astype(np.int32), v.astype(np.float32)
