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


def column_ordered_schedule(rowptr, colidx, trow, P):
    """The launch schedule PCSR_FLAG_COLUMN_ORDER documents, restated with numpy: items of
    panels that own several items sorted by (first column, item), the other items in index
    order, each list cut into 8 contiguous slices of equal work (vectors + 8 per item), XCD x
    running its slice of the first list and then its slice of the second.  Returns
    (sched int32[M, 4], xcd_bounds int32[9]); record = first vector, count, panel, slot."""
    M = trow.shape[0]
    per_panel = np.bincount(trow, minlength=P)
    is_long = per_panel[trow] > 1
    slot = np.full(M, -1, np.int64)
    slot[is_long] = np.arange(int(is_long.sum()))
    length = np.diff(rowptr.astype(np.int64))
    items = np.arange(M)
    longs = items[is_long]
    longs = longs[np.lexsort((longs, colidx[rowptr[longs]]))]
    shorts = items[~is_long]

    def slices(lst):
        cum = np.concatenate([[0], np.cumsum(length[lst] + 8)])
        return [0] + [int(np.searchsorted(cum, cum[-1] * x // 8, side="left")) for x in range(1, 8)] + [len(lst)]

    lb, sb = slices(longs), slices(shorts)
    order, xb = [], [0]
    for x in range(8):
        order += [longs[lb[x]:lb[x + 1]], shorts[sb[x]:sb[x + 1]]]
        xb.append(xb[-1] + (lb[x + 1] - lb[x]) + (sb[x + 1] - sb[x]))
    order = np.concatenate(order) if M else np.zeros(0, np.int64)
    sched = np.stack([rowptr[order], length[order], trow[order], slot[order]], axis=1).astype(np.int32)
    return sched, np.asarray(xb, np.int32)


def near_diagonal_share(rowptr, colidx, width=512):
    """Share of the nonzeros with |column - row| < width (the library's own 17th feature)."""
    rows = np.repeat(np.arange(rowptr.shape[0] - 1, dtype=np.int64), np.diff(rowptr.astype(np.int64)))
    return float(np.mean(np.abs(colidx.astype(np.int64) - rows) < width)) if colidx.size else 0.0
