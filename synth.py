"""Seeded synthetic SpMM inputs shaped like the paper's workload classes.

The paper evaluates on SNAP / DIMACS10 / OGB graphs (Section 6.1), which are not
available offline.  These generators stand in for them: Poisson-degree uniform
graphs, road-like geometric grids, R-MAT power-law graphs and stochastic block
models, i.e. the locality / degree-distribution classes the paper's introduction
and Section 6.1 describe.

This module holds no SpMM or PCSR arithmetic.  It only draws graphs, edge values
and dense operands from a seeded PCG64 stream, so the CPU oracle and the HIP path
can be fed identical inputs.  Everything returned is a numpy array:
``rowptr`` int32[n+1], ``colidx`` int32[nnz] (sorted, duplicate free per row),
``vals`` float32[nnz].
"""
from __future__ import annotations

import dataclasses
import os
import pathlib

import numpy as np

BASE_SEED = 0xC0FFEE


@dataclasses.dataclass
class Graph:
    name: str
    n_rows: int
    n_cols: int
    rowptr: np.ndarray
    colidx: np.ndarray
    vals: np.ndarray

    @property
    def nnz(self) -> int:
        return int(self.colidx.shape[0])

    def degrees(self) -> np.ndarray:
        return np.diff(self.rowptr.astype(np.int64))


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(seed))


def csr_from_edges(n_rows: int, n_cols: int, src: np.ndarray, dst: np.ndarray):
    """Sort (src, dst) pairs row-major, drop duplicates, return (rowptr, colidx)."""
    key = src.astype(np.int64) * np.int64(n_cols) + dst.astype(np.int64)
    key = np.unique(key)
    rows = key // np.int64(n_cols)
    colidx = (key - rows * np.int64(n_cols)).astype(np.int32)
    counts = np.bincount(rows, minlength=n_rows)
    rowptr = np.zeros(n_rows + 1, dtype=np.int64)
    np.cumsum(counts, out=rowptr[1:])
    assert rowptr[-1] < 2**31
    return rowptr.astype(np.int32), colidx


def values_inv_row_degree(rowptr: np.ndarray) -> np.ndarray:
    """a_ij = 1/deg(i): mean aggregation."""
    deg = np.diff(rowptr.astype(np.int64))
    return np.repeat(1.0 / np.maximum(deg, 1), deg).astype(np.float32)


def values_gcn(rowptr: np.ndarray, colidx: np.ndarray, n_cols: int) -> np.ndarray:
    """a_ij = 1/sqrt(max(1,outdeg_i) * max(1,indeg_j)); for a symmetric pattern this
    is the usual 1/sqrt(deg_i deg_j) GCN normalisation."""
    outdeg = np.diff(rowptr.astype(np.int64))
    indeg = np.bincount(colidx, minlength=n_cols)
    ri = np.repeat(np.maximum(outdeg, 1).astype(np.float64), outdeg)
    cj = np.maximum(indeg, 1).astype(np.float64)[colidx]
    return (1.0 / np.sqrt(ri * cj)).astype(np.float32)


def dense_operand(n: int, K: int, dist: str, seed: int) -> np.ndarray:
    """B (n x K, row-major fp32): 'uniform' = U(-1,1), 'normal' = N(0,1)."""
    rng = _rng(seed ^ 0xB0B)
    if dist == "uniform":
        B = rng.random((n, K), dtype=np.float32)
        B *= 2.0
        B -= 1.0
        return B
    if dist == "normal":
        return rng.standard_normal((n, K), dtype=np.float32)
    raise ValueError(dist)


# --------------------------------------------------------------------------- C1
def poisson_uniform(n: int = 4096, mean_deg: float = 8.0, seed: int = BASE_SEED + 1) -> Graph:
    """Each row draws Poisson(mean_deg) distinct uniformly random column ids; 1/deg values."""
    rng = _rng(seed)
    deg = np.minimum(rng.poisson(mean_deg, n), n)
    src = np.repeat(np.arange(n, dtype=np.int64), deg)
    dst = np.empty(src.shape[0], dtype=np.int64)
    pos = 0
    for i in range(n):
        d = int(deg[i])
        if d:
            dst[pos:pos + d] = rng.choice(n, size=d, replace=False)
            pos += d
    rowptr, colidx = csr_from_edges(n, n, src, dst)
    return Graph("poisson_uniform", n, n, rowptr, colidx, values_inv_row_degree(rowptr))


# --------------------------------------------------------------------------- C2
def road_grid(width: int = 2000, height: int = 1000, mean_draw: float = 2.1,
              seed: int = BASE_SEED + 2) -> Graph:
    """Road-like geometric graph: one node per cell of a width x height grid, ids in
    row-major grid order, each node displaced by a uniform jitter inside its cell.
    A node draws m ~ Poisson(mean_draw) and links to its m geometrically nearest
    nodes among the 8 surrounding cells; links are made undirected and deduplicated,
    so (mutual picks collapsing) the mean degree is about 3 for the default mean_draw and
    neighbours are near in id order.
    GCN-normalised values."""
    rng = _rng(seed)
    n = width * height
    ids = np.arange(n, dtype=np.int64)
    x = (ids % width).astype(np.int32)
    y = (ids // width).astype(np.int32)
    jx = rng.uniform(-0.4, 0.4, n).astype(np.float32)
    jy = rng.uniform(-0.4, 0.4, n).astype(np.float32)
    m = np.minimum(rng.poisson(mean_draw, n), 8).astype(np.int8)
    offs = [(-1, -1), (0, -1), (1, -1), (-1, 0), (1, 0), (-1, 1), (0, 1), (1, 1)]
    dist = np.empty((n, 8), dtype=np.float32)
    for k, (dx, dy) in enumerate(offs):
        nx, ny = x + dx, y + dy
        ok = (nx >= 0) & (nx < width) & (ny >= 0) & (ny < height)
        nid = np.where(ok, ny.astype(np.int64) * width + nx, 0)
        ddx = (dx + jx[nid]) - jx
        ddy = (dy + jy[nid]) - jy
        d2 = ddx * ddx + ddy * ddy
        dist[:, k] = np.where(ok, d2, np.float32(np.inf))
    order = np.argsort(dist, axis=1, kind="stable")
    srcs, dsts = [], []
    for r in range(8):
        k = order[:, r]
        take = (m > r) & np.isfinite(dist[ids, k])
        u = ids[take]
        kk = k[take]
        dxs = np.array([o[0] for o in offs], dtype=np.int64)[kk]
        dys = np.array([o[1] for o in offs], dtype=np.int64)[kk]
        v = (y[take].astype(np.int64) + dys) * width + (x[take].astype(np.int64) + dxs)
        srcs.append(u)
        dsts.append(v)
    u = np.concatenate(srcs)
    v = np.concatenate(dsts)
    src = np.concatenate([u, v])
    dst = np.concatenate([v, u])
    rowptr, colidx = csr_from_edges(n, n, src, dst)
    return Graph("road_grid", n, n, rowptr, colidx, values_gcn(rowptr, colidx, n))


# ---------------------------------------------------------------------- C3 / C5
def _rmat_edges(scale: int, n_edges: int, a: float, b: float, c: float,
                rng: np.random.Generator, chunk: int = 1 << 24):
    src = np.empty(n_edges, dtype=np.int64)
    dst = np.empty(n_edges, dtype=np.int64)
    ab, abc = np.float32(a + b), np.float32(a + b + c)
    a32 = np.float32(a)
    for lo in range(0, n_edges, chunk):
        hi = min(n_edges, lo + chunk)
        s = np.zeros(hi - lo, dtype=np.int64)
        d = np.zeros(hi - lo, dtype=np.int64)
        for _ in range(scale):
            r = rng.random(hi - lo, dtype=np.float32)
            sbit = r >= ab
            dbit = ((r >= a32) & (r < ab)) | (r >= abc)
            s = (s << 1) | sbit
            d = (d << 1) | dbit
        src[lo:hi] = s
        dst[lo:hi] = d
    return src, dst


def rmat(scale: int = 20, edge_factor: int = 16, a: float = 0.57, b: float = 0.19,
         c: float = 0.19, symmetric: bool = False, permute: bool = True,
         min_dmax: int = 0, seed: int = BASE_SEED + 3) -> Graph:
    """R-MAT graph with 2**scale nodes and edge_factor * 2**scale edge draws,
    self loops kept, duplicates removed.  ``permute`` relabels node ids with a random
    permutation (poor locality); ``symmetric`` adds the reverse of every edge.
    If ``min_dmax`` > 0 and the largest row is shorter, the busiest node receives
    extra undirected edges to targets drawn with probability proportional to current
    degree (Chung-Lu style) until its row is long enough.  GCN-normalised values."""
    rng = _rng(seed)
    n = 1 << scale
    src, dst = _rmat_edges(scale, edge_factor * n, a, b, c, rng)
    if permute:
        perm = rng.permutation(n).astype(np.int64)
        src, dst = perm[src], perm[dst]
    if symmetric:
        src, dst = np.concatenate([src, dst]), np.concatenate([dst, src])
    rowptr, colidx = csr_from_edges(n, n, src, dst)
    del src, dst
    if min_dmax:
        deg = np.diff(rowptr.astype(np.int64))
        hub = int(np.argmax(deg))
        if deg[hub] < min_dmax:
            p = deg.astype(np.float64)
            p /= p.sum()
            extra = rng.choice(n, size=int(2.5 * (min_dmax - deg[hub])) + 1024, p=p)
            rows = np.repeat(np.arange(n, dtype=np.int64), deg)
            hubs = np.full(extra.shape[0], hub, dtype=np.int64)
            s2 = np.concatenate([rows, hubs, extra])
            d2 = np.concatenate([colidx.astype(np.int64), extra, hubs])
            rowptr, colidx = csr_from_edges(n, n, s2, d2)
    name = f"rmat{scale}" + ("_sym" if symmetric else "") + ("_perm" if permute else "")
    return Graph(name, n, n, rowptr, colidx, values_gcn(rowptr, colidx, n))


# --------------------------------------------------------------------------- C4
def sbm(n: int = 250_000, n_blocks: int = 500, mean_deg: float = 50.0, p_intra: float = 0.9,
        shuffled: bool = False, seed: int = BASE_SEED + 4) -> Graph:
    """Stochastic block model: equal blocks of consecutive ids; each row draws
    Poisson(mean_deg) edges, each inside its own block with probability p_intra
    (uniform over the block) and uniform over all nodes otherwise; duplicates removed.
    ``shuffled`` applies a random relabelling to the same graph.  1/deg values."""
    rng = _rng(seed)
    bs = n // n_blocks
    assert bs * n_blocks == n
    deg = rng.poisson(mean_deg, n)
    src = np.repeat(np.arange(n, dtype=np.int64), deg)
    total = src.shape[0]
    intra = rng.random(total, dtype=np.float32) < np.float32(p_intra)
    dst = np.where(intra, (src // bs) * bs + rng.integers(0, bs, total),
                   rng.integers(0, n, total))
    if shuffled:
        perm = _rng(seed ^ 0x5EED).permutation(n).astype(np.int64)
        src, dst = perm[src], perm[dst]
    rowptr, colidx = csr_from_edges(n, n, src, dst)
    return Graph("sbm_shuffled" if shuffled else "sbm_clustered", n, n, rowptr, colidx,
                 values_inv_row_degree(rowptr))


# ------------------------------------------------------------------- workloads
# name -> (graph factory, B distribution, default K list).  "full" sizes follow the
# benchmark configurations; "small" sizes are what the CPU oracle finishes in seconds.
def workload(name: str, size: str = "full") -> Graph:
    """The named workload.  With SYNTH_CACHE_DIR set, generated graphs are kept there as
    .npz files and read back on later calls (the scale-22 R-MAT takes about half a minute to
    draw); the arrays are the same either way."""
    cache = os.environ.get("SYNTH_CACHE_DIR")
    if not cache:
        return _generate(name, size)
    path = pathlib.Path(cache) / f"{name}-{size}.npz"
    if path.exists():
        z = np.load(path, allow_pickle=False)
        return Graph(str(z["name"]), int(z["n_rows"]), int(z["n_cols"]), z["rowptr"], z["colidx"], z["vals"])
    g = _generate(name, size)
    path.parent.mkdir(parents=True, exist_ok=True)
    tmp = path.with_suffix(".tmp.npz")
    np.savez(tmp, name=g.name, n_rows=g.n_rows, n_cols=g.n_cols, rowptr=g.rowptr, colidx=g.colidx, vals=g.vals)
    tmp.replace(path)
    return g


def _generate(name: str, size: str) -> Graph:
    full = size == "full"
    if name == "poisson":
        return poisson_uniform(4096 if full else 1024)
    if name == "road":
        return road_grid(2000, 1000) if full else road_grid(211, 97)
    if name == "rmat20":
        return rmat(20 if full else 13, 16, permute=True, symmetric=False)
    if name == "sbm":
        return sbm(250_000, 500) if full else sbm(12_000, 24)
    if name == "sbm_shuffled":
        return sbm(250_000, 500, shuffled=True) if full else sbm(12_000, 24, shuffled=True)
    if name == "rmat22":
        if full:
            return rmat(22, 16, permute=False, symmetric=True, min_dmax=100_001,
                        seed=BASE_SEED + 5)
        return rmat(14, 16, permute=False, symmetric=True, seed=BASE_SEED + 5)
    if name in EXTRA:
        return EXTRA[name]()
    raise ValueError(name)


# Further inputs, used only to check the configuration rule on shapes it was not fitted to
# (Section 6.1 stresses the diversity of the evaluated matrices): other sizes, degrees and
# degree skews of the same four generator families.  They have one size.
EXTRA = {
    "x_poisson_d8": lambda: poisson_like(400_000, 8.0, BASE_SEED + 11),
    "x_poisson_d32": lambda: poisson_like(200_000, 32.0, BASE_SEED + 12),
    "x_poisson_d96": lambda: poisson_like(60_000, 96.0, BASE_SEED + 13),
    "x_road_small": lambda: road_grid(700, 500, seed=BASE_SEED + 14),
    "x_road_dense": lambda: road_grid(1200, 800, mean_draw=5.0, seed=BASE_SEED + 15),
    "x_rmat18": lambda: rmat(18, 16, permute=True, symmetric=True, seed=BASE_SEED + 16),
    "x_rmat19_ef8": lambda: rmat(19, 8, permute=False, symmetric=False, seed=BASE_SEED + 17),
    "x_rmat17_ef64": lambda: rmat(17, 64, permute=True, symmetric=False, seed=BASE_SEED + 18),
    "x_sbm_small_blocks": lambda: sbm(200_000, 4000, mean_deg=20.0, seed=BASE_SEED + 19),
    "x_sbm_big_blocks": lambda: sbm(120_000, 24, mean_deg=80.0, p_intra=0.7, seed=BASE_SEED + 20),
    "x_cliques": lambda: cliques(300_000, 24.0, 0.1, BASE_SEED + 21),
    "x_cliques_noisy": lambda: cliques(300_000, 24.0, 0.5, BASE_SEED + 22),
}

# A second such set, drawn after the rule had been revised with the first set in view, so
# that the score on it says something about inputs the rule has never been compared with.
EXTRA2 = {
    "y_poisson_d64": lambda: poisson_like(150_000, 64.0, BASE_SEED + 31),
    "y_poisson_d160": lambda: poisson_like(30_000, 160.0, BASE_SEED + 32),
    "y_poisson_d16": lambda: poisson_like(500_000, 16.0, BASE_SEED + 33),
    "y_sbm_shuffled_d72": lambda: sbm(90_000, 300, mean_deg=72.0, shuffled=True, seed=BASE_SEED + 34),
    "y_sbm_d72": lambda: sbm(90_000, 300, mean_deg=72.0, seed=BASE_SEED + 34),
    "y_sbm_d44_leaky": lambda: sbm(160_000, 400, mean_deg=44.0, p_intra=0.75, seed=BASE_SEED + 35),
    "y_rmat16_ef32": lambda: rmat(16, 32, permute=True, symmetric=True, seed=BASE_SEED + 36),
    "y_rmat21_ef4": lambda: rmat(21, 4, permute=False, symmetric=False, seed=BASE_SEED + 37),
    "y_road_wide": lambda: road_grid(3000, 300, mean_draw=3.0, seed=BASE_SEED + 38),
    "y_cliques_big": lambda: cliques(200_000, 48.0, 0.2, BASE_SEED + 39),
}
EXTRA.update(EXTRA2)

# A third set, drawn after the second revision of the rule (which had both earlier sets in view).
EXTRA3 = {
    "z_poisson_d48": lambda: poisson_like(220_000, 48.0, BASE_SEED + 41),
    "z_poisson_d120": lambda: poisson_like(50_000, 120.0, BASE_SEED + 42),
    "z_sbm_shuffled_d56": lambda: sbm(120_000, 240, mean_deg=56.0, shuffled=True, seed=BASE_SEED + 43),
    "z_sbm_d56_large": lambda: sbm(400_000, 800, mean_deg=56.0, seed=BASE_SEED + 44),
    "z_sbm_blocks2000": lambda: sbm(100_000, 50, mean_deg=60.0, p_intra=0.8, seed=BASE_SEED + 45),
    "z_rmat18_ef24": lambda: rmat(18, 24, permute=True, symmetric=False, seed=BASE_SEED + 46),
    "z_road_sparse": lambda: road_grid(1500, 900, mean_draw=1.6, seed=BASE_SEED + 47),
    "z_cliques_mid": lambda: cliques(250_000, 32.0, 0.3, BASE_SEED + 48),
}
EXTRA.update(EXTRA3)

# A fourth set, drawn after the third revision: the only one the final rule never saw.
EXTRA4 = {
    "w_poisson_d80": lambda: poisson_like(100_000, 80.0, BASE_SEED + 51),
    "w_poisson_d200": lambda: poisson_like(24_000, 200.0, BASE_SEED + 52),
    "w_sbm_shuffled_d44": lambda: sbm(300_000, 600, mean_deg=44.0, shuffled=True, seed=BASE_SEED + 53),
    "w_sbm_d64_mid": lambda: sbm(200_000, 500, mean_deg=64.0, seed=BASE_SEED + 54),
    "w_rmat19_ef12": lambda: rmat(19, 12, permute=True, symmetric=True, seed=BASE_SEED + 55),
    "w_rmat17_ef40": lambda: rmat(17, 40, permute=False, symmetric=False, seed=BASE_SEED + 56),
    "w_road_mid": lambda: road_grid(1000, 600, mean_draw=2.5, seed=BASE_SEED + 57),
    "w_cliques_40": lambda: cliques(150_000, 40.0, 0.15, BASE_SEED + 58),
}
EXTRA.update(EXTRA4)


def cliques(n: int, mean_size: float, noise: float, seed: int) -> Graph:
    """Co-authorship-like graph: consecutive ids are cut into cliques of 4 + Poisson(mean_size-4)
    nodes (every member linked to every member, itself included), and each row gets
    Poisson(noise * clique size) extra uniformly random columns.  Adjacent rows share almost all
    their columns, the low-padding regime of the paper's Table 1.  1/deg values."""
    rng = _rng(seed)
    sizes = 4 + rng.poisson(max(mean_size - 4.0, 0.0), int(n / mean_size * 1.2) + 8)
    ends = np.cumsum(sizes)
    k = int(np.searchsorted(ends, n))
    sizes = sizes[:k + 1].copy()
    sizes[k] -= ends[k] - n
    sizes = sizes[sizes > 0]
    start = np.repeat(np.cumsum(sizes) - sizes, sizes)      # first id of each node's clique
    size = np.repeat(sizes, sizes)
    src = np.repeat(np.arange(n, dtype=np.int64), size)
    within = np.arange(src.shape[0], dtype=np.int64) - np.repeat(np.cumsum(size) - size, size)
    dst = np.repeat(start, size) + within
    extra = rng.poisson(noise * size)
    src2 = np.repeat(np.arange(n, dtype=np.int64), extra)
    dst2 = rng.integers(0, n, src2.shape[0])
    rowptr, colidx = csr_from_edges(n, n, np.concatenate([src, src2]), np.concatenate([dst, dst2]))
    return Graph(f"cliques_{n}_{noise:g}", n, n, rowptr, colidx, values_inv_row_degree(rowptr))


def poisson_like(n: int, mean_deg: float, seed: int) -> Graph:
    """Poisson(mean_deg) uniformly random columns per row (duplicates dropped), vectorised for
    large n; 1/deg values."""
    rng = _rng(seed)
    deg = rng.poisson(mean_deg, n)
    src = np.repeat(np.arange(n, dtype=np.int64), deg)
    dst = rng.integers(0, n, src.shape[0])
    rowptr, colidx = csr_from_edges(n, n, src, dst)
    return Graph(f"poisson_like_{n}_{mean_deg:g}", n, n, rowptr, colidx, values_inv_row_degree(rowptr))


WORKLOADS = {
    "poisson": dict(B="uniform", K=[32]),
    "road": dict(B="normal", K=[128]),
    "rmat20": dict(B="normal", K=[64]),
    "sbm": dict(B="uniform", K=[256]),
    "sbm_shuffled": dict(B="uniform", K=[256]),
    "rmat22": dict(B="normal", K=[16, 32, 64, 128, 256, 512]),
}
WORKLOADS.update({name: dict(B="normal", K=[32, 128]) for name in EXTRA})
