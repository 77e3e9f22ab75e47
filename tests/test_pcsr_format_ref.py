"""Pins for the numpy PCSR-format reference and the scalar formulas (Section 4.2,
Eqs. (1)-(4), Tables 2 and 3)."""
import pathlib

import numpy as np
import pytest

from oracle import pcsr_format as pf
import synth
from tests.helpers import random_csr

GOLDEN = pathlib.Path(__file__).parent / "golden"


def test_gap_matches_table2():
    rows = [l.split() for l in (GOLDEN / "table2_gap.txt").read_text().splitlines()
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 14
    for dim, F, gap in rows:
        assert pf.mac_job_gap(int(dim), int(F), omega=32) == int(gap)


def test_gap_is_remainder_complement():
    # dim = 80, F = 2, omega = 32: the residual warp does 80 mod 64 = 16 of 64 jobs
    assert pf.mac_job_gap(80, 2, 32) == 48
    assert pf.mac_job_gap(16, 1, 32) == 0 + (16 - 16)  # dim < F*omega: tn = dim = tr
    assert pf.mac_job_gap(48, 1, 32) == 32 - 16


def test_padding_ratio_range_from_table1():
    for line in (GOLDEN / "table1_padding.txt").read_text().splitlines():
        if not line.strip() or line.startswith("#"):
            continue
        V, pr = line.split()
        assert 0.0 <= float(pr) / 100 <= 1 - 1 / int(V)
    assert pf.padding_ratio(100, 100, 1) == 0.0
    assert pf.padding_ratio(100, 50, 2) == 0.0
    assert pf.padding_ratio(100, 100, 2) == 0.5


def test_hand_worked_panel_example():
    # rows: 0 -> (c0: a=1, c2: b=2); 1 -> (c0: e=5, c3: f=6); 2 -> (c1: 7); 3 -> empty.
    # a and e share column 0, so with V = 2 they pack into one vector (Section 4.2 examples).
    rowptr = np.array([0, 2, 4, 5, 5], np.int32)
    colidx = np.array([0, 2, 0, 3, 1], np.int32)
    vals = np.array([1, 2, 5, 6, 7], np.float32)
    pc = pf.pcsr_ref(4, rowptr, colidx, vals, V=2, S=False)
    assert pc["P"] == 2 and pc["M"] == 2 and pc["nnz_v"] == 4
    assert pc["rowptr"].tolist() == [0, 3, 4]
    assert pc["colidx"].tolist() == [0, 2, 3, 1]
    assert pc["val"].tolist() == [1, 5, 2, 0, 0, 6, 7, 0]
    assert pc["trow"].size == 0
    assert pf.padding_ratio(5, 4, 2) == 1 - 5 / 8
    # balancing with SG = 2: panel 0 (3 vectors) -> items of 2 and 1; panel 1 -> one item
    ps = pf.pcsr_ref(4, rowptr, colidx, vals, V=2, S=True, SG=2)
    assert ps["rowptr"].tolist() == [0, 2, 3, 4]
    assert ps["trow"].tolist() == [0, 0, 1]
    assert ps["colidx"].tolist() == pc["colidx"].tolist() and ps["val"].tolist() == pc["val"].tolist()
    assert pf.split_ratio(ps["M"], ps["P"]) == 1.5


@pytest.mark.parametrize("S", [False, True])
def test_v1_is_csr(S):
    g = synth.workload("poisson", "small")
    pc = pf.pcsr_ref(g.n_rows, g.rowptr, g.colidx, g.vals, V=1, S=S, SG=1 << 20)
    assert np.array_equal(pc["rowptr"], g.rowptr)
    assert np.array_equal(pc["colidx"], g.colidx)
    assert np.array_equal(pc["val"].view(np.uint32), g.vals.view(np.uint32))
    assert pc["trow"].size == (g.n_rows if S else 0)
    if S:
        assert np.array_equal(pc["trow"], np.arange(g.n_rows))


@pytest.mark.parametrize("n", [1, 2, 9, 40])
@pytest.mark.parametrize("V", [1, 2])
@pytest.mark.parametrize("S,SG", [(False, 0), (True, 0), (True, 3)])
def test_round_trip_to_coo(n, V, S, SG):
    rng = np.random.default_rng(n * 10 + V)
    rowptr, colidx, vals, dense = random_csr(rng, n, n + 3, 0.3)
    pc = pf.pcsr_ref(n, rowptr, colidx, vals, V, S, SG, omega=4)
    r, c, v = pf.pcsr_to_coo(n, pc)
    back = np.zeros_like(dense)
    nz = v != 0
    assert np.all(back[r[nz], c[nz]] == 0)        # no (row, col) stored twice
    back[r[nz], c[nz]] = v[nz]
    assert np.array_equal(back, dense)
    assert pc["P"] == -(-n // V)
    nnz = colidx.size
    assert nnz <= pc["nnz_v"] * V and pc["nnz_v"] <= nnz
    assert 0 <= pf.padding_ratio(nnz, pc["nnz_v"], V) <= 1 - 1 / V + 1e-12
    # every vector holds at least one nonzero; padding slots are +0.0f
    vv = pc["val"].reshape(-1, V)
    assert np.all((vv != 0).any(axis=1))
    assert np.all(pc["val"].view(np.uint32)[pc["val"] == 0] == 0)


def test_columns_ascending_inside_panels_and_split_invariants():
    g = synth.workload("rmat20", "small")
    for V in (1, 2):
        base = pf.pcsr_ref(g.n_rows, g.rowptr, g.colidx, g.vals, V, False)
        for p in range(base["P"]):
            seg = base["colidx"][base["rowptr"][p]:base["rowptr"][p + 1]]
            assert np.all(np.diff(seg) > 0)
        for omega in (32, 64):
            pc = pf.pcsr_ref(g.n_rows, g.rowptr, g.colidx, g.vals, V, True, 0, omega)
            SG, M, P = pc["SG"], pc["M"], pc["P"]
            assert SG % omega == 0 and SG > 0
            lens = np.diff(pc["rowptr"])
            assert lens.min() >= 0 and lens.max() <= SG
            assert pc["rowptr"][0] == 0 and pc["rowptr"][-1] == pc["nnz_v"]
            assert np.all(np.diff(pc["trow"]) >= 0)
            assert np.array_equal(np.unique(pc["trow"]), np.arange(P))
            plen = np.diff(base["rowptr"].astype(np.int64))
            assert M == int(np.maximum(1, -(-plen // SG)).sum())
            assert pf.split_ratio(M, P) >= 1.0
            # all items of a panel but the last are full
            last_of_panel = np.r_[pc["trow"][1:] != pc["trow"][:-1], True]
            assert np.all(lens[~last_of_panel] == SG)
            # per-panel totals unchanged
            assert np.array_equal(np.bincount(pc["trow"], weights=lens, minlength=P), plen)
            assert np.array_equal(pc["colidx"], base["colidx"])


def test_split_closed_forms():
    # all rows within SG: nothing changes
    g = synth.workload("road", "small")
    pc = pf.pcsr_ref(g.n_rows, g.rowptr, g.colidx, g.vals, 1, True, 0, 64)
    assert pc["SG"] == 64 and pc["M"] == pc["P"] and np.array_equal(pc["rowptr"], g.rowptr)
    # one row of length L in an otherwise empty matrix, explicit SG
    n, L, SG = 10, 1000, 64
    rowptr = np.zeros(n + 1, np.int32)
    rowptr[4:] = L
    colidx = np.arange(L, dtype=np.int32)
    pc = pf.pcsr_ref(n, rowptr, colidx, np.ones(L, np.float32), 1, True, SG)
    assert pc["M"] == (n - 1) + -(-L // SG) == 9 + 16
    assert np.diff(pc["rowptr"]).tolist() == [0, 0, 0] + [64] * 15 + [40] + [0] * 6
    assert pc["trow"].tolist() == [0, 1, 2] + [3] * 16 + [4, 5, 6, 7, 8, 9]
    # Eq. (3) on that matrix: one non-empty panel of 1000 vectors -> SG = ceil(1000/32)*32
    assert pf.pcsr_ref(n, rowptr, colidx, np.ones(L, np.float32), 1, True, 0, 32)["SG"] == 1024
    assert pf.split_granularity(np.array([0, 0, 0]), 32) == 32


def test_split_granularity_values():
    # 10 panels, 7 non-empty, 70*7 vectors: average 70 -> ceil(70/32)*32 = 96; omega 64 -> 128
    lens = np.array([70, 0, 70, 70, 0, 70, 70, 0, 70, 70])
    rp = np.r_[0, np.cumsum(lens)]
    assert pf.split_granularity(rp, 32) == 96
    assert pf.split_granularity(rp, 64) == 128
    # average exactly 64 stays 64; 64 + a little rounds up
    assert pf.split_granularity(np.array([0, 64, 128]), 64) == 64
    assert pf.split_granularity(np.array([0, 64, 129]), 64) == 128


def test_padding_closed_forms():
    n = 12
    rowptr = np.arange(n + 1, dtype=np.int32)
    diag = pf.pcsr_ref(n, rowptr, np.arange(n, dtype=np.int32), np.ones(n, np.float32), 2, False)
    assert diag["nnz_v"] == n and pf.padding_ratio(n, diag["nnz_v"], 2) == 0.5
    # identical row pairs: every vector is full
    cols = np.array([1, 4, 7], np.int32)
    rowptr = np.arange(0, 3 * n + 1, 3, dtype=np.int32)
    colidx = np.tile(cols, n)
    vals = np.arange(1, 3 * n + 1, dtype=np.float32)
    pc = pf.pcsr_ref(n, rowptr, colidx, vals, 2, False)
    assert pc["nnz_v"] == 3 * n // 2 and pf.padding_ratio(3 * n, pc["nnz_v"], 2) == 0.0
    assert pc["val"][:6].tolist() == [1, 4, 2, 5, 3, 6]
    # odd n: the last panel's second slot is padding
    pc = pf.pcsr_ref(3, np.array([0, 1, 2, 3], np.int32), np.array([0, 0, 2], np.int32),
                     np.array([1, 2, 3], np.float32), 2, False)
    assert pc["P"] == 2 and pc["colidx"].tolist() == [0, 2] and pc["val"].tolist() == [1, 2, 3, 0]


def test_features_hand_example():
    # 4 x 6: row0 cols {0, 5}; row1 cols {0}; row2 empty; row3 cols {1, 2, 3}
    rowptr = np.array([0, 2, 3, 3, 6], np.int32)
    colidx = np.array([0, 5, 0, 1, 2, 3], np.int32)
    f = dict(zip(pf.FEATURE_NAMES, pf.features(4, 6, rowptr, colidx, omega=2)))
    assert f["n"] == 4 and f["n_hat"] == 3 and f["nnz"] == 6
    assert f["delta"] == 0.75 and f["d"] == 1.5 and f["d_hat"] == 2.0 and f["d_max"] == 3
    deg = np.array([2, 1, 0, 3.0])
    assert f["CV"] == pytest.approx(np.sqrt(((deg - 1.5) ** 2).mean()) / 1.5)
    assert f["CV_hat"] == pytest.approx(np.sqrt(((deg[[0, 1, 3]] - 2) ** 2).mean()) / 2)
    assert f["rho"] == 6 / 24
    assert f["b"] == (5 + 0 + 0 + 2) / 4 and f["b_max"] == 5
    assert f["PR_1"] == 0.0
    # V=2: panel0 cols {0,5} (col 0 shared) -> 2 vectors; panel1 cols {1,2,3} -> 3 vectors
    assert f["PR_2"] == pytest.approx(1 - 6 / (5 * 2))
    # V=1, omega=2: d_hat = 2 -> SG = 2 -> items 1,1,1,2 -> SR = 5/4
    assert f["SR_1"] == 5 / 4
    # V=2: 5 vectors over 2 panels: SG = ceil(2.5/2)*2 = 4 -> items 1,1 -> SR = 1
    assert f["SR_2"] == 1.0
