"""CPU-side checks of the C-ABI library: exported symbols, host PCSR generation bit-exact
against the numpy format reference, feature extraction, error paths.  No GPU calls."""
import ctypes
import pathlib
import re

import numpy as np
import pytest

import paper_2605_15695_amd as pc
from oracle import pcsr_format as pf
import synth
from paper_2605_15695_amd import binding
from tests.helpers import column_ordered_schedule, near_diagonal_share, random_csr

ROOT = pathlib.Path(__file__).resolve().parent.parent
HOST = pc.PCSR_FLAG_HOST_ONLY


def _bits(a):
    return a.view(np.uint32) if a.dtype == np.float32 else a


def _assert_same(e, r):
    for k in ("P", "M", "nnz_v", "V", "SG"):
        assert e[k] == r[k], k
    for k in ("rowptr", "colidx", "val", "trow"):
        assert e[k].dtype == r[k].dtype and np.array_equal(_bits(e[k]), _bits(r[k])), k


def test_every_declared_symbol_is_exported():
    header = (ROOT / "include" / "pcsr.h").read_text()
    names = set(re.findall(r"^(?:int|int32_t|int64_t|const char \*)\s*(pcsr_[a-z_]+)\(", header, re.M))
    assert len(names) >= 11
    assert {"pcsr_build", "pcsr_spmm", "pcsr_free"} <= names
    lib = ctypes.CDLL(str(binding.LIB_PATH))
    for n in sorted(names):
        assert hasattr(lib, n), n


@pytest.mark.parametrize("name", ["poisson", "road", "rmat20", "sbm", "sbm_shuffled", "rmat22"])
@pytest.mark.parametrize("V", [1, 2])
@pytest.mark.parametrize("S,SG,omega", [(0, 0, 0), (1, 0, 0), (1, 0, 32), (1, 5, 0)])
def test_host_generation_bit_exact(name, V, S, SG, omega):
    g = synth.workload(name, "small")
    h = pc.pcsr_build(g.n_rows, g.n_cols, g.rowptr, g.colidx, g.vals,
                      pc.make_params(V=V, S=S, SG=SG, omega=omega, flags=HOST))
    _assert_same(pc.pcsr_export(h), pf.pcsr_ref(g.n_rows, g.rowptr, g.colidx, g.vals, V, S, SG, omega or 64))
    h.close()


@pytest.mark.parametrize("n", [0, 1, 2, 3, 17])
@pytest.mark.parametrize("V", [1, 2])
@pytest.mark.parametrize("S", [0, 1])
def test_host_generation_tiny_and_degenerate(n, V, S):
    rng = np.random.default_rng(n + 7)
    if n == 0:
        rowptr, colidx, vals = np.zeros(1, np.int32), np.zeros(0, np.int32), np.zeros(0, np.float32)
    else:
        rowptr, colidx, vals, _ = random_csr(rng, n, n + 2, 0.4, empty_rows=(0,) if n > 1 else ())
    h = pc.pcsr_build(n, n + 2, rowptr, colidx, vals, pc.make_params(V=V, S=S, SG=2 if S else 0, flags=HOST))
    _assert_same(pc.pcsr_export(h), pf.pcsr_ref(n, rowptr, colidx, vals, V, S, 2 if S else 0, 64))


def test_explicit_zero_is_kept_as_a_vector():
    rowptr = np.array([0, 2, 3], np.int32)
    colidx = np.array([1, 4, 2], np.int32)
    vals = np.array([0.0, 3.0, -0.0], np.float32)
    for V in (1, 2):
        h = pc.pcsr_build(2, 5, rowptr, colidx, vals, pc.make_params(V=V, flags=HOST))
        e = pc.pcsr_export(h)
        _assert_same(e, pf.pcsr_ref(2, rowptr, colidx, vals, V, 0))
        assert e["nnz_v"] == 3


@pytest.mark.parametrize("name", ["poisson", "road", "rmat20", "sbm"])
@pytest.mark.parametrize("omega", [32, 64])
def test_features_match_reference(name, omega):
    g = synth.workload(name, "small")
    f = pc.pcsr_features(g.n_rows, g.n_cols, g.rowptr, g.colidx, omega)
    r = pf.features(g.n_rows, g.n_cols, g.rowptr, g.colidx, omega)
    assert np.allclose(f[:16], r, rtol=1e-12, atol=0)          # Table 3
    assert f[14] == 0.0 and 0.0 <= f[15] <= 0.5 and f[9] >= 1.0 and f[10] >= 1.0
    assert f[16] == pytest.approx(near_diagonal_share(g.rowptr, g.colidx), rel=1e-12)   # the library's own


def test_near_diagonal_feature_closed_forms():
    n = 3000
    eye_rp, eye_ci = np.arange(n + 1, dtype=np.int32), np.arange(n, dtype=np.int32)
    assert pc.pcsr_features(n, n, eye_rp, eye_ci)[16] == 1.0
    far = ((np.arange(n) + 512) % n).astype(np.int32)            # every nonzero exactly 512 (or more) away
    assert pc.pcsr_features(n, n, eye_rp, far)[16] == 0.0
    near = ((np.arange(n) + 511) % n).astype(np.int32)
    assert pc.pcsr_features(n, n, eye_rp, near)[16] == pytest.approx((n - 511) / n)
    assert pc.pcsr_features(3, 5, np.zeros(4, np.int32), np.zeros(0, np.int32))[16] == 0.0


def test_gap_export_matches_table2():
    for line in (ROOT / "tests/golden/table2_gap.txt").read_text().splitlines():
        if line.strip() and not line.startswith("#"):
            dim, F, gap = map(int, line.split())
            assert pc.pcsr_mac_job_gap(dim, F, 32) == gap
    assert pc.pcsr_mac_job_gap(0, 1, 32) == -1


def _expect(code, *args, **kw):
    with pytest.raises(pc.PcsrError) as ei:
        pc.pcsr_build(*args, **kw)
    assert ei.value.code == code


def test_error_paths():
    rp = np.array([0, 2, 3], np.int32)
    ci = np.array([0, 1, 2], np.int32)
    va = np.ones(3, np.float32)
    P = lambda **k: pc.make_params(flags=HOST, **k)  # noqa: E731
    _expect(binding.PCSR_E_UNSUPPORTED, 2, 3, rp, ci, va, P(V=3))
    _expect(binding.PCSR_E_UNSUPPORTED, 2, 3, rp, ci, va, P(S=2))
    _expect(binding.PCSR_E_UNSUPPORTED, 2, 3, rp, ci, va, P(lanes_per_row=3))
    _expect(binding.PCSR_E_UNSUPPORTED, 2, 3, rp, ci, va, P(vec=3))
    _expect(binding.PCSR_E_UNSUPPORTED, 2, 3, rp, ci, va, P(waves_per_wg=3))
    _expect(binding.PCSR_E_INVALID_ARG, 2, 3, rp, ci, va, P(SG=-1))
    # malformed CSR
    _expect(binding.PCSR_E_BAD_CSR, 2, 3, np.array([0, 3, 2], np.int32), ci, va, P())        # not monotone
    _expect(binding.PCSR_E_BAD_CSR, 2, 3, np.array([1, 2, 3], np.int32), ci, va, P())        # start != 0
    _expect(binding.PCSR_E_BAD_CSR, 2, 3, np.array([0, 2, 2], np.int32), ci, va, P())        # end != nnz
    _expect(binding.PCSR_E_BAD_CSR, 2, 3, rp, np.array([0, 3, 2], np.int32), va, P())        # col >= n_cols
    _expect(binding.PCSR_E_BAD_CSR, 2, 3, rp, np.array([0, -1, 2], np.int32), va, P())       # negative col
    _expect(binding.PCSR_E_BAD_CSR, 2, 3, rp, np.array([1, 0, 2], np.int32), va, P())        # unsorted
    _expect(binding.PCSR_E_BAD_CSR, 2, 3, rp, np.array([1, 1, 2], np.int32), va, P())        # duplicate
    # reserved must be zero
    p = P()
    p.reserved[0] = 5
    _expect(binding.PCSR_E_INVALID_ARG, 2, 3, rp, ci, va, p)
    # SpMM on a host-only handle is refused, never silently computed elsewhere
    h = pc.pcsr_build(2, 3, rp, ci, va, P())
    lib = binding._lib()
    assert lib.pcsr_spmm(h.raw, None, None, 4, None) == binding.PCSR_E_UNSUPPORTED
    assert lib.pcsr_spmm(None, None, None, 4, None) == binding.PCSR_E_INVALID_ARG
    assert lib.pcsr_free(None) == 0
    assert "CSR" in pc.pcsr_strerror(binding.PCSR_E_BAD_CSR)


def test_launch_resolution():
    g = synth.workload("poisson", "small")
    h = pc.pcsr_build(g.n_rows, g.n_cols, g.rowptr, g.colidx, g.vals, pc.make_params(flags=HOST))
    q = pc.pcsr_query_launch(h, 8)
    assert (q["lanes_per_row"], q["vec"], q["rep"]) == (4, 4, 1) and q["grid_y"] == 1
    q = pc.pcsr_query_launch(h, 16)                      # rows of 8 on average: 16 lanes of one dword
    assert (q["lanes_per_row"], q["vec"], q["rep"]) == (16, 1, 1) and q["grid_y"] == 1
    per_wg = q["waves_per_wg"] * 4
    # one work-balanced item range per XCD: 8 x the workgroups of the longest range
    assert q["grid_x"] % 8 == 0 and -(-g.n_rows // per_wg) <= q["grid_x"] <= -(-g.n_rows // per_wg) + 64
    pc.pcsr_set_kernel_params(h, flags=pc.PCSR_FLAG_NO_XCD_REMAP)
    assert pc.pcsr_query_launch(h, 16)["grid_x"] == -(-g.n_rows // per_wg)
    pc.pcsr_set_kernel_params(h)
    q = pc.pcsr_query_launch(h, 512)
    assert q["lanes_per_row"] * q["vec"] * q["rep"] * q["grid_y"] >= 512
    q = pc.pcsr_query_launch(h, 33)
    assert q["vec"] == 1 and q["lanes_per_row"] * q["rep"] * q["grid_y"] >= 33
    pc.pcsr_set_kernel_params(h, 8, 2, 2, 1)
    q = pc.pcsr_query_launch(h, 128)
    assert (q["lanes_per_row"], q["vec"], q["rep"], q["waves_per_wg"], q["grid_y"]) == (8, 2, 2, 1, 4)
    with pytest.raises(pc.PcsrError):
        pc.pcsr_query_launch(h, 33)          # vec = 2 does not divide 33
    with pytest.raises(pc.PcsrError):
        pc.pcsr_set_kernel_params(h, 5, 0, 0, 0)
    with pytest.raises(pc.PcsrError):
        pc.pcsr_set_kernel_params(h, items_per_group=3)
    pc.pcsr_set_kernel_params(h, 32, 4, 1, 4, 4)
    q = pc.pcsr_query_launch(h, 128)
    assert q["items_per_group"] == 4 and q["grid_x"] % 8 == 0
    assert -(-g.n_rows // (4 * 2 * 4)) <= q["grid_x"] <= -(-g.n_rows // (4 * 2 * 4)) + 64
    pc.pcsr_set_kernel_params(h, 4, 4, 1, 4, 4)          # items_per_group must be < lanes_per_row
    with pytest.raises(pc.PcsrError):
        pc.pcsr_query_launch(h, 16)


def test_select_returns_valid_tuple():
    for name in ("road", "rmat20", "sbm"):
        g = synth.workload(name, "small")
        f = pc.pcsr_features(g.n_rows, g.n_cols, g.rowptr, g.colidx)
        p = pc.pcsr_select(f, 64)
        assert p.V in (1, 2) and p.S in (0, 1)
    assert pc.pcsr_select(pc.pcsr_features(*(lambda g: (g.n_rows, g.n_cols, g.rowptr, g.colidx))(
        synth.workload("road", "small"))), 64).S == 0


def test_select_always_returns_a_tuple_the_library_can_launch():
    """Whatever the features (random, extreme, non-finite) and the width, the rule returns
    parameters inside the documented domains, and a handle built from them resolves to a
    launch shape that exists."""
    rng = np.random.default_rng(11)
    g = synth.workload("sbm", "small")
    base = np.array(pc.pcsr_features(g.n_rows, g.n_cols, g.rowptr, g.colidx), dtype=np.float64)
    handles = {}
    for trial in range(400):
        f = base.copy()
        if trial % 4:
            f[0] = f[1] = float(rng.choice([1, 50, 4096, 90_000, 250_000, 4_000_000, 2**31 - 1]))
            f[4] = f[5] = float(rng.choice([0.0, 1.0, 3.0, 7.9, 12.0, 39.9, 40.0, 200.0, 1e5]))
            f[6] = f[5] * float(rng.choice([1.0, 2.0, 100.0, 1e4]))
            f[7] = f[8] = float(rng.choice([0.0, 0.1, 1.49, 1.51, 8.0]))
            f[15] = float(rng.choice([0.0, 0.1, 0.19, 0.2, 0.3, 0.45, 0.5]))
            f[16] = float(rng.choice([0.0, 1e-4, 0.01, 0.3, 0.6, 0.9, 1.0]))
        if trial % 50 == 49:
            f[int(rng.integers(0, f.shape[0]))] = float(rng.choice([np.nan, np.inf, -np.inf, -1.0]))
        K = int(rng.choice([1, 2, 3, 7, 8, 9, 12, 16, 17, 24, 32, 33, 48, 64, 96, 100, 128, 255, 256, 512, 2048]))
        p = pc.pcsr_select(f, K)
        assert p.V in (1, 2) and p.S in (0, 1) and p.SG >= 0 and p.omega in (0, 32, 64)
        assert p.lanes_per_row in (4, 8, 16, 32, 64) and p.vec in (1, 2, 4) and K % p.vec == 0
        assert p.rep in (1, 2, 4) and 1 <= p.waves_per_wg <= 16 and p.items_per_group in (0, 1)
        assert p.col_window in (0, 512)
        if p.col_window:
            assert (p.col_window + 1) * (p.lanes_per_row * p.vec * p.rep + 4) * 4 <= 160 * 1024
            assert p.S == 0 and p.V == 1 and p.flags & pc.PCSR_FLAG_WINDOW_IF_USEFUL
        if p.flags & pc.PCSR_FLAG_COLUMN_ORDER:
            assert p.S == 1
        # the launch shape exists for a handle of that format (built once per format)
        key = (p.V, p.S, min(p.SG, 64), p.col_window, p.flags & pc.PCSR_FLAG_COLUMN_ORDER)
        if key not in handles:
            handles[key] = pc.pcsr_build(g.n_rows, g.n_cols, g.rowptr, g.colidx, g.vals, pc.make_params(
                V=p.V, S=p.S, SG=key[2], col_window=p.col_window, flags=HOST | key[4]))
        h = handles[key]
        pc.pcsr_set_kernel_params(h, p.lanes_per_row, p.vec, p.rep, p.waves_per_wg, 0)
        q = pc.pcsr_query_launch(h, K)
        assert q["lanes_per_row"] == p.lanes_per_row and q["vec"] == p.vec and q["grid_y"] >= 1
        assert q["lanes_per_row"] * q["vec"] * q["rep"] * q["grid_y"] >= K
    for h in handles.values():
        h.close()


def test_reorder_is_a_permutation_and_recovers_planted_clusters():
    g = synth.workload("sbm_shuffled", "small")          # 24 blocks of 500, ids shuffled
    perm, ncl = pc.pcsr_reorder(g.n_rows, g.rowptr, g.colidx)
    assert np.array_equal(np.sort(perm), np.arange(g.n_rows))
    assert ncl == 24
    perm2, _ = pc.pcsr_reorder(g.n_rows, g.rowptr, g.colidx)
    assert np.array_equal(perm, perm2)                   # deterministic
    rp, ci, va = pc.pcsr_permute_csr(g.n_rows, g.rowptr, g.colidx, g.vals, perm)
    # the relabelled matrix is P A P^T: compare with scipy
    import scipy.sparse as sp
    A = sp.csr_matrix((g.vals, g.colidx, g.rowptr), shape=(g.n_rows, g.n_cols)).tocoo()
    A2 = sp.csr_matrix((A.data, (perm[A.row], perm[A.col])), shape=A.shape)
    A2.sort_indices()
    assert np.array_equal(rp, A2.indptr) and np.array_equal(ci, A2.indices)
    assert np.array_equal(va.view(np.uint32), A2.data.astype(np.float32).view(np.uint32))
    # rows of one planted block end up contiguous: the average row bandwidth collapses
    b_before = pc.pcsr_features(g.n_rows, g.n_cols, g.rowptr, g.colidx)[12]
    b_after = pc.pcsr_features(g.n_rows, g.n_cols, rp, ci)[12]
    assert b_after < 0.8 * b_before
    h = pc.pcsr_build(g.n_rows, g.n_cols, rp, ci, va, pc.make_params(col_window=1024, flags=HOST))
    assert pc.pcsr_window_stats(h)["hit_fraction"] > 0.85


def test_reorder_error_paths_and_degenerate_inputs():
    perm, ncl = pc.pcsr_reorder(0, np.zeros(1, np.int32), np.zeros(0, np.int32))
    assert perm.size == 0 and ncl == 0
    perm, ncl = pc.pcsr_reorder(5, np.zeros(6, np.int32), np.zeros(0, np.int32))
    assert np.array_equal(perm, np.arange(5)) and ncl == 5
    with pytest.raises(pc.PcsrError):
        pc.pcsr_reorder(2, np.array([0, 1, 2], np.int32), np.array([0, 5], np.int32))
    with pytest.raises(pc.PcsrError):
        pc.pcsr_permute_csr(2, np.array([0, 1, 2], np.int32), np.array([0, 1], np.int32),
                            np.ones(2, np.float32), np.array([0, 0], np.int32))
    # a column outside [0, n) cannot be relabelled: an error, not a silently wrong row
    for bad in (5, -1):
        with pytest.raises(pc.PcsrError) as ei:
            pc.pcsr_permute_csr(2, np.array([0, 1, 2], np.int32), np.array([0, bad], np.int32),
                                np.ones(2, np.float32), np.array([1, 0], np.int32))
        assert ei.value.code == binding.PCSR_E_BAD_CSR


def test_workspace_size_of_the_balanced_write_back():
    """V*K floats per work item of every panel that was split; nothing without balancing or
    with the atomic write-back."""
    g = synth.workload("rmat20", "small")
    for V in (1, 2):
        h = pc.pcsr_build(g.n_rows, g.n_cols, g.rowptr, g.colidx, g.vals, pc.make_params(V=V, S=1, SG=16, flags=HOST))
        r = pf.pcsr_ref(g.n_rows, g.rowptr, g.colidx, g.vals, V, 1, 16, 64)
        per_panel = np.bincount(r["trow"], minlength=r["P"])
        slots = int(per_panel[per_panel > 1].sum())
        assert slots > 0
        assert pc.pcsr_workspace_bytes(h, 40) == slots * V * 40 * 4
        pc.pcsr_set_kernel_params(h, flags=pc.PCSR_FLAG_ATOMIC_SPLIT)
        assert pc.pcsr_workspace_bytes(h, 40) == 0
        with pytest.raises(pc.PcsrError):
            pc.pcsr_reserve_workspace(h, 40)              # host-only handle: nothing to reserve on
        h.close()
    h = pc.pcsr_build(g.n_rows, g.n_cols, g.rowptr, g.colidx, g.vals, pc.make_params(V=1, S=0, flags=HOST))
    assert pc.pcsr_workspace_bytes(h, 40) == 0
    h.close()


def test_transpose_csr_host():
    import scipy.sparse as sp
    rng = np.random.default_rng(4)
    rowptr, colidx, vals, dense = random_csr(rng, 13, 29, 0.3, empty_rows=(2,))
    trp, tci, tva = pc.pcsr_transpose_csr(13, 29, rowptr, colidx, vals)
    At = sp.csr_matrix(dense.T)
    At.sort_indices()
    assert np.array_equal(trp, At.indptr) and np.array_equal(tci, At.indices)
    assert np.array_equal(tva, At.data)
    with pytest.raises(pc.PcsrError):
        pc.pcsr_transpose_csr(2, 2, np.array([0, 1, 2], np.int32), np.array([0, 7], np.int32),
                              np.ones(2, np.float32))


@pytest.mark.parametrize("name", ["rmat20", "rmat22", "sbm", "poisson"])
@pytest.mark.parametrize("V,SG", [(1, 4), (2, 16), (1, 0)])
def test_column_ordered_schedule_host(name, V, SG):
    g = synth.workload(name, "small")
    h = pc.pcsr_build(g.n_rows, g.n_cols, g.rowptr, g.colidx, g.vals,
                      pc.make_params(V=V, S=1, SG=SG, flags=HOST | pc.PCSR_FLAG_COLUMN_ORDER))
    e = pc.pcsr_export(h)
    got = pc.pcsr_export_schedule(h)
    sched, xb = column_ordered_schedule(e["rowptr"], e["colidx"], e["trow"], e["P"])
    assert np.array_equal(got["xcd_bounds"], xb)
    assert np.array_equal(got["sched"], sched)
    # a permutation of the items: every vector range appears exactly once
    assert np.array_equal(np.sort(got["sched"][:, 0] * 1), np.sort(e["rowptr"][:-1]))
    h.close()
    h = pc.pcsr_build(g.n_rows, g.n_cols, g.rowptr, g.colidx, g.vals, pc.make_params(V=V, S=1, SG=SG, flags=HOST))
    assert pc.pcsr_export_schedule(h)["sched"] is None
    h.close()
    with pytest.raises(pc.PcsrError):                       # needs balancing
        pc.pcsr_build(g.n_rows, g.n_cols, g.rowptr, g.colidx, g.vals,
                      pc.make_params(V=V, S=0, flags=HOST | pc.PCSR_FLAG_COLUMN_ORDER))


def test_reorder_by_degree():
    g = synth.workload("rmat20", "small")
    perm = pc.pcsr_reorder_by_degree(g.n_rows, g.rowptr, g.colidx)
    assert np.array_equal(np.sort(perm), np.arange(g.n_rows))
    indeg = np.bincount(g.colidx, minlength=g.n_cols)
    # new id = rank by descending in-degree, ties in original order
    expect = np.empty(g.n_rows, np.int32)
    expect[np.argsort(-indeg, kind="stable")] = np.arange(g.n_rows)
    assert np.array_equal(perm, expect)
    rp, ci, va = pc.pcsr_permute_csr(g.n_rows, g.rowptr, g.colidx, g.vals, perm)
    indeg2 = np.bincount(ci, minlength=g.n_cols)
    assert np.all(np.diff(indeg2) <= 0)                      # hubs first
    with pytest.raises(pc.PcsrError):
        pc.pcsr_reorder_by_degree(2, np.array([0, 1, 2], np.int32), np.array([0, 5], np.int32))
    assert pc.pcsr_reorder_by_degree(0, np.zeros(1, np.int32), np.zeros(0, np.int32)).size == 0


def test_selector_proposes_the_window_only_where_the_build_keeps_it():
    g = synth.workload("sbm", "small")                       # 24 communities of 500 consecutive ids
    f = np.array(pc.pcsr_features(g.n_rows, g.n_cols, g.rowptr, g.colidx), dtype=np.float64)
    # 12,000 rows give 24 window blocks: far too few for 256 compute units, so no window
    small = pc.pcsr_select(f, 128)
    assert small.col_window == 0 and small.S == 0 and small.V == 1
    f[0] = f[1] = 250_000                                    # the same structure at the full size
    assert pc.pcsr_select(f, 32).col_window == 0            # narrow B rows: the plain kernel ties
    assert pc.pcsr_select(f, 64).col_window == 512
    f[0] = f[1] = 150_000
    assert pc.pcsr_select(f, 64).col_window == 0            # 150,000 rows x 1 slice: too few blocks
    f[0] = f[1] = 250_000
    sel = pc.pcsr_select(f, 128)
    assert sel.col_window == 512 and sel.S == 0 and sel.flags & pc.PCSR_FLAG_WINDOW_IF_USEFUL
    sel.flags |= HOST
    h = pc.pcsr_build(g.n_rows, g.n_cols, g.rowptr, g.colidx, g.vals, sel)
    st = pc.pcsr_window_stats(h)
    assert st["col_window"] == 512 and st["hit_fraction"] > 0.85 and 400 <= st["items_per_block"] <= 500
    assert pc.pcsr_query_launch(h, 128)["lds_bytes"] > 0
    h.close()
    # the same request on the shuffled graph: the build finds no blocks and drops the window
    gs = synth.workload("sbm_shuffled", "small")
    fs = np.array(pc.pcsr_features(gs.n_rows, gs.n_cols, gs.rowptr, gs.colidx), dtype=np.float64)
    shuffled = pc.pcsr_select(fs, 128)
    # long rows, scattered columns: items of 32 in column order from K = 64, paired rows below
    assert shuffled.col_window == 0 and shuffled.S == 1 and shuffled.SG == 32
    assert shuffled.flags & pc.PCSR_FLAG_COLUMN_ORDER and shuffled.lanes_per_row == 16
    narrow = pc.pcsr_select(fs, 32)                           # too few rows to pair them
    assert narrow.S == 0 and narrow.V == 1 and narrow.col_window == 0
    fs[0] = fs[1] = 250_000
    fs[16] = 0.002                                            # near-diagonal share of uniform columns at that size
    assert pc.pcsr_select(fs, 128).col_window == 0
    narrow = pc.pcsr_select(fs, 32)                           # B = 32 MB, scattered: a dword per lane
    assert (narrow.S, narrow.V, narrow.lanes_per_row, narrow.vec, narrow.rep) == (0, 1, 32, 1, 1)
    fs[0] = fs[1] = 100_000                                   # B = 12.8 MB: rows paired instead
    fs[16] = 0.005
    narrow = pc.pcsr_select(fs, 32)
    assert narrow.S == 0 and narrow.V == 2 and narrow.waves_per_wg == 2 and narrow.vec == 4
    k16 = pc.pcsr_select(fs, 16)                              # K = 16: 16 lanes of one dword
    assert (k16.lanes_per_row, k16.vec, k16.rep) == (16, 1, 1)
    road = synth.workload("road", "small")
    fr = pc.pcsr_features(road.n_rows, road.n_cols, road.rowptr, road.colidx)
    r16 = pc.pcsr_select(fr, 16)                              # rows of 3: many rows per wavefront
    assert (r16.V, r16.lanes_per_row, r16.vec) == (2, 4, 4)
    h = pc.pcsr_build(gs.n_rows, gs.n_cols, gs.rowptr, gs.colidx, gs.vals, sel)
    assert pc.pcsr_window_stats(h)["col_window"] == 0
    q = pc.pcsr_query_launch(h, 128)
    assert q["lds_bytes"] == 0 and q["waves_per_wg"] <= 8
    h.close()
    # without the flag the window blocks are kept whatever they look like
    h = pc.pcsr_build(gs.n_rows, gs.n_cols, gs.rowptr, gs.colidx, gs.vals, pc.make_params(col_window=512, flags=HOST))
    assert pc.pcsr_window_stats(h)["col_window"] == 512
    h.close()
