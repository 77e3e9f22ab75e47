"""GPU parity: the HIP path, called through the C ABI, against the fp64 CPU oracle.

Acceptance for every element: |C - C_ref| <= 1e-5 * sum_j |a_ij b_jk| + 1e-6.
PCSR arrays read back from the device must equal the numpy format reference bit for bit.
"""
import itertools

import numpy as np
import pytest

import oracle
import paper_2605_15695_amd as pc
from oracle import pcsr_format as pf
import synth
from tests.helpers import column_ordered_schedule, near_diagonal_share, random_csr

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

RTOL, ATOL = 1e-5, 1e-6


def _spmm(g, B, params, K, prefill=float("nan"), stream=None, kernel=None):
    h = pc.pcsr_build(g.n_rows, g.n_cols, g.rowptr, g.colidx, g.vals, params)
    if kernel:
        pc.pcsr_set_kernel_params(h, *kernel)
    Bd = torch.from_numpy(B).cuda()
    Cd = torch.full((g.n_rows, K), prefill, dtype=torch.float32, device="cuda")
    pc.pcsr_spmm(h, Bd, Cd, K, stream)
    torch.cuda.synchronize()
    out = Cd.cpu().numpy()
    h.close()
    return out


def _check(C, ref, bound, what=""):
    ok, worst = oracle.within_tolerance(C, ref, bound, RTOL, ATOL)
    assert ok, f"{what}: worst err/limit = {worst:.3g}"


_ORACLE_CACHE = {}


def _oracle(name, g, K, dist):
    key = (name, K, dist)
    if key not in _ORACLE_CACHE:
        B = synth.dense_operand(g.n_cols, K, dist, 17 + K)
        _ORACLE_CACHE[key] = (B,) + oracle.spmm(g.rowptr, g.colidx, g.vals, B)
    return _ORACLE_CACHE[key]


_GRAPHS = {}


def _graph(name):
    if name not in _GRAPHS:
        _GRAPHS[name] = synth.workload(name, "small")
    return _GRAPHS[name]


@pytest.mark.parametrize("name", list(synth.WORKLOADS))
@pytest.mark.parametrize("V,S", [(1, 0), (1, 1), (2, 0), (2, 1)])
def test_workloads_default_kernel(name, V, S):
    g = _graph(name)
    spec = synth.WORKLOADS[name]
    for K in sorted(set(spec["K"]) | {16}):
        B, ref, bound = _oracle(name, g, K, spec["B"])
        print(f"case {name} V={V} S={S} K={K}", flush=True)
        C = _spmm(g, B, pc.make_params(V=V, S=S), K)
        _check(C, ref, bound, f"{name} V={V} S={S} K={K}")


@pytest.mark.parametrize("V,S", [(1, 0), (1, 1), (2, 0), (2, 1)])
def test_every_kernel_variant(V, S):
    """All (lanes_per_row, vec, rep) instances, each at a K that needs two grid.y slices
    with a ragged last slice, on a skewed graph with an odd row count."""
    g0 = _graph("rmat20")
    n = g0.n_rows - 1                       # odd: the last V=2 panel is short
    nnz = int(g0.rowptr[n])
    cols_ok = g0.colidx[:nnz] < n
    # drop the last row and column so the matrix stays square
    keep = np.nonzero(cols_ok)[0]
    row_of = np.repeat(np.arange(n), np.diff(g0.rowptr[:n + 1]))[keep]
    rowptr = np.zeros(n + 1, np.int32)
    np.cumsum(np.bincount(row_of, minlength=n), out=rowptr[1:])
    g = synth.Graph("rmat_odd", n, n, rowptr, g0.colidx[keep], g0.vals[keep])
    h = pc.pcsr_build(g.n_rows, g.n_cols, g.rowptr, g.colidx, g.vals, pc.make_params(V=V, S=S, SG=32))
    waves_cycle = itertools.cycle([1, 2, 4, 8])
    cache = {}
    for lpr, vec, rep in itertools.product([4, 8, 16, 32, 64], [1, 2, 4], [1, 2, 4]):
        K = lpr * vec * rep + vec * 3       # second slice covers 3 lanes' worth only
        if K not in cache:
            B = synth.dense_operand(n, K, "normal", K)
            cache[K] = (torch.from_numpy(B).cuda(),) + oracle.spmm(g.rowptr, g.colidx, g.vals, B)
        Bd, ref, bound = cache[K]
        waves = next(waves_cycle)
        print(f"case V={V} S={S} lpr={lpr} vec={vec} rep={rep} waves={waves} K={K}", flush=True)
        pc.pcsr_set_kernel_params(h, lpr, vec, rep, waves, flags=pc.PCSR_FLAG_NO_XCD_REMAP if rep == 2 else 0)
        q = pc.pcsr_query_launch(h, K)
        assert q["grid_y"] == 2
        Cd = torch.full((n, K), float("nan"), dtype=torch.float32, device="cuda")
        pc.pcsr_spmm(h, Bd, Cd, K)
        torch.cuda.synchronize()
        _check(Cd.cpu().numpy(), ref, bound, f"V={V} S={S} lpr={lpr} vec={vec} rep={rep}")
    h.close()


@pytest.mark.parametrize("name", ["sbm", "road"])
@pytest.mark.parametrize("V", [1, 2])
def test_batched_kernel_variants(name, V):
    """items_per_group in {2, 4}: every instance, ragged K over two grid.y slices, odd row count."""
    g0 = _graph(name)
    n = g0.n_rows - 1
    nnz = int(g0.rowptr[n])
    g = synth.Graph(name + "_odd", n, g0.n_cols, g0.rowptr[:n + 1].copy(), g0.colidx[:nnz], g0.vals[:nnz])
    h = pc.pcsr_build(g.n_rows, g.n_cols, g.rowptr, g.colidx, g.vals, pc.make_params(V=V, S=0))
    cache = {}
    tested = 0
    waves_cycle = itertools.cycle([1, 2, 4, 8])
    for ipg, lpr, vec, rep in itertools.product([2, 4], [4, 8, 16, 32, 64], [1, 2, 4], [1, 2, 4]):
        K = lpr * vec * rep + vec * 3
        pc.pcsr_set_kernel_params(h, lpr, vec, rep, next(waves_cycle), ipg)
        try:
            q = pc.pcsr_query_launch(h, K)
        except pc.PcsrError:
            assert not (ipg < lpr and V * vec * rep * ipg <= 32)
            continue
        assert q["items_per_group"] == ipg and q["grid_y"] == 2
        if K not in cache:
            B = synth.dense_operand(g.n_cols, K, "normal", K)
            cache[K] = (torch.from_numpy(B).cuda(),) + oracle.spmm(g.rowptr, g.colidx, g.vals, B)
        Bd, ref, bound = cache[K]
        print(f"case {name} V={V} ipg={ipg} lpr={lpr} vec={vec} rep={rep} K={K}", flush=True)
        Cd = torch.full((n, K), float("nan"), dtype=torch.float32, device="cuda")
        pc.pcsr_spmm(h, Bd, Cd, K)
        torch.cuda.synchronize()
        _check(Cd.cpu().numpy(), ref, bound, f"{name} V={V} ipg={ipg} lpr={lpr} vec={vec} rep={rep}")
        tested += 1
    assert tested >= 30
    h.close()


def test_batched_kernel_refused_where_it_does_not_apply():
    g = _graph("rmat20")                     # longest row > 1024
    h = pc.pcsr_build(g.n_rows, g.n_cols, g.rowptr, g.colidx, g.vals, pc.make_params(V=1, S=0))
    pc.pcsr_set_kernel_params(h, items_per_group=2)
    with pytest.raises(pc.PcsrError):
        pc.pcsr_query_launch(h, 64)
    h.close()
    h = pc.pcsr_build(g.n_rows, g.n_cols, g.rowptr, g.colidx, g.vals, pc.make_params(V=1, S=1, SG=64))
    pc.pcsr_set_kernel_params(h, items_per_group=2)
    with pytest.raises(pc.PcsrError):
        pc.pcsr_query_launch(h, 64)
    h.close()


@pytest.mark.parametrize("name", ["sbm", "sbm_shuffled", "road", "poisson"])
@pytest.mark.parametrize("V", [1, 2])
@pytest.mark.parametrize("wc", [256, 1024])
def test_column_window_kernel(name, V, wc):
    """B window staged in LDS: clustered input (most gathers from LDS), shuffled and
    road-like inputs (few or no windows), several slice shapes and workgroup sizes."""
    g = _graph(name)
    h = pc.pcsr_build(g.n_rows, g.n_cols, g.rowptr, g.colidx, g.vals, pc.make_params(V=V, col_window=wc))
    st = pc.pcsr_window_stats(h)
    assert st["col_window"] == wc and 1 <= st["items_per_block"] <= wc
    if name == "sbm" and wc == 1024:
        assert st["hit_fraction"] > 0.7
    assert 0.0 <= st["hit_fraction"] <= 1.0
    spec = synth.WORKLOADS[name]
    for K, kern in [(64, None), (40, None), (256, None), (64, (8, 4, 1, 4)), (48, (16, 1, 2, 16)),
                    (24, (4, 2, 1, 8))]:
        if kern:
            pc.pcsr_set_kernel_params(h, *kern)
        else:
            pc.pcsr_set_kernel_params(h)
        q = pc.pcsr_query_launch(h, K)
        assert 0 < q["lds_bytes"] <= 160 * 1024
        B, ref, bound = _oracle(name, g, K, spec["B"])
        print(f"case window {name} V={V} wc={wc} K={K} {q}", flush=True)
        Cd = torch.full((g.n_rows, K), float("nan"), dtype=torch.float32, device="cuda")
        pc.pcsr_spmm(h, torch.from_numpy(B).cuda(), Cd, K)
        torch.cuda.synchronize()
        _check(Cd.cpu().numpy(), ref, bound, f"window {name} V={V} wc={wc} K={K} {kern}")
    h.close()


def test_column_window_edges():
    """Window wider than the matrix, last block partly filled, odd row count with V = 2."""
    rng = np.random.default_rng(11)
    rp, ci, va, _ = random_csr(rng, 301, 200, 0.5)          # n_cols < col_window
    g = synth.Graph("dense_small", 301, 200, rp, ci, va)
    for V in (1, 2):
        for K in (16, 36):
            B = synth.dense_operand(200, K, "uniform", K)
            ref, bound = oracle.spmm(rp, ci, va, B)
            C = _spmm(g, B, pc.make_params(V=V, col_window=256), K)
            _check(C, ref, bound, f"window edges V={V} K={K}")
    h = pc.pcsr_build(301, 200, rp, ci, va, pc.make_params(col_window=256))
    assert pc.pcsr_window_stats(h)["hit_fraction"] == 1.0
    h.close()
    # CSR arrays in device memory: copied to the host for the window build (the caller's
    # parameter struct is not modified by the binding)
    prm = pc.make_params(V=2, col_window=256)
    hd = pc.pcsr_build(301, 200, *(torch.from_numpy(x).cuda() for x in (rp, ci, va)), prm)
    assert prm.flags == 0 and pc.pcsr_window_stats(hd)["hit_fraction"] == 1.0
    B = synth.dense_operand(200, 16, "uniform", 16)
    ref, bound = oracle.spmm(rp, ci, va, B)
    Cd = torch.full((301, 16), float("nan"), dtype=torch.float32, device="cuda")
    pc.pcsr_spmm(hd, torch.from_numpy(B).cuda(), Cd, 16)
    torch.cuda.synchronize()
    _check(Cd.cpu().numpy(), ref, bound, "window build from device CSR")
    hd.close()
    with pytest.raises(pc.PcsrError):
        pc.pcsr_build(301, 200, rp, ci, va, pc.make_params(S=1, col_window=256))
    with pytest.raises(pc.PcsrError):
        pc.pcsr_build(301, 200, rp, ci, va, pc.make_params(col_window=300))


def _tiny_cases():
    rng = np.random.default_rng(3)
    cases = {}
    cases["n1"] = (1, 1, np.array([0, 1], np.int32), np.array([0], np.int32), np.array([2.5], np.float32))
    cases["n1_empty"] = (1, 4, np.array([0, 0], np.int32), np.zeros(0, np.int32), np.zeros(0, np.float32))
    rp, ci, va, _ = random_csr(rng, 3, 5, 0.6)
    cases["n3_rect"] = (3, 5, rp, ci, va)
    rp, ci, va, _ = random_csr(rng, 37, 37, 0.2, empty_rows=(0, 1, 35, 36))
    cases["empty_first_last"] = (37, 37, rp, ci, va)
    rp, ci, va, _ = random_csr(rng, 9, 700, 0.01, full_rows=(4,))
    cases["one_dense_row"] = (9, 700, rp, ci, va)
    rp, ci, va, _ = random_csr(rng, 64, 300, 0.0, full_rows=(7, 8, 40))
    cases["only_long_rows"] = (64, 300, rp, ci, va)
    cases["all_empty"] = (10, 10, np.zeros(11, np.int32), np.zeros(0, np.int32), np.zeros(0, np.float32))
    return cases


@pytest.mark.parametrize("case", list(_tiny_cases()))
def test_tiny_adversarial_all_tuples(case):
    n_rows, n_cols, rp, ci, va = _tiny_cases()[case]
    g = synth.Graph(case, n_rows, n_cols, rp, ci, va)
    for K in (16, 20, 1):
        B = synth.dense_operand(n_cols, K, "uniform", 5)
        ref, bound = oracle.spmm(rp, ci, va, B)
        for V, S, SG in [(1, 0, 0), (2, 0, 0), (1, 1, 0), (2, 1, 0), (1, 1, 3), (2, 1, 3), (1, 1, 64)]:
            kernels = [None, (4, 0, 0, 1), (64, 0, 1, 2), (16, 1, 2, 8)]
            if not S:
                kernels += [(8, 0, 1, 2, 4), (64, 0, 0, 1, 2)]
            for kern in kernels:
                print(f"case {case} K={K} V={V} S={S} SG={SG} kernel={kern}", flush=True)
                C = _spmm(g, B, pc.make_params(V=V, S=S, SG=SG), K, kernel=kern)
                _check(C, ref, bound, f"{case} K={K} V={V} S={S} SG={SG} {kern}")


@pytest.mark.parametrize("name", ["rmat20", "road"])
@pytest.mark.parametrize("V,S,SG", [(1, 0, 0), (2, 0, 0), (1, 1, 0), (2, 1, 16)])
def test_device_arrays_bit_exact(name, V, S, SG):
    g = _graph(name)
    h = pc.pcsr_build(g.n_rows, g.n_cols, g.rowptr, g.colidx, g.vals, pc.make_params(V=V, S=S, SG=SG))
    e = pc.pcsr_export(h)
    r = pf.pcsr_ref(g.n_rows, g.rowptr, g.colidx, g.vals, V, S, SG, 64)
    for k in ("P", "M", "nnz_v", "V", "SG"):
        assert e[k] == r[k]
    for k in ("rowptr", "colidx", "trow"):
        assert np.array_equal(e[k], r[k]), k
    assert np.array_equal(e["val"].view(np.uint32), r["val"].view(np.uint32))
    h.close()


def test_device_csr_input_and_side_stream():
    g = _graph("sbm")
    K = 64
    B, ref, bound = _oracle("sbm", g, K, "uniform")
    rp, ci, va = (torch.from_numpy(x).cuda() for x in (g.rowptr, g.colidx, g.vals))
    h = pc.pcsr_build(g.n_rows, g.n_cols, rp, ci, va, pc.make_params(V=2, S=1, SG=16))
    s = torch.cuda.Stream()
    Bd = torch.from_numpy(B).cuda()
    Cd = torch.empty((g.n_rows, K), dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        pc.pcsr_spmm(h, Bd, Cd, K, s)
    s.synchronize()
    _check(Cd.cpu().numpy(), ref, bound, "device csr")
    h.close()


def test_unsplit_path_is_bit_reproducible_and_overwrites():
    g = _graph("rmat20")
    K = 32
    B, ref, bound = _oracle("rmat20", g, K, "normal")
    for V in (1, 2):
        a = _spmm(g, B, pc.make_params(V=V, S=0), K, prefill=float("nan"))
        b = _spmm(g, B, pc.make_params(V=V, S=0), K, prefill=123.0)
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
    # balancing on: rows are cleared before accumulation, whatever C held
    c = _spmm(g, B, pc.make_params(V=1, S=1, SG=8), K, prefill=1e30)
    _check(c, ref, bound, "S=1 prefilled")


def test_identity_and_all_ones_closed_forms():
    n, K = 1000, 48
    eye = synth.Graph("eye", n, n, np.arange(n + 1, dtype=np.int32), np.arange(n, dtype=np.int32),
                      np.ones(n, np.float32))
    B = synth.dense_operand(n, K, "normal", 1)
    for V in (1, 2):
        C = _spmm(eye, B, pc.make_params(V=V), K)
        assert np.array_equal(C.view(np.uint32), B.view(np.uint32))
    g = _graph("sbm")
    C = _spmm(g, np.ones((g.n_cols, 16), np.float32), pc.make_params(V=1, S=1, SG=8), 16)
    assert np.allclose(C, 1.0, rtol=0, atol=2e-6)


def test_long_row_accumulation_stays_in_tolerance():
    """One row with 150k nonzeros and all-ones B: the worst case for fp32 error growth."""
    n, L = 8, 150_000
    rowptr = np.zeros(n + 1, np.int32)
    rowptr[3:] = L
    g = synth.Graph("long", n, L, rowptr, np.arange(L, dtype=np.int32),
                    np.random.default_rng(0).uniform(0.5, 1.5, L).astype(np.float32))
    B = np.ones((L, 16), np.float32)
    ref, bound = oracle.spmm(g.rowptr, g.colidx, g.vals, B)
    for S in (0, 1):
        for kern in (None, (64, 1, 1, 1), (4, 4, 1, 4)):
            C = _spmm(g, B, pc.make_params(V=1, S=S, SG=64 if S else 0), 16, kernel=kern)
            _check(C, ref, bound, f"long row S={S} {kern}")


@pytest.mark.parametrize("V", [1, 2])
@pytest.mark.parametrize("K", [4, 6, 64, 68, 200])
def test_split_panels_with_many_items_are_reduced_by_a_workgroup(V, K):
    """Rows cut into 63 to 2000 items: panels with more than 64 partial rows are added up
    by a workgroup each (16 threads per vector of C, then their partial sums), the others by
    one thread per vector.  Both must match the oracle, give the same bits on a second run
    over different garbage, and the same bits from the host-built, the GPU-built and the
    column-ordered handle."""
    SG = 4
    lengths = [63 * SG, 64 * SG, 64 * SG + 1, 65 * SG, 66 * SG, 200 * SG + 3, 2000 * SG, 1, 0, 7, 129 * SG]
    if V == 2:
        lengths.append(300 * SG)  # an odd number of rows: the last panel has one row
    rng = np.random.default_rng(5 + K)
    n_cols = 9001
    rowptr = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int32)
    colidx = np.concatenate([np.sort(rng.choice(n_cols, L, replace=False)) for L in lengths]).astype(np.int32)
    vals = rng.uniform(-1.0, 1.0, colidx.shape[0]).astype(np.float32)
    g = synth.Graph("many_items", len(lengths), n_cols, rowptr, colidx, vals)
    B = synth.dense_operand(n_cols, K, "normal", 23)
    ref, bound = oracle.spmm(g.rowptr, g.colidx, g.vals, B)
    Bd = torch.from_numpy(B).cuda()
    outs = []
    for flags in (0, pc.PCSR_FLAG_GPU_BUILD, pc.PCSR_FLAG_COLUMN_ORDER):
        h = pc.pcsr_build(g.n_rows, g.n_cols, g.rowptr, g.colidx, g.vals,
                          pc.make_params(V=V, S=1, SG=SG, flags=flags))
        for fill in (float("nan"), -3e33):
            Cd = torch.full((g.n_rows, K), fill, dtype=torch.float32, device="cuda")
            pc.pcsr_spmm(h, Bd, Cd, K)
            torch.cuda.synchronize()
            outs.append(Cd.cpu().numpy())
        h.close()
    _check(outs[0], ref, bound, f"V={V} K={K}")
    for o in outs[1:]:
        assert np.array_equal(outs[0].view(np.uint32), o.view(np.uint32))


_FULL = {}


def _full_graph(name):
    """Full-size workloads are generated once per test process (rmat22 takes about a minute)."""
    if name not in _FULL:
        _FULL.clear()                            # keep at most one: rmat22 alone holds 1.5 GB
        _FULL[name] = synth.workload(name, "full")
    return _FULL[name]


def _sample_rows(g, n_random=20000):
    rng = np.random.default_rng(0)
    deg = g.degrees()
    return np.unique(np.concatenate([rng.integers(0, g.n_rows, n_random), [0, g.n_rows - 1],
                                     np.argsort(deg)[-50:], np.nonzero(deg == 0)[0][:50]]))


@pytest.mark.parametrize("name,K", [("poisson", 32), ("road", 128), ("rmat20", 64), ("sbm", 256),
                                    ("sbm_shuffled", 256), ("rmat22", 16), ("rmat22", 32), ("rmat22", 64),
                                    ("rmat22", 128)])
def test_full_size_sampled_rows(name, K):
    """Every benchmark workload at full size in the launch configuration bench.py times
    (the library's own pick); the oracle recomputes a sample of rows one by one, the
    longest rows and some empty ones included."""
    g = _full_graph(name)
    B = synth.dense_operand(g.n_cols, K, synth.WORKLOADS[name]["B"], 2)
    sel = pc.pcsr_select(pc.pcsr_features(g.n_rows, g.n_cols, g.rowptr, g.colidx), K)
    h = pc.pcsr_build(g.n_rows, g.n_cols, g.rowptr, g.colidx, g.vals, sel)
    print(f"case full {name} K={K} V={sel.V} S={sel.S} SG={sel.SG} {pc.pcsr_query_launch(h, K)}", flush=True)
    Bd = torch.from_numpy(B).cuda()
    Cd = torch.full((g.n_rows, K), float("nan"), dtype=torch.float32, device="cuda")
    pc.pcsr_spmm(h, Bd, Cd, K)
    torch.cuda.synchronize()
    rows = _sample_rows(g)
    ref, bound = oracle.spmm_rows(g.rowptr, g.colidx, g.vals, B, rows)
    got = Cd[torch.from_numpy(rows).cuda()].cpu().numpy()
    _check(got, ref, bound, f"{name} full sampled")
    # property that holds at any size: nothing left unwritten
    assert not torch.isnan(Cd).any().item()
    h.close()


@pytest.mark.parametrize("K", [256, 512])
def test_largest_workload_where_offsets_need_64_bits(K):
    """R-MAT scale 22 at the widths where B and C reach 2^32 bytes (K = 256) and 2^33 bytes, 2^31
    elements (K = 512): the library's own pick (the configuration bench.py times), the tuple the
    recorded sweeps rank first there (V=2, S=1, SG=1024), the same with the atomic
    write-back, and an unsplit V=1 tuple, each against oracle rows that include the
    162K-nonzero rows, the last row and 6000 random ones.  The balanced results must also
    be the same bits on a second run."""
    g = _full_graph("rmat22")
    assert g.n_rows * K * 4 >= 2**32
    B = synth.dense_operand(g.n_cols, K, "normal", 2)
    rows = _sample_rows(g, 6000)
    assert rows[-1] == g.n_rows - 1
    # many sampled rows start past 2^31 bytes (K = 256: signed 32-bit byte offsets would wrap) or
    # past 2^32 bytes (K = 512: unsigned ones would too; the last element index is 2^31 - 1)
    assert (rows.astype(np.int64) * K * 4 >= (2**31 if K == 256 else 2**32)).sum() > 1000
    ref, bound = oracle.spmm_rows(g.rowptr, g.colidx, g.vals, B, rows)
    Bd = torch.from_numpy(B).cuda()
    del B
    rows_d = torch.from_numpy(rows).cuda()
    Cd = torch.empty((g.n_rows, K), dtype=torch.float32, device="cuda")
    sel = pc.pcsr_select(pc.pcsr_features(g.n_rows, g.n_cols, g.rowptr, g.colidx), K)
    tuples = [("selected", sel, 0),
              ("V=2 S=1 SG=1024", pc.make_params(V=2, S=1, SG=1024, lanes_per_row=16, vec=4, rep=1, waves_per_wg=2), 0),
              ("V=2 S=1 SG=1024 atomic", None, pc.PCSR_FLAG_ATOMIC_SPLIT),
              ("V=1 S=0", pc.make_params(V=1, S=0, lanes_per_row=64, vec=4, rep=K // 256, waves_per_wg=4), 0)]
    h = None
    for what, params, kflags in tuples:
        if params is not None:
            if h is not None:
                h.close()
            h = pc.pcsr_build(g.n_rows, g.n_cols, g.rowptr, g.colidx, g.vals, params)
        else:
            pc.pcsr_set_kernel_params(h, 16, 4, 1, 2, 0, kflags)
        print(f"case rmat22 K={K} {what} {pc.pcsr_query_launch(h, K)}", flush=True)
        Cd.fill_(float("nan"))
        pc.pcsr_spmm(h, Bd, Cd, K)
        torch.cuda.synchronize()
        got = Cd[rows_d].cpu().numpy()
        _check(got, ref, bound, f"rmat22 K={K} {what}")
        assert not torch.isnan(Cd).any().item()
        if not kflags:
            first = Cd[rows_d].clone()
            tail = Cd[-4096:].clone()
            Cd.fill_(1e30)
            pc.pcsr_spmm(h, Bd, Cd, K)
            torch.cuda.synchronize()
            assert torch.equal(first.view(torch.int32), Cd[rows_d].view(torch.int32)), what
            assert torch.equal(tail.view(torch.int32), Cd[-4096:].view(torch.int32)), what
    h.close()


@pytest.mark.parametrize("name", ["rmat20", "rmat22", "sbm"])
@pytest.mark.parametrize("V", [1, 2])
def test_balanced_write_back_is_deterministic_and_needs_no_clean_output(name, V):
    """S = 1 without atomics: two runs over outputs prefilled with different garbage give
    identical bits; the handle built by GPU kernels and the one with the column-ordered
    schedule (which only changes when an item runs, not what it adds up) give the same bits
    as the host-built one; the atomic write-back stays within tolerance of the oracle."""
    g = _graph(name)
    K = 48
    B, ref, bound = _oracle(name, g, K, synth.WORKLOADS[name]["B"])
    Bd = torch.from_numpy(B).cuda()
    outs = []
    for flags in (0, pc.PCSR_FLAG_GPU_BUILD, pc.PCSR_FLAG_COLUMN_ORDER,
                  pc.PCSR_FLAG_COLUMN_ORDER | pc.PCSR_FLAG_NO_XCD_REMAP,
                  pc.PCSR_FLAG_COLUMN_ORDER | pc.PCSR_FLAG_GPU_BUILD):
        h = pc.pcsr_build(g.n_rows, g.n_cols, g.rowptr, g.colidx, g.vals, pc.make_params(V=V, S=1, SG=8, flags=flags))
        e = pc.pcsr_export(h)
        n_items = int(np.sum(np.bincount(e["trow"], minlength=e["P"])[np.bincount(e["trow"], minlength=e["P"]) > 1]))
        assert pc.pcsr_workspace_bytes(h, K) == n_items * V * K * 4
        for fill in (float("nan"), 1e30):
            Cd = torch.full((g.n_rows, K), fill, dtype=torch.float32, device="cuda")
            pc.pcsr_spmm(h, Bd, Cd, K)
            torch.cuda.synchronize()
            outs.append(Cd.cpu().numpy())
        pc.pcsr_set_kernel_params(h, flags=pc.PCSR_FLAG_ATOMIC_SPLIT)
        assert pc.pcsr_workspace_bytes(h, K) == 0
        Cd = torch.full((g.n_rows, K), float("nan"), dtype=torch.float32, device="cuda")
        pc.pcsr_spmm(h, Bd, Cd, K)
        torch.cuda.synchronize()
        _check(Cd.cpu().numpy(), ref, bound, f"{name} V={V} atomic write-back")
        h.close()
    _check(outs[0], ref, bound, f"{name} V={V} two-pass write-back")
    for o in outs[1:]:
        assert np.array_equal(outs[0].view(np.uint32), o.view(np.uint32))


@pytest.mark.parametrize("name", ["rmat20", "rmat22", "sbm", "poisson"])
@pytest.mark.parametrize("V,SG", [(1, 4), (2, 16), (1, 0)])
@pytest.mark.parametrize("device_csr", [False, True])
def test_column_ordered_schedule_built_on_the_gpu(name, V, SG, device_csr):
    """The schedule generated by GPU kernels equals the numpy restatement (and so the host
    builder's), and the handle computes the right product."""
    g = _graph(name)
    arrs = [g.rowptr, g.colidx, g.vals]
    flags = pc.PCSR_FLAG_COLUMN_ORDER
    if device_csr:
        arrs = [torch.from_numpy(x).cuda() for x in arrs]
    else:
        flags |= pc.PCSR_FLAG_GPU_BUILD
    h = pc.pcsr_build(g.n_rows, g.n_cols, *arrs, pc.make_params(V=V, S=1, SG=SG, flags=flags))
    e = pc.pcsr_export(h)
    got = pc.pcsr_export_schedule(h)
    sched, xb = column_ordered_schedule(e["rowptr"], e["colidx"], e["trow"], e["P"])
    assert np.array_equal(got["xcd_bounds"], xb)
    assert np.array_equal(got["sched"], sched)
    K = 24
    B, ref, bound = _oracle(name, g, K, synth.WORKLOADS[name]["B"])
    Cd = torch.full((g.n_rows, K), float("nan"), dtype=torch.float32, device="cuda")
    pc.pcsr_spmm(h, torch.from_numpy(B).cuda(), Cd, K)
    torch.cuda.synchronize()
    _check(Cd.cpu().numpy(), ref, bound, f"gpu-built column order {name} V={V} SG={SG}")
    h.close()


def test_workspace_grows_with_k_and_can_be_reserved_before_capture():
    g = _graph("rmat20")
    h = pc.pcsr_build(g.n_rows, g.n_cols, g.rowptr, g.colidx, g.vals, pc.make_params(V=1, S=1, SG=16))
    assert pc.pcsr_workspace_bytes(h, 64) == 4 * pc.pcsr_workspace_bytes(h, 16) > 0
    for K in (16, 64, 32):                       # grows once, then shrinking K reuses the block
        B, ref, bound = _oracle("rmat20", g, K, "normal")
        Cd = torch.full((g.n_rows, K), float("nan"), dtype=torch.float32, device="cuda")
        pc.pcsr_spmm(h, torch.from_numpy(B).cuda(), Cd, K)
        torch.cuda.synchronize()
        _check(Cd.cpu().numpy(), ref, bound, f"workspace K={K}")
    K = 128
    B, ref, bound = _oracle("rmat20", g, K, "normal")
    Bd = torch.from_numpy(B).cuda()
    Cd = torch.zeros((g.n_rows, K), dtype=torch.float32, device="cuda")
    pc.pcsr_reserve_workspace(h, K)              # instead of a warm-up call outside the capture
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        pc.pcsr_spmm(h, Bd, Cd, K, torch.cuda.current_stream())
    outs = []
    for replay in range(3):
        Cd.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        outs.append(Cd.clone())
        _check(Cd.cpu().numpy(), ref, bound, f"captured S=1 replay {replay}")
    assert torch.equal(outs[0], outs[1]) and torch.equal(outs[0], outs[2])
    h.close()
    h0 = pc.pcsr_build(g.n_rows, g.n_cols, g.rowptr, g.colidx, g.vals, pc.make_params(V=2, S=0))
    assert pc.pcsr_workspace_bytes(h0, 64) == 0
    h0.close()


def test_non_finite_b_row_stays_in_the_rows_that_reference_it():
    """A B row of +Inf may only reach the C rows whose A row has that column (V = 1: the
    format adds no padding): the batched walk must select, not multiply by zero."""
    g = _graph("road")
    K = 32
    B = synth.dense_operand(g.n_cols, K, "normal", 9).copy()
    bad_col = int(g.colidx[g.rowptr[g.n_rows // 2]])
    B[bad_col] = np.inf
    touched = np.zeros(g.n_rows, bool)
    touched[np.repeat(np.arange(g.n_rows), g.degrees())[g.colidx == bad_col]] = True
    ref, bound = oracle.spmm(g.rowptr, g.colidx, g.vals, B)
    assert np.isfinite(ref[~touched]).all() and not np.isfinite(ref[touched]).any()
    for kern in [(8, 4, 1, 2, 1), (8, 4, 1, 2, 2), (8, 4, 1, 2, 4), (16, 2, 1, 4, 4), (64, 1, 1, 1, 2)]:
        C = _spmm(g, B, pc.make_params(V=1, S=0), K, kernel=kern)
        assert np.isfinite(C[~touched]).all(), kern
        assert np.isposinf(ref[touched]).all() and np.isposinf(C[touched]).all(), kern
        ok, worst = oracle.within_tolerance(C[~touched], ref[~touched], bound[~touched], RTOL, ATOL)
        assert ok, (kern, worst)


@pytest.mark.parametrize("K", [48, 80, 96, 112, 144, 160, 176, 208, 240])
def test_widths_that_are_not_powers_of_two(K):
    """The paper sweeps dim in steps of 16 (Section 6.2); widths that leave a MAC-job gap
    (Eq. (1)) for every power-of-two tile must still be exact in every column."""
    g = _graph("rmat20")
    B, ref, bound = _oracle("rmat20", g, K, "normal")
    for params, kern in [(pc.make_params(V=1, S=0), None), (pc.make_params(V=2, S=1, SG=32), None),
                         (pc.make_params(V=1, S=1, SG=64), (8, 4, 1, 2)),     # several 32-column slices
                         (pc.make_params(V=1, S=0), (4, 4, 4, 4))]:
        C = _spmm(g, B, params, K, kernel=kern)
        _check(C, ref, bound, f"K={K} {kern}")
    f = pc.pcsr_features(g.n_rows, g.n_cols, g.rowptr, g.colidx)
    sel = pc.pcsr_select(f, K)
    C = _spmm(g, B, sel, K)
    _check(C, ref, bound, f"K={K} selected")


@pytest.mark.parametrize("name", ["poisson", "road", "rmat20", "sbm", "rmat22"])
@pytest.mark.parametrize("V", [1, 2])
@pytest.mark.parametrize("S,SG,omega", [(0, 0, 0), (1, 0, 0), (1, 0, 32), (1, 5, 0)])
@pytest.mark.parametrize("device_csr", [False, True])
def test_gpu_side_generation_bit_exact(name, V, S, SG, omega, device_csr):
    """PCSR arrays generated by GPU kernels equal the numpy format reference bit for bit."""
    g = _graph(name)
    if device_csr:
        arrs = [torch.from_numpy(x).cuda() for x in (g.rowptr, g.colidx, g.vals)]
        flags = 0
    else:
        arrs = [g.rowptr, g.colidx, g.vals]
        flags = pc.PCSR_FLAG_GPU_BUILD
    h = pc.pcsr_build(g.n_rows, g.n_cols, *arrs, pc.make_params(V=V, S=S, SG=SG, omega=omega, flags=flags))
    e = pc.pcsr_export(h)
    r = pf.pcsr_ref(g.n_rows, g.rowptr, g.colidx, g.vals, V, S, SG, omega or 64)
    for k in ("P", "M", "nnz_v", "V", "SG"):
        assert e[k] == r[k], k
    for k in ("rowptr", "colidx", "trow"):
        assert np.array_equal(e[k], r[k]), k
    assert np.array_equal(e["val"].view(np.uint32), r["val"].view(np.uint32))
    # and the handle computes the right product
    K = 16
    B, ref, bound = _oracle(name, g, K, synth.WORKLOADS[name]["B"])
    Cd = torch.full((g.n_rows, K), float("nan"), dtype=torch.float32, device="cuda")
    pc.pcsr_spmm(h, torch.from_numpy(B).cuda(), Cd, K)
    torch.cuda.synchronize()
    _check(Cd.cpu().numpy(), ref, bound, f"gpu build {name} V={V} S={S}")
    h.close()


def test_gpu_side_generation_degenerate_and_bad_input():
    G = pc.PCSR_FLAG_GPU_BUILD
    for n in (0, 1, 3):
        rowptr = np.zeros(n + 1, np.int32)
        for V in (1, 2):
            for S in (0, 1):
                h = pc.pcsr_build(n, 4, rowptr, np.zeros(0, np.int32), np.zeros(0, np.float32),
                                  pc.make_params(V=V, S=S, flags=G))
                e = pc.pcsr_export(h)
                r = pf.pcsr_ref(n, rowptr, np.zeros(0, np.int32), np.zeros(0, np.float32), V, S, 0, 64)
                assert e["M"] == r["M"] and np.array_equal(e["rowptr"], r["rowptr"])
                assert np.array_equal(e["trow"], r["trow"])
                h.close()
    rp = np.array([0, 2, 3], np.int32)
    va = np.ones(3, np.float32)
    for bad_cols in ([1, 0, 2], [1, 1, 2], [0, 3, 2], [0, -1, 2]):
        with pytest.raises(pc.PcsrError) as ei:
            pc.pcsr_build(2, 3, rp, np.array(bad_cols, np.int32), va, pc.make_params(flags=G))
        assert ei.value.code == pc.binding.PCSR_E_BAD_CSR
    with pytest.raises(pc.PcsrError) as ei:
        pc.pcsr_build(2, 3, np.array([0, 3, 2], np.int32), np.array([0, 1, 2], np.int32), va,
                      pc.make_params(flags=G))
    assert ei.value.code == pc.binding.PCSR_E_BAD_CSR


def test_spmm_argument_checks():
    g = _graph("poisson")
    h = pc.pcsr_build(g.n_rows, g.n_cols, g.rowptr, g.colidx, g.vals, pc.make_params())
    K = 32
    assert pc.pcsr_query_launch(h, K)["vec"] == 4
    buf = torch.zeros((g.n_rows + g.n_cols) * K + 8, dtype=torch.float32, device="cuda")
    lib = pc.binding._lib()
    base = buf.data_ptr()
    # overlapping B and C
    assert lib.pcsr_spmm(h.raw, base, base + 4 * K, K, None) == pc.binding.PCSR_E_INVALID_ARG
    # misaligned for float4 loads
    assert lib.pcsr_spmm(h.raw, base + 4, base + 4 * (g.n_cols * K + 4), K, None) == pc.binding.PCSR_E_INVALID_ARG
    assert lib.pcsr_spmm(h.raw, base, base + 4 * g.n_cols * K, 0, None) == pc.binding.PCSR_E_UNSUPPORTED
    assert lib.pcsr_spmm(h.raw, None, base, K, None) == pc.binding.PCSR_E_INVALID_ARG
    # adjacent but disjoint is fine
    assert lib.pcsr_spmm(h.raw, base, base + 4 * g.n_cols * K, K, None) == 0
    torch.cuda.synchronize()
    h.close()


@pytest.mark.parametrize("name", ["sbm_shuffled", "rmat20"])
def test_reordered_problem_gives_the_same_product(name):
    """A' = P A P^T, B' = P B  =>  C' = P C: the library's reorder + relabel against the
    oracle on the original problem."""
    g = _graph(name)
    K = 32
    B, ref, bound = _oracle(name, g, K, "normal")
    perm, _ = pc.pcsr_reorder(g.n_rows, g.rowptr, g.colidx)
    rp, ci, va = pc.pcsr_permute_csr(g.n_rows, g.rowptr, g.colidx, g.vals, perm)
    g2 = synth.Graph(name + "_r", g.n_rows, g.n_cols, rp, ci, va)
    B2 = np.empty_like(B)
    B2[perm] = B
    sel = pc.pcsr_select(pc.pcsr_features(g2.n_rows, g2.n_cols, rp, ci), K)
    C2 = _spmm(g2, B2, sel, K)
    _check(C2[perm], ref, bound, f"reordered {name}")


@pytest.mark.parametrize("V,S", [(1, 0), (2, 1)])
def test_spmm_can_be_captured_in_a_hip_graph(V, S):
    """pcsr_spmm allocates nothing and only launches kernels, so a launch-bound loop of
    SpMMs can be captured once and replayed; every replay must equal the eager result."""
    g = _graph("poisson")
    K = 32
    B, ref, bound = _oracle("poisson", g, K, "uniform")
    h = pc.pcsr_build(g.n_rows, g.n_cols, g.rowptr, g.colidx, g.vals, pc.make_params(V=V, S=S, SG=4 if S else 0))
    Bd = torch.from_numpy(B).cuda()
    Cd = torch.zeros((g.n_rows, K), dtype=torch.float32, device="cuda")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        pc.pcsr_spmm(h, Bd, Cd, K, side)          # warm-up outside the capture
    side.synchronize()
    eager = Cd.clone()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        for _ in range(4):
            pc.pcsr_spmm(h, Bd, Cd, K, torch.cuda.current_stream())
    for replay in range(3):
        Cd.fill_(float("nan"))                     # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        if S == 0:
            assert torch.equal(Cd, eager), f"replay {replay}"
        _check(Cd.cpu().numpy(), ref, bound, f"graph replay {replay} V={V} S={S}")
    h.close()


@pytest.mark.parametrize("K", [1, 2, 3, 6, 1000, 2048])
def test_extreme_widths(K):
    g = _graph("sbm")
    g = synth.Graph("sbm_head", 2000, g.n_cols, g.rowptr[:2001].copy(), g.colidx[:g.rowptr[2000]],
                    g.vals[:g.rowptr[2000]])
    B = synth.dense_operand(g.n_cols, K, "uniform", K)
    ref, bound = oracle.spmm(g.rowptr, g.colidx, g.vals, B)
    for V, S in [(1, 0), (2, 1)]:
        C = _spmm(g, B, pc.make_params(V=V, S=S, SG=16 if S else 0), K)
        _check(C, ref, bound, f"K={K} V={V} S={S}")


def test_two_handles_on_two_streams_concurrently():
    g1, g2 = _graph("rmat20"), _graph("road")
    K = 64
    B1, ref1, bound1 = _oracle("rmat20", g1, K, "normal")
    B2, ref2, bound2 = _oracle("road", g2, K, "normal")
    h1 = pc.pcsr_build(g1.n_rows, g1.n_cols, g1.rowptr, g1.colidx, g1.vals, pc.make_params(S=1, SG=32))
    h2 = pc.pcsr_build(g2.n_rows, g2.n_cols, g2.rowptr, g2.colidx, g2.vals, pc.make_params(V=2))
    B1d, B2d = torch.from_numpy(B1).cuda(), torch.from_numpy(B2).cuda()
    C1d = torch.empty((g1.n_rows, K), dtype=torch.float32, device="cuda")
    C2d = torch.empty((g2.n_rows, K), dtype=torch.float32, device="cuda")
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    for _ in range(10):
        pc.pcsr_spmm(h1, B1d, C1d, K, s1)
        pc.pcsr_spmm(h2, B2d, C2d, K, s2)
    s1.synchronize()
    s2.synchronize()
    _check(C1d.cpu().numpy(), ref1, bound1, "stream 1")
    _check(C2d.cpu().numpy(), ref2, bound2, "stream 2")
    h1.close()
    h2.close()


def test_seeded_random_configurations():
    """120 seeded random (matrix, K, format, launch shape) combinations against the oracle."""
    rng = np.random.default_rng(2024)
    done = 0
    for case in range(120):
        n_rows = int(rng.integers(1, 400))
        n_cols = int(rng.integers(1, 600))
        density = float(rng.choice([0.0, 0.01, 0.05, 0.3, 0.9]))
        rp, ci, va, _ = random_csr(rng, n_rows, n_cols, density,
                                   full_rows=(int(rng.integers(0, n_rows)),) if rng.random() < 0.3 else ())
        K = int(rng.choice([1, 2, 4, 7, 8, 12, 16, 24, 32, 48, 64, 100, 128, 132, 256]))
        V = int(rng.choice([1, 2]))
        S = int(rng.choice([0, 1]))
        SG = int(rng.choice([0, 1, 3, 64])) if S else 0
        cw = int(rng.choice([0, 0, 256, 512])) if not S else 0
        vec = int(rng.choice([v for v in (1, 2, 4) if K % v == 0]))
        lpr = int(rng.choice([4, 8, 16, 32, 64]))
        rep = int(rng.choice([1, 2, 4]))
        waves = int(rng.choice([1, 2, 4, 8]))
        ipg = int(rng.choice([1, 1, 2, 4])) if not S and not cw else 1
        flags = pc.PCSR_FLAG_NO_XCD_REMAP if rng.random() < 0.3 else 0
        if rng.random() < 0.3 and not cw:
            flags |= pc.PCSR_FLAG_GPU_BUILD
        if S and rng.random() < 0.4:
            flags |= pc.PCSR_FLAG_ATOMIC_SPLIT
        what = (f"case {case}: {n_rows}x{n_cols} d={density} K={K} V={V} S={S} SG={SG} cw={cw} "
                f"lpr={lpr} vec={vec} rep={rep} waves={waves} ipg={ipg} flags={flags}")
        print(what, flush=True)
        g = synth.Graph("rnd", n_rows, n_cols, rp, ci, va)
        h = pc.pcsr_build(n_rows, n_cols, rp, ci, va, pc.make_params(V=V, S=S, SG=SG, col_window=cw, flags=flags))
        pc.pcsr_set_kernel_params(h, lpr, vec, rep, waves, ipg,
                                  flags & (pc.PCSR_FLAG_NO_XCD_REMAP | pc.PCSR_FLAG_ATOMIC_SPLIT))
        # the refusals pcsr.h documents: items_per_group needs ipg < lanes and V*vec*rep*ipg <= 32,
        # the column window needs col_window + 1 rows of (lanes*vec*rep + 4) floats within 160 KiB of LDS
        refuse = (ipg > 1 and not (ipg < lpr and V * vec * rep * ipg <= 32)) or \
                 (cw > 0 and (cw + 1) * (lpr * vec * rep + 4) * 4 > 160 * 1024)
        try:
            q = pc.pcsr_query_launch(h, K)
        except pc.PcsrError as e:
            assert refuse and e.code == pc.binding.PCSR_E_UNSUPPORTED, what
            h.close()
            continue
        assert not refuse, what
        if q["grid_y"] > 64:
            h.close()
            continue
        B = synth.dense_operand(n_cols, K, "normal", case)
        ref, bound = oracle.spmm(rp, ci, va, B)
        Cd = torch.full((n_rows, K), float("nan"), dtype=torch.float32, device="cuda")
        pc.pcsr_spmm(h, torch.from_numpy(B).cuda(), Cd, K)
        torch.cuda.synchronize()
        _check(Cd.cpu().numpy(), ref, bound, what)
        h.close()
        done += 1
    assert done >= 80


def test_parameterised_kernel_reduces_to_algorithm_1_bit_for_bit():
    """Algorithm 2 with V=1, F=1, S=False is Algorithm 1 (Section 4.3).  On a matrix whose rows
    all fit one chunk the two walk each row's nonzeros in the same order with the same fused
    multiply-add, so the results must be identical bit patterns; the lane mapping (lanes per
    row, vector width, waves per workgroup) must not matter."""
    import ctypes

    from paper_2605_15695_amd import sweep as sw

    g = _graph("road")                                     # longest row: 8 nonzeros
    assert g.degrees().max() <= 8
    K = 96
    B, ref, bound = _oracle("road", g, K, "normal")
    lib = sw._baseline_lib()
    d = [torch.from_numpy(x).cuda() for x in (g.rowptr, g.colidx, g.vals)]
    Bd = torch.from_numpy(B).cuda()
    C1 = torch.full((g.n_rows, K), float("nan"), dtype=torch.float32, device="cuda")
    rc = lib.alg1_spmm(g.n_rows, d[0].data_ptr(), d[1].data_ptr(), d[2].data_ptr(), Bd.data_ptr(),
                       C1.data_ptr(), K, 4, None)
    assert rc == 0
    torch.cuda.synchronize()
    _check(C1.cpu().numpy(), ref, bound, "Algorithm 1 baseline")
    h = pc.pcsr_build(g.n_rows, g.n_cols, g.rowptr, g.colidx, g.vals, pc.make_params(V=1, S=0))
    for kern in [(64, 1, 1, 4), (8, 4, 1, 2), (16, 2, 1, 1), (32, 1, 1, 8), (8, 4, 4, 4)]:
        pc.pcsr_set_kernel_params(h, *kern)
        C2 = torch.full((g.n_rows, K), float("nan"), dtype=torch.float32, device="cuda")
        pc.pcsr_spmm(h, Bd, C2, K)
        torch.cuda.synchronize()
        assert torch.equal(C1.view(torch.int32), C2.view(torch.int32)), kern
    h.close()


@pytest.mark.parametrize("name", ["poisson", "road", "rmat20", "sbm", "rmat22"])
@pytest.mark.parametrize("omega", [32, 64])
def test_gpu_side_features_match_reference(name, omega):
    g = _graph(name)
    f = pc.pcsr_features(g.n_rows, g.n_cols, torch.from_numpy(g.rowptr).cuda(),
                         torch.from_numpy(g.colidx).cuda(), omega)
    r = pf.features(g.n_rows, g.n_cols, g.rowptr, g.colidx, omega)
    assert np.allclose(f[:16], r, rtol=1e-11, atol=0), (f, r)
    assert f[16] == pytest.approx(near_diagonal_share(g.rowptr, g.colidx), rel=1e-12)
    assert np.array_equal(f, pc.pcsr_features(g.n_rows, g.n_cols, g.rowptr, g.colidx, omega)) or \
        np.allclose(f, pc.pcsr_features(g.n_rows, g.n_cols, g.rowptr, g.colidx, omega), rtol=1e-11)
    # degenerate shapes
    z = pc.pcsr_features(3, 5, torch.zeros(4, dtype=torch.int32, device="cuda"),
                         torch.zeros(0, dtype=torch.int32, device="cuda"), omega)
    assert np.array_equal(z[:16], pf.features(3, 5, np.zeros(4, np.int32), np.zeros(0, np.int32), omega))
    assert z[16] == 0.0
