"""CPU checks of the measurement helpers: shape enumeration of the sweep, the report."""
import io
import json
from contextlib import redirect_stdout

from paper_2605_15695_amd import report, sweep


def test_kernel_shapes_cover_k_without_idle_repeats():
    for K in (16, 32, 48, 64, 96, 128, 160, 256, 512, 33):
        shapes = sweep.kernel_shapes(K, quick=False)
        assert shapes
        for lpr, vec, rep in shapes:
            assert K % vec == 0
            tile = lpr * vec * rep
            assert tile * 8 >= K                       # at most 8 grid.y slices
            assert lpr * vec * (rep - 1) < K           # no repeat entirely past K
    quick = sweep.kernel_shapes(128, quick=True)
    # the widest load, plus the two 64-column slices made of narrow loads
    assert quick and all(v == 4 or (l, v, r) in ((32, 2, 1), (64, 1, 1)) for l, v, r in quick)
    assert (32, 2, 1) in quick and (64, 1, 1) in quick
    assert {v for _, v, _ in sweep.kernel_shapes(32, quick=True)} == {1, 2, 4}


def test_report_table_and_geomean(tmp_path):
    base = dict(workload="w", size="full", K=64, nnz=1000, n=100, bytes_min=10_000)
    recs = [
        dict(base, kind="pcsr", V=1, S=0, SG=0, lanes_per_row=16, vec=4, rep=1, waves_per_wg=4,
             items_per_group=1, ms_median=0.5, gflops=256.0, roofline_frac=0.25),
        dict(base, kind="pcsr", V=2, S=0, SG=0, lanes_per_row=16, vec=4, rep=1, waves_per_wg=4,
             items_per_group=1, ms_median=1.0, gflops=128.0, roofline_frac=0.125),
        dict(base, kind="hipsparse", alg="default", ms_median=2.0),
        dict(base, kind="selected", ms_median=0.625),
    ]
    p = tmp_path / "s.jsonl"
    p.write_text("\n".join(json.dumps(r) for r in recs) + "\n")
    out = io.StringIO()
    with redirect_stdout(out):
        assert report.main([str(p)]) == 0
    text = out.getvalue()
    assert "| w | 64 | 100 | 1000 | 1,0,0 / 16,4,1,4,1 | 0.5000 |" in text and text.count("| - |") == 1
    assert "4.00x" in text and "**4.00x**" in text and "80.0 %" in text
