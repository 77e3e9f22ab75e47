"""CPU oracle package: TEST INFRASTRUCTURE ONLY.

`spmm` / `spmm_rows` wrap the plain C routine in spmm_oracle.c (fp64, row by row over
the input CSR; Section 2 problem statement and the loop of Algorithm 1).
`pcsr_format` is the numpy reference of the PCSR arrays and of Eqs. (1)-(4) / Table 3.
Nothing here is imported by the product package; only tests/, the smoke check and the
bench's cpu_baseline leg use it.
"""
from __future__ import annotations

import ctypes

import numpy as np

from . import pcsr_format  # noqa: F401
from .build import build as _build

_LIB = None


def _lib():
    global _LIB
    if _LIB is None:
        lib = ctypes.CDLL(str(_build(force=False)))
        i64, i32, vp = ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p
        lib.oracle_spmm_csr.argtypes = [i64, vp, vp, vp, vp, i64, vp, vp, i32]
        lib.oracle_spmm_csr.restype = ctypes.c_int
        lib.oracle_spmm_csr_rows.argtypes = [vp, vp, vp, vp, i64, vp, i64, vp, vp, i32]
        lib.oracle_spmm_csr_rows.restype = ctypes.c_int
        lib.oracle_max_threads.restype = ctypes.c_int
        _LIB = lib
    return _LIB


def _c(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a, a.ctypes.data


def max_threads() -> int:
    return int(_lib().oracle_max_threads())


def spmm(rowptr, colidx, vals, B, want_bound=True, n_threads=0):
    """C_ref (fp64) and bound = sum |a*b| (fp64) for every row.  B is (n_cols, K) fp32."""
    rowptr, p_r = _c(rowptr, np.int32)
    colidx, p_c = _c(colidx, np.int32)
    vals, p_v = _c(vals, np.float32)
    B, p_b = _c(B, np.float32)
    n = rowptr.shape[0] - 1
    K = B.shape[1]
    if colidx.size:
        assert 0 <= int(colidx.min()) and int(colidx.max()) < B.shape[0]
    C = np.empty((n, K), dtype=np.float64)
    bound = np.empty((n, K), dtype=np.float64) if want_bound else None
    rc = _lib().oracle_spmm_csr(n, p_r, p_c, p_v, p_b, K, C.ctypes.data,
                                bound.ctypes.data if want_bound else None, n_threads)
    assert rc == 0
    return C, bound


def spmm_rows(rowptr, colidx, vals, B, rows, n_threads=0):
    """C_ref and bound for the selected output rows only."""
    rowptr, p_r = _c(rowptr, np.int32)
    colidx, p_c = _c(colidx, np.int32)
    vals, p_v = _c(vals, np.float32)
    B, p_b = _c(B, np.float32)
    rows, p_rows = _c(rows, np.int64)
    K = B.shape[1]
    C = np.empty((rows.shape[0], K), dtype=np.float64)
    bound = np.empty((rows.shape[0], K), dtype=np.float64)
    rc = _lib().oracle_spmm_csr_rows(p_r, p_c, p_v, p_b, K, p_rows, rows.shape[0],
                                     C.ctypes.data, bound.ctypes.data, n_threads)
    assert rc == 0
    return C, bound


def within_tolerance(C_test, C_ref, bound, rtol=1e-5, atol=1e-6):
    """Element-wise acceptance |C - C_ref| <= rtol*bound + atol; returns (ok, worst ratio)."""
    err = np.abs(np.asarray(C_test, dtype=np.float64) - C_ref)
    lim = rtol * bound + atol
    ratio = float((err / lim).max()) if err.size else 0.0
    return bool(np.all(err <= lim)) and np.all(np.isfinite(C_test)), ratio
