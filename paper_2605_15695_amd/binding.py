"""Thin ctypes binding of libpcsr.so: argument marshalling only, same names as the C ABI.

Every step of the path runs inside the library.  torch is used by callers for device
memory and streams; this module only reads `data_ptr()` / `cuda_stream` from them.
"""
from __future__ import annotations

import ctypes
import pathlib

import numpy as np

_PKG = pathlib.Path(__file__).resolve().parent
LIB_PATH = _PKG / "libpcsr.so"

PCSR_OK = 0
PCSR_E_INVALID_ARG, PCSR_E_BAD_CSR, PCSR_E_UNSUPPORTED = -1, -2, -3
PCSR_E_TOO_LARGE, PCSR_E_OOM, PCSR_E_HIP = -4, -5, -6
PCSR_FLAG_DEVICE_CSR, PCSR_FLAG_NO_VALIDATE, PCSR_FLAG_NO_XCD_REMAP, PCSR_FLAG_HOST_ONLY = 1, 2, 4, 8
PCSR_FLAG_GPU_BUILD = 16
PCSR_FLAG_ATOMIC_SPLIT = 32
PCSR_FLAG_COLUMN_ORDER = 64
PCSR_FLAG_WINDOW_IF_USEFUL = 128
PCSR_N_FEATURES = 17
FEATURE_NAMES = ("n", "n_hat", "nnz", "delta", "d", "d_hat", "d_max", "CV", "CV_hat",
                 "SR_1", "SR_2", "rho", "b", "b_max", "PR_1", "PR_2", "near_512")


class pcsr_params_t(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("V", "S", "SG", "omega", "lanes_per_row", "vec", "rep", "waves_per_wg", "flags",
                 "items_per_group", "col_window")]
    _fields_ += [("reserved", ctypes.c_int32 * 1)]


class PcsrError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        msg = _lib().pcsr_strerror(code).decode()
        if code == PCSR_E_HIP:
            msg += f" (hipError {_lib().pcsr_last_hip_error()})"
        super().__init__(f"{where}: {msg} [{code}]")


_LIB = None


def _lib():
    global _LIB
    if _LIB is None:
        if not LIB_PATH.exists():
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2605_15695_amd.build` "
                "(there is no CPU fallback)")
        lib = ctypes.CDLL(str(LIB_PATH))
        i64, i32, vp = ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p
        pp = ctypes.POINTER(pcsr_params_t)
        lib.pcsr_build.argtypes = [i64, i64, i64, vp, vp, vp, pp, ctypes.POINTER(vp)]
        lib.pcsr_spmm.argtypes = [vp, vp, vp, i32, vp]
        lib.pcsr_free.argtypes = [vp]
        lib.pcsr_spmm_static.argtypes = [vp, vp, vp, i32, vp]
        lib.pcsr_static_scratch_bytes.restype = i64
        lib.pcsr_workspace_bytes.argtypes = [vp, i32, ctypes.POINTER(i64)]
        lib.pcsr_reserve_workspace.argtypes = [vp, i32]
        lib.pcsr_set_kernel_params.argtypes = [vp, i32, i32, i32, i32, i32, i32]
        lib.pcsr_query_launch.argtypes = [vp, i32, ctypes.POINTER(i32 * 8)]
        lib.pcsr_window_stats.argtypes = [vp, ctypes.POINTER(ctypes.c_double * 3)]
        lib.pcsr_export.argtypes = [vp, ctypes.POINTER(i64 * 6), vp, vp, vp, vp]
        lib.pcsr_export_schedule.argtypes = [vp, ctypes.POINTER(i64), vp, vp]
        lib.pcsr_features.argtypes = [i64, i64, i64, vp, vp, i32, vp, i32]
        lib.pcsr_features_device.argtypes = [i64, i64, i64, vp, vp, i32, vp, i32]
        lib.pcsr_select.argtypes = [vp, i32, pp]
        lib.pcsr_reorder.argtypes = [i64, vp, vp, i32, vp, ctypes.POINTER(i64)]
        lib.pcsr_permute_csr.argtypes = [i64, vp, vp, vp, vp, vp, vp, vp]
        lib.pcsr_reorder_by_degree.argtypes = [i64, vp, vp, vp]
        lib.pcsr_transpose_csr.argtypes = [i64, i64, vp, vp, vp, vp, vp, vp]
        lib.pcsr_mac_job_gap.argtypes = [i32, i32, i32]
        lib.pcsr_mac_job_gap.restype = i32
        lib.pcsr_strerror.argtypes = [ctypes.c_int]
        lib.pcsr_strerror.restype = ctypes.c_char_p
        lib.pcsr_last_hip_error.restype = ctypes.c_int
        for name in ("pcsr_build", "pcsr_spmm", "pcsr_free", "pcsr_set_kernel_params",
                     "pcsr_query_launch", "pcsr_export", "pcsr_features", "pcsr_select",
                     "pcsr_window_stats", "pcsr_features_device", "pcsr_reorder", "pcsr_permute_csr",
                     "pcsr_transpose_csr", "pcsr_workspace_bytes", "pcsr_reserve_workspace", "pcsr_spmm_static",
                     "pcsr_export_schedule", "pcsr_reorder_by_degree"):
            getattr(lib, name).restype = ctypes.c_int
        _LIB = lib
    return _LIB


def _ptr(a, dtype=None):
    """Address of a numpy array or torch tensor (contiguous, right dtype); (keepalive, ptr, is_device)."""
    if a is None:
        return None, None, False
    if isinstance(a, np.ndarray):
        if dtype is not None and a.dtype != dtype:
            a = a.astype(dtype)
        a = np.ascontiguousarray(a)
        return a, a.ctypes.data, False
    # torch tensor
    if not a.is_contiguous():
        raise ValueError("tensor must be contiguous")
    if dtype is not None and np.dtype(str(a.dtype).replace("torch.", "")) != dtype:
        raise ValueError(f"tensor dtype {a.dtype} != {dtype}")
    return a, a.data_ptr(), a.is_cuda


def make_params(V=1, S=0, SG=0, omega=0, lanes_per_row=0, vec=0, rep=0, waves_per_wg=0, flags=0,
                items_per_group=0, col_window=0):
    p = pcsr_params_t()
    p.V, p.S, p.SG, p.omega = V, int(S), SG, omega
    p.lanes_per_row, p.vec, p.rep, p.waves_per_wg, p.flags = lanes_per_row, vec, rep, waves_per_wg, flags
    p.items_per_group = items_per_group
    p.col_window = col_window
    return p


class Handle:
    """Owns a pcsr_handle_t; freed on close() or garbage collection."""

    def __init__(self, raw, n_rows, n_cols):
        self.raw = raw
        self.n_rows, self.n_cols = n_rows, n_cols

    def close(self):
        if self.raw:
            pcsr_free(self)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def pcsr_build(n_rows, n_cols, rowptr, colidx, vals, params=None) -> Handle:
    k0, p_r, dev_r = _ptr(rowptr, np.dtype(np.int32))
    k1, p_c, dev_c = _ptr(colidx, np.dtype(np.int32))
    k2, p_v, dev_v = _ptr(vals, np.dtype(np.float32))
    nnz = int(k1.shape[0]) if k1 is not None else 0
    if int(k0.shape[0]) != n_rows + 1:
        raise ValueError("rowptr must have n_rows + 1 entries")
    if k2 is not None and int(k2.shape[0]) != nnz:
        raise ValueError("vals and colidx differ in length")
    p = pcsr_params_t()                      # a copy: the caller's struct is left as it is
    ctypes.memmove(ctypes.byref(p), ctypes.byref(params if params is not None else make_params()),
                   ctypes.sizeof(p))
    if dev_r or dev_c or dev_v:
        if not (dev_r and dev_c and dev_v):
            raise ValueError("CSR arrays must be all host or all device")
        p.flags |= PCSR_FLAG_DEVICE_CSR
    out = ctypes.c_void_p()
    rc = _lib().pcsr_build(n_rows, n_cols, nnz, p_r, p_c, p_v, ctypes.byref(p), ctypes.byref(out))
    if rc != PCSR_OK:
        raise PcsrError(rc, "pcsr_build")
    return Handle(out.value, n_rows, n_cols)


def pcsr_spmm(h: Handle, B, C, K: int, stream=None) -> None:
    """B, C: torch device tensors (fp32, contiguous).  stream: torch.cuda.Stream, raw handle or None."""
    _, p_b, dev_b = _ptr(B, np.dtype(np.float32))
    _, p_c, dev_c = _ptr(C, np.dtype(np.float32))
    if not (dev_b and dev_c):
        raise ValueError("B and C must be device tensors")
    if B.numel() != h.n_cols * K or C.numel() != h.n_rows * K:
        raise ValueError("B must be n_cols x K and C n_rows x K")
    s = getattr(stream, "cuda_stream", stream)
    rc = _lib().pcsr_spmm(h.raw, p_b, p_c, K, s)
    if rc != PCSR_OK:
        raise PcsrError(rc, "pcsr_spmm")


def pcsr_workspace_bytes(h: Handle, K: int) -> int:
    out = ctypes.c_int64(0)
    rc = _lib().pcsr_workspace_bytes(h.raw, K, ctypes.byref(out))
    if rc != PCSR_OK:
        raise PcsrError(rc, "pcsr_workspace_bytes")
    return int(out.value)


def pcsr_reserve_workspace(h: Handle, K: int) -> None:
    rc = _lib().pcsr_reserve_workspace(h.raw, K)
    if rc != PCSR_OK:
        raise PcsrError(rc, "pcsr_reserve_workspace")


def pcsr_spmm_static(h: Handle, B, C, K: int, stream=None) -> None:
    """pcsr_spmm with the library's fixed workspace: allocates nothing."""
    _, p_b, dev_b = _ptr(B, np.dtype(np.float32))
    _, p_c, dev_c = _ptr(C, np.dtype(np.float32))
    if not (dev_b and dev_c):
        raise ValueError("B and C must be device tensors")
    if B.numel() != h.n_cols * K or C.numel() != h.n_rows * K:
        raise ValueError("B must be n_cols x K and C n_rows x K")
    s = getattr(stream, "cuda_stream", stream)
    rc = _lib().pcsr_spmm_static(h.raw, p_b, p_c, K, s)
    if rc != PCSR_OK:
        raise PcsrError(rc, "pcsr_spmm_static")


def pcsr_static_scratch_bytes() -> int:
    return int(_lib().pcsr_static_scratch_bytes())


def pcsr_free(h: Handle) -> None:
    raw, h.raw = h.raw, None
    rc = _lib().pcsr_free(raw)
    if rc != PCSR_OK:
        raise PcsrError(rc, "pcsr_free")


def pcsr_set_kernel_params(h: Handle, lanes_per_row=0, vec=0, rep=0, waves_per_wg=0,
                           items_per_group=0, flags=0) -> None:
    rc = _lib().pcsr_set_kernel_params(h.raw, lanes_per_row, vec, rep, waves_per_wg, items_per_group, flags)
    if rc != PCSR_OK:
        raise PcsrError(rc, "pcsr_set_kernel_params")


def pcsr_query_launch(h: Handle, K: int) -> dict:
    out = (ctypes.c_int32 * 8)()
    rc = _lib().pcsr_query_launch(h.raw, K, ctypes.byref(out))
    if rc != PCSR_OK:
        raise PcsrError(rc, "pcsr_query_launch")
    return dict(zip(("lanes_per_row", "vec", "rep", "waves_per_wg", "grid_x", "grid_y", "items_per_group",
                     "lds_bytes"), list(out)))


def pcsr_window_stats(h: Handle) -> dict:
    out = (ctypes.c_double * 3)()
    rc = _lib().pcsr_window_stats(h.raw, ctypes.byref(out))
    if rc != PCSR_OK:
        raise PcsrError(rc, "pcsr_window_stats")
    return dict(col_window=int(out[0]), items_per_block=float(out[1]), hit_fraction=float(out[2]))


def pcsr_export(h: Handle) -> dict:
    sizes = (ctypes.c_int64 * 6)()
    rc = _lib().pcsr_export(h.raw, ctypes.byref(sizes), None, None, None, None)
    if rc != PCSR_OK:
        raise PcsrError(rc, "pcsr_export")
    P, M, nnz_v, V, SG, has_trow = list(sizes)
    rowptr = np.empty(M + 1, np.int32)
    colidx = np.empty(nnz_v, np.int32)
    val = np.empty(nnz_v * V, np.float32)
    trow = np.empty(M if has_trow else 0, np.int32)
    rc = _lib().pcsr_export(h.raw, ctypes.byref(sizes), rowptr.ctypes.data, colidx.ctypes.data,
                            val.ctypes.data, trow.ctypes.data if has_trow else None)
    if rc != PCSR_OK:
        raise PcsrError(rc, "pcsr_export")
    return dict(P=P, M=M, nnz_v=nnz_v, V=V, SG=SG, rowptr=rowptr, colidx=colidx, val=val, trow=trow)


def pcsr_export_schedule(h: Handle) -> dict:
    """xcd_bounds int32[9] and, for a column-ordered handle, sched int32[M, 4] (else None)."""
    n = ctypes.c_int64(0)
    xb = np.zeros(9, np.int32)
    rc = _lib().pcsr_export_schedule(h.raw, ctypes.byref(n), None, xb.ctypes.data)
    if rc != PCSR_OK:
        raise PcsrError(rc, "pcsr_export_schedule")
    sched = None
    if n.value:
        sched = np.empty((n.value, 4), np.int32)
        rc = _lib().pcsr_export_schedule(h.raw, ctypes.byref(n), sched.ctypes.data, xb.ctypes.data)
        if rc != PCSR_OK:
            raise PcsrError(rc, "pcsr_export_schedule")
    return dict(xcd_bounds=xb, sched=sched)


def pcsr_features(n_rows, n_cols, rowptr, colidx, omega=0) -> np.ndarray:
    """Table 3 features; device tensors are routed to the GPU implementation."""
    k0, p_r, dev_r = _ptr(rowptr, np.dtype(np.int32))
    k1, p_c, dev_c = _ptr(colidx, np.dtype(np.int32))
    out = np.empty(PCSR_N_FEATURES, np.float64)
    if dev_r or dev_c:
        if not (dev_r and dev_c):
            raise ValueError("rowptr and colidx must be both host or both device")
        rc = _lib().pcsr_features_device(n_rows, n_cols, int(k1.shape[0]), p_r, p_c, omega, out.ctypes.data,
                                         PCSR_N_FEATURES)
        if rc != PCSR_OK:
            raise PcsrError(rc, "pcsr_features_device")
        return out
    rc = _lib().pcsr_features(n_rows, n_cols, int(k1.shape[0]), p_r, p_c, omega, out.ctypes.data,
                              PCSR_N_FEATURES)
    if rc != PCSR_OK:
        raise PcsrError(rc, "pcsr_features")
    return out


def pcsr_select(features, K: int) -> pcsr_params_t:
    f = np.ascontiguousarray(features, dtype=np.float64)
    if f.shape[0] < PCSR_N_FEATURES:
        raise ValueError("features too short")
    p = pcsr_params_t()
    rc = _lib().pcsr_select(f.ctypes.data, K, ctypes.byref(p))
    if rc != PCSR_OK:
        raise PcsrError(rc, "pcsr_select")
    return p


def pcsr_reorder(n, rowptr, colidx, max_rounds=0):
    """Returns (perm int32[n] with perm[old] = new, number of clusters)."""
    k0, p_r, _ = _ptr(rowptr, np.dtype(np.int32))
    k1, p_c, _ = _ptr(colidx, np.dtype(np.int32))
    perm = np.empty(n, np.int32)
    ncl = ctypes.c_int64(0)
    rc = _lib().pcsr_reorder(n, p_r, p_c, max_rounds, perm.ctypes.data, ctypes.byref(ncl))
    if rc != PCSR_OK:
        raise PcsrError(rc, "pcsr_reorder")
    return perm, int(ncl.value)


def pcsr_reorder_by_degree(n, rowptr, colidx):
    """perm int32[n] with perm[old] = new: nodes by descending in-degree."""
    k0, p_r, _ = _ptr(rowptr, np.dtype(np.int32))
    k1, p_c, _ = _ptr(colidx, np.dtype(np.int32))
    perm = np.empty(n, np.int32)
    rc = _lib().pcsr_reorder_by_degree(n, p_r, p_c, perm.ctypes.data)
    if rc != PCSR_OK:
        raise PcsrError(rc, "pcsr_reorder_by_degree")
    return perm


def pcsr_permute_csr(n, rowptr, colidx, vals, perm):
    """Symmetric relabelling P A P^T; returns (rowptr, colidx, vals) of the relabelled matrix."""
    k0, p_r, _ = _ptr(rowptr, np.dtype(np.int32))
    k1, p_c, _ = _ptr(colidx, np.dtype(np.int32))
    k2, p_v, _ = _ptr(vals, np.dtype(np.float32))
    k3, p_p, _ = _ptr(perm, np.dtype(np.int32))
    if int(k3.shape[0]) != n:
        raise ValueError("perm must have n entries")
    o_r = np.empty(n + 1, np.int32)
    o_c = np.empty(k1.shape[0], np.int32)
    o_v = np.empty(k1.shape[0], np.float32)
    rc = _lib().pcsr_permute_csr(n, p_r, p_c, p_v, p_p, o_r.ctypes.data, o_c.ctypes.data, o_v.ctypes.data)
    if rc != PCSR_OK:
        raise PcsrError(rc, "pcsr_permute_csr")
    return o_r, o_c, o_v


def pcsr_transpose_csr(n_rows, n_cols, rowptr, colidx, vals):
    """CSR of A^T; returns (rowptr int32[n_cols+1], colidx, vals)."""
    k0, p_r, _ = _ptr(rowptr, np.dtype(np.int32))
    k1, p_c, _ = _ptr(colidx, np.dtype(np.int32))
    k2, p_v, _ = _ptr(vals, np.dtype(np.float32))
    o_r = np.empty(n_cols + 1, np.int32)
    o_c = np.empty(k1.shape[0], np.int32)
    o_v = np.empty(k1.shape[0], np.float32)
    rc = _lib().pcsr_transpose_csr(n_rows, n_cols, p_r, p_c, p_v, o_r.ctypes.data, o_c.ctypes.data,
                                   o_v.ctypes.data)
    if rc != PCSR_OK:
        raise PcsrError(rc, "pcsr_transpose_csr")
    return o_r, o_c, o_v


def pcsr_mac_job_gap(dim: int, F: int, omega: int) -> int:
    return int(_lib().pcsr_mac_job_gap(dim, F, omega))


def pcsr_strerror(code: int) -> str:
    return _lib().pcsr_strerror(code).decode()
