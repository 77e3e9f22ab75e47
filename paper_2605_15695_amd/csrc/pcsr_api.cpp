// C ABI of the PCSR SpMM library (see include/pcsr.h for the contract of each call).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstring>
#include <new>
#include <vector>

#include "../../include/pcsr.h"
#include "pcsr_build_gpu.h"
#include "pcsr_host.h"
#include "pcsr_kernels.h"

namespace {

constexpr uint32_t kMagic = 0x50435352u; // "PCSR"

thread_local int g_last_hip = 0;

inline bool hip_ok(hipError_t e)
{
    if (e == hipSuccess) return true;
    g_last_hip = (int)e;
    (void)hipGetLastError(); // clear the sticky error so later calls are not blamed
    return false;
}

inline bool is_pow2(int x) { return x > 0 && (x & (x - 1)) == 0; }

int check_kernel_params(int lpr, int vec, int rep, int waves, int ipg)
{
    if (ipg != 0 && ipg != 1 && ipg != 2 && ipg != 4) return PCSR_E_UNSUPPORTED;
    if (lpr != 0 && !(is_pow2(lpr) && lpr >= 4 && lpr <= 64)) return PCSR_E_UNSUPPORTED;
    if (vec != 0 && vec != 1 && vec != 2 && vec != 4) return PCSR_E_UNSUPPORTED;
    if (rep != 0 && rep != 1 && rep != 2 && rep != 4) return PCSR_E_UNSUPPORTED;
    if (waves != 0 && waves != 1 && waves != 2 && waves != 4 && waves != 8 && waves != 16)
        return PCSR_E_UNSUPPORTED;
    return PCSR_OK;
}

} // namespace

struct pcsr_handle_s {
    uint32_t magic = kMagic;
    pcsr::HostPcsr host; // arrays kept only for host-only handles; scalars always valid
    bool host_only = false;
    int device = -1;
    int32_t *d_rowptr = nullptr;
    int32_t *d_colidx = nullptr;
    float *d_val = nullptr;
    int32_t *d_trow = nullptr;
    int32_t *d_split = nullptr;       // panels that own more than one item, ascending
    int32_t *d_item_slot = nullptr;   // per item: workspace slot, -1 for a sole item (S only)
    int32_t *d_sched = nullptr;       // column-ordered schedule: 4 int32 per launch position
    int32_t *d_split_slot = nullptr;  // their first workspace slots (n_split + 1 entries)
    int32_t *d_long = nullptr;        // positions in d_split of panels with more than kLongPanelSlots items
    int64_t n_long = 0;
    int32_t *d_win = nullptr;     // window start per item block
    int32_t *d_win_ptr = nullptr; // item range per item block
    int32_t *d_win_lo = nullptr;  // per item: run of vectors inside the block's window
    int32_t *d_win_hi = nullptr;
    int64_t n_win_blocks = 0;
    int64_t n_split = 0;
    int64_t n_split_items = 0; // workspace slots: items that belong to split panels
    float *d_ws = nullptr;     // partial rows of those items, grown on demand
    size_t ws_bytes = 0;
    int32_t lpr = 0, vec = 0, rep = 0, waves = 0, ipg = 0, flags = 0;
};

namespace {

inline bool valid(pcsr_handle_t h) { return h && h->magic == kMagic; }

void release_device(pcsr_handle_t h)
{
    if (h->d_rowptr) (void)hipFree(h->d_rowptr);
    if (h->d_colidx) (void)hipFree(h->d_colidx);
    if (h->d_val) (void)hipFree(h->d_val);
    if (h->d_trow) (void)hipFree(h->d_trow);
    if (h->d_split) (void)hipFree(h->d_split);
    if (h->d_item_slot) (void)hipFree(h->d_item_slot);
    if (h->d_sched) (void)hipFree(h->d_sched);
    if (h->d_split_slot) (void)hipFree(h->d_split_slot);
    if (h->d_long) (void)hipFree(h->d_long);
    if (h->d_win) (void)hipFree(h->d_win);
    if (h->d_win_ptr) (void)hipFree(h->d_win_ptr);
    if (h->d_win_lo) (void)hipFree(h->d_win_lo);
    if (h->d_win_hi) (void)hipFree(h->d_win_hi);
    if (h->d_ws) (void)hipFree(h->d_ws);
    h->d_rowptr = h->d_colidx = h->d_trow = h->d_split = h->d_win = nullptr;
    h->d_item_slot = h->d_sched = h->d_split_slot = h->d_long = h->d_win_ptr = nullptr;
    h->d_win_lo = h->d_win_hi = nullptr;
    h->d_val = h->d_ws = nullptr;
    h->ws_bytes = 0;
}

template <class T> int upload(const std::vector<T> &src, T **dst)
{
    *dst = nullptr;
    // one spare element so empty arrays still have a valid device address
    size_t bytes = (src.size() + 1) * sizeof(T);
    hipError_t e = hipMalloc((void **)dst, bytes);
    if (e == hipErrorOutOfMemory) {
        (void)hipGetLastError();
        return PCSR_E_OOM;
    }
    if (!hip_ok(e)) return PCSR_E_HIP;
    if (!src.empty() && !hip_ok(hipMemcpy(*dst, src.data(), src.size() * sizeof(T), hipMemcpyHostToDevice)))
        return PCSR_E_HIP;
    return PCSR_OK;
}

// Lists the split panels (by position in the split tables) with more than
// pcsr::kLongPanelSlots items and puts the list in device memory: the second pass of the
// balanced write-back gives those panels a workgroup each.  split_slot: n_split + 1 entries
// in host memory.
static int upload_long_panels(pcsr_handle_s *h, const int32_t *split_slot)
{
    std::vector<int32_t> list;
    for (int64_t q = 0; q < h->n_split; ++q)
        if (split_slot[q + 1] - split_slot[q] > pcsr::kLongPanelSlots) list.push_back((int32_t)q);
    h->n_long = (int64_t)list.size();
    if (list.empty()) return PCSR_OK;
    return upload(list, &h->d_long);
}

// Launch shape for width K under the handle's kernel parameters ("0 = auto" resolved).
int resolve_launch(pcsr_handle_t h, int32_t K, pcsr::LaunchShape *ls)
{
    if (K <= 0) return PCSR_E_UNSUPPORTED;
    int vec = h->vec ? h->vec : (K % 4 == 0 ? 4 : (K % 2 == 0 ? 2 : 1));
    // as pcsr_select: K of 9..16 is served by 16 lanes of one dword unless rows are very short
    if (!h->vec && !h->lpr && K > 8 && K <= 16 && h->host.win_cols == 0 &&
        h->host.nnz_v >= 8 * std::max<int64_t>(h->host.P, 1))
        vec = 1;
    if (K % vec != 0) return PCSR_E_UNSUPPORTED;
    int lpr = h->lpr;
    if (!lpr) {
        int need = (K + vec - 1) / vec;
        if (h->host.win_cols > 0) {
            // column window: the staged slice (win_cols rows of lanes*vec columns) gets 128 KiB
            const int fit = (128 * 1024 / 4 / h->host.win_cols - 4) / vec;
            if (need > fit) need = fit;
        }
        // balanced (power-law) handles: four items per wavefront, as pcsr_select picks
        const int cap = h->host.S ? 16 : 64;
        lpr = 4;
        while (lpr < need && lpr < cap) lpr <<= 1;
    }
    int rep = h->rep;
    if (!rep) {
        int need = (K + lpr * vec - 1) / (lpr * vec);
        rep = 1;
        if (h->host.win_cols == 0 && !h->host.S)
            while (rep < need && rep < 4) rep <<= 1;
    }
    int waves = h->waves ? h->waves : 4;
    int ipg = h->ipg ? h->ipg : 1;
    if (ipg > 1) {
        // the batched walk accumulates each item sequentially and has no atomic write-back
        if (h->host.S || h->host.max_item_len > 1024) return PCSR_E_UNSUPPORTED;
    }
    const int64_t tile = (int64_t)lpr * vec * rep;
    ls->window = 0;
    ls->lds_bytes = 0;
    int64_t gx;
    if (h->host.win_cols > 0) {
        // column-window kernel: one workgroup per item block
        if (h->host.S || ipg > 1) return PCSR_E_UNSUPPORTED;
        if (!pcsr::window_kernel_exists(h->host.V, lpr, vec, rep)) return PCSR_E_UNSUPPORTED;
        // win_cols rows of B and one row of zeros, each padded by 4 floats
        const int64_t lds = ((int64_t)h->host.win_cols + 1) * (tile + 4) * 4;
        if (lds > 160 * 1024) return PCSR_E_UNSUPPORTED;
        if (!h->waves) waves = 16;
        ls->window = 1;
        ls->lds_bytes = (int32_t)lds;
        gx = h->n_win_blocks;
    } else {
        if (waves > 8) return PCSR_E_UNSUPPORTED;
        if (!pcsr::kernel_exists(h->host.V, h->host.S, lpr, vec, rep, ipg)) return PCSR_E_UNSUPPORTED;
        const int64_t items_per_wg = (int64_t)waves * (64 / lpr) * ipg;
        if (h->flags & PCSR_FLAG_NO_XCD_REMAP) {
            gx = (h->host.M + items_per_wg - 1) / items_per_wg;
        } else {
            // every XCD walks its own item range: 8 x the workgroups of the longest range
            int64_t longest = 0;
            for (int x = 0; x < 8; ++x)
                longest = std::max<int64_t>(longest, h->host.xcd_bounds[x + 1] - h->host.xcd_bounds[x]);
            gx = 8 * ((longest + items_per_wg - 1) / items_per_wg);
        }
    }
    const int64_t gy = (K + tile - 1) / tile;
    if (gx > 0x7fffffffLL || gy > 65535) return PCSR_E_TOO_LARGE;
    ls->lpr = lpr;
    ls->vec = vec;
    ls->rep = rep;
    ls->waves = waves;
    ls->ipg = ipg;
    ls->grid_x = (int32_t)gx;
    ls->grid_y = (int32_t)gy;
    return PCSR_OK;
}

} // namespace

extern "C" {

int pcsr_build(int64_t n_rows, int64_t n_cols, int64_t nnz, const int32_t *rowptr,
               const int32_t *colidx, const float *vals, const pcsr_params_t *p,
               pcsr_handle_t *out)
{
    if (!out || !rowptr || n_rows < 0 || n_cols < 0 || nnz < 0) return PCSR_E_INVALID_ARG;
    if (nnz > 0 && (!colidx || !vals)) return PCSR_E_INVALID_ARG;
    pcsr_params_t prm;
    std::memset(&prm, 0, sizeof(prm));
    if (p) prm = *p;
    if (prm.V == 0) prm.V = 1;
    if (prm.V != 1 && prm.V != 2) return PCSR_E_UNSUPPORTED;
    if (prm.S != 0 && prm.S != 1) return PCSR_E_UNSUPPORTED;
    if (prm.SG < 0 || prm.omega < 0) return PCSR_E_INVALID_ARG;
    if (prm.reserved[0]) return PCSR_E_INVALID_ARG;
    if (prm.col_window != 0 && prm.col_window != 256 && prm.col_window != 512 && prm.col_window != 1024 &&
        prm.col_window != 2048)
        return PCSR_E_UNSUPPORTED;
    if (prm.col_window && prm.S) return PCSR_E_UNSUPPORTED;
    if (nnz >= (int64_t(1) << 31) || n_rows >= (int64_t(1) << 31) - 1 || n_cols >= (int64_t(1) << 31))
        return PCSR_E_TOO_LARGE;
    int rc = check_kernel_params(prm.lanes_per_row, prm.vec, prm.rep, prm.waves_per_wg, prm.items_per_group);
    if (rc != PCSR_OK) return rc;
    const bool host_only = (prm.flags & PCSR_FLAG_HOST_ONLY) != 0;
    if (host_only && (prm.flags & PCSR_FLAG_DEVICE_CSR)) return PCSR_E_INVALID_ARG;

    const bool device_csr = (prm.flags & PCSR_FLAG_DEVICE_CSR) != 0;
    const bool column_order = (prm.flags & PCSR_FLAG_COLUMN_ORDER) != 0;
    if (column_order && (!prm.S || prm.col_window)) return PCSR_E_UNSUPPORTED;
    if ((device_csr || (prm.flags & PCSR_FLAG_GPU_BUILD)) && !prm.col_window) {
        if (host_only) return PCSR_E_INVALID_ARG;
        // ---- PCSR generation on the GPU
        int32_t *t_rowptr = nullptr, *t_colidx = nullptr;
        float *t_vals = nullptr;
        auto drop_tmp = [&] {
            if (t_rowptr) (void)hipFree(t_rowptr);
            if (t_colidx) (void)hipFree(t_colidx);
            if (t_vals) (void)hipFree(t_vals);
        };
        if (!device_csr) {
            bool ok = hip_ok(hipMalloc((void **)&t_rowptr, sizeof(int32_t) * (n_rows + 1))) &&
                      hip_ok(hipMalloc((void **)&t_colidx, sizeof(int32_t) * (nnz + 1))) &&
                      hip_ok(hipMalloc((void **)&t_vals, sizeof(float) * (nnz + 1))) &&
                      hip_ok(hipMemcpy(t_rowptr, rowptr, sizeof(int32_t) * (n_rows + 1), hipMemcpyHostToDevice)) &&
                      (nnz == 0 ||
                       (hip_ok(hipMemcpy(t_colidx, colidx, sizeof(int32_t) * nnz, hipMemcpyHostToDevice)) &&
                        hip_ok(hipMemcpy(t_vals, vals, sizeof(float) * nnz, hipMemcpyHostToDevice))));
            if (!ok) {
                drop_tmp();
                return PCSR_E_HIP;
            }
            rowptr = t_rowptr;
            colidx = t_colidx;
            vals = t_vals;
        }
        pcsr::DeviceBuild db;
        int herr = 0;
        rc = pcsr::build_device(n_rows, n_cols, nnz, rowptr, colidx, vals, prm.V, prm.S, prm.SG, prm.omega,
                                !(prm.flags & PCSR_FLAG_NO_VALIDATE), column_order, &db, &herr);
        drop_tmp();
        if (rc != PCSR_OK) {
            if (rc == PCSR_E_HIP) g_last_hip = herr;
            return rc;
        }
        pcsr_handle_s *h = new (std::nothrow) pcsr_handle_s();
        if (!h) {
            (void)hipFree(db.rowptr);
            (void)hipFree(db.colidx);
            (void)hipFree(db.val);
            if (db.trow) (void)hipFree(db.trow);
            if (db.split) (void)hipFree(db.split);
            if (db.item_slot) (void)hipFree(db.item_slot);
            if (db.sched) (void)hipFree(db.sched);
            if (db.split_slot) (void)hipFree(db.split_slot);
            return PCSR_E_OOM;
        }
        h->host.n_rows = n_rows;
        h->host.n_cols = n_cols;
        h->host.nnz = nnz;
        h->host.V = prm.V;
        h->host.S = prm.S;
        h->host.P = db.P;
        h->host.M = db.M;
        h->host.nnz_v = db.nnz_v;
        h->host.SG = db.SG;
        h->host.max_item_len = db.max_item_len;
        for (int x = 0; x < 9; ++x) h->host.xcd_bounds[x] = db.xcd_bounds[x];
        h->d_rowptr = db.rowptr;
        h->d_colidx = db.colidx;
        h->d_val = db.val;
        h->d_trow = db.trow;
        h->d_split = db.split;
        h->d_item_slot = db.item_slot;
        h->d_sched = db.sched;
        h->d_split_slot = db.split_slot;
        h->n_split = db.n_split;
        h->n_split_items = db.n_split_items;
        h->lpr = prm.lanes_per_row;
        h->vec = prm.vec;
        h->rep = prm.rep;
        h->waves = prm.waves_per_wg;
        h->ipg = prm.items_per_group;
        h->flags = prm.flags;
        if (!hip_ok(hipGetDevice(&h->device))) {
            release_device(h);
            delete h;
            return PCSR_E_HIP;
        }
        if (h->n_split > 0) {
            int rc2 = PCSR_E_OOM;
            try {
                std::vector<int32_t> slots((size_t)h->n_split + 1);
                rc2 = hip_ok(hipMemcpy(slots.data(), h->d_split_slot, slots.size() * sizeof(int32_t),
                                       hipMemcpyDeviceToHost))
                          ? upload_long_panels(h, slots.data())
                          : PCSR_E_HIP;
            } catch (const std::bad_alloc &) {
                rc2 = PCSR_E_OOM;
            }
            if (rc2 != PCSR_OK) {
                release_device(h);
                delete h;
                return rc2;
            }
        }
        *out = h;
        return PCSR_OK;
    }

    try {
        // The column-window build runs on the host: CSR arrays handed over in device memory
        // are copied there first (every other device-CSR build took the GPU branch above).
        std::vector<int32_t> s_rowptr, s_colidx;
        std::vector<float> s_vals;
        if (device_csr) {
            s_rowptr.resize(n_rows + 1);
            s_colidx.resize(nnz);
            s_vals.resize(nnz);
            if (!hip_ok(hipMemcpy(s_rowptr.data(), rowptr, sizeof(int32_t) * (n_rows + 1), hipMemcpyDeviceToHost)))
                return PCSR_E_HIP;
            if (nnz > 0 &&
                (!hip_ok(hipMemcpy(s_colidx.data(), colidx, sizeof(int32_t) * nnz, hipMemcpyDeviceToHost)) ||
                 !hip_ok(hipMemcpy(s_vals.data(), vals, sizeof(float) * nnz, hipMemcpyDeviceToHost))))
                return PCSR_E_HIP;
            rowptr = s_rowptr.data();
            colidx = s_colidx.data();
            vals = s_vals.data();
        }
        if (!(prm.flags & PCSR_FLAG_NO_VALIDATE)) {
            rc = pcsr::validate_csr(n_rows, n_cols, nnz, rowptr, colidx);
            if (rc != PCSR_OK) return rc;
        } else if (rowptr[0] != 0 || rowptr[n_rows] != nnz) {
            return PCSR_E_BAD_CSR;
        }

        pcsr_handle_s *h = new pcsr_handle_s();
        rc = pcsr::build_host(n_rows, n_cols, nnz, rowptr, colidx, vals, prm.V, prm.S, prm.SG,
                              prm.omega, &h->host);
        if (rc != PCSR_OK) {
            delete h;
            return rc;
        }
        if (column_order) {
            rc = pcsr::schedule_by_column(&h->host);
            if (rc != PCSR_OK) {
                delete h;
                return rc;
            }
        }
        if (prm.col_window) {
            rc = pcsr::choose_windows(&h->host, prm.col_window);
            if (rc != PCSR_OK) {
                delete h;
                return rc;
            }
        }
        h->n_win_blocks = (int64_t)h->host.win_start.size();
        h->host_only = host_only;
        h->lpr = prm.lanes_per_row;
        h->vec = prm.vec;
        h->rep = prm.rep;
        h->waves = prm.waves_per_wg;
        h->ipg = prm.items_per_group;
        h->flags = prm.flags;
        if (prm.col_window && (prm.flags & PCSR_FLAG_WINDOW_IF_USEFUL) &&
            (h->host.win_hit < 0.5 || h->host.M < 128 * h->n_win_blocks)) {
            // no structure for the window kernel to use: an ordinary handle
            h->host.win_cols = 0;
            h->host.win_hit = 0.0;
            h->n_win_blocks = 0;
            std::vector<int32_t>().swap(h->host.win_start);
            std::vector<int32_t>().swap(h->host.win_ptr);
            std::vector<int32_t>().swap(h->host.win_lo);
            std::vector<int32_t>().swap(h->host.win_hi);
            h->lpr = h->vec = h->rep = h->waves = h->ipg = 0;
        }
        h->n_split = (int64_t)h->host.split_panels.size();
        h->n_split_items = h->host.split_slot.empty() ? 0 : h->host.split_slot.back();
        if (!host_only) {
            if (!hip_ok(hipGetDevice(&h->device))) {
                delete h;
                return PCSR_E_HIP;
            }
            rc = upload(h->host.rowptr, &h->d_rowptr);
            if (rc == PCSR_OK) rc = upload(h->host.colidx, &h->d_colidx);
            if (rc == PCSR_OK) rc = upload(h->host.val, &h->d_val);
            if (rc == PCSR_OK && h->host.S) rc = upload(h->host.trow, &h->d_trow);
            if (rc == PCSR_OK && h->n_split) rc = upload(h->host.split_panels, &h->d_split);
            if (rc == PCSR_OK && h->host.S) rc = upload(h->host.item_slot, &h->d_item_slot);
            if (rc == PCSR_OK && !h->host.sched.empty()) rc = upload(h->host.sched, &h->d_sched);
            if (rc == PCSR_OK && h->n_split) rc = upload(h->host.split_slot, &h->d_split_slot);
            if (rc == PCSR_OK && h->n_split) rc = upload_long_panels(h, h->host.split_slot.data());
            if (rc == PCSR_OK && h->host.win_cols) rc = upload(h->host.win_start, &h->d_win);
            if (rc == PCSR_OK && h->host.win_cols) rc = upload(h->host.win_ptr, &h->d_win_ptr);
            if (rc == PCSR_OK && h->host.win_cols) rc = upload(h->host.win_lo, &h->d_win_lo);
            if (rc == PCSR_OK && h->host.win_cols) rc = upload(h->host.win_hi, &h->d_win_hi);
            if (rc != PCSR_OK) {
                release_device(h);
                delete h;
                return rc;
            }
            // the device copies are the product; drop the host staging arrays
            std::vector<int32_t>().swap(h->host.rowptr);
            std::vector<int32_t>().swap(h->host.colidx);
            std::vector<float>().swap(h->host.val);
            std::vector<int32_t>().swap(h->host.trow);
            std::vector<int32_t>().swap(h->host.split_panels);
            std::vector<int32_t>().swap(h->host.item_slot);
            std::vector<int32_t>().swap(h->host.sched);
            std::vector<int32_t>().swap(h->host.split_slot);
            std::vector<int32_t>().swap(h->host.win_start);
            std::vector<int32_t>().swap(h->host.win_ptr);
            std::vector<int32_t>().swap(h->host.win_lo);
            std::vector<int32_t>().swap(h->host.win_hi);
        }
        *out = h;
        return PCSR_OK;
    } catch (const std::bad_alloc &) {
        return PCSR_E_OOM;
    }
}

// Bytes of workspace one SpMM of width K needs: V*K floats per item of a split panel
// (deterministic balanced write-back only).
static int64_t workspace_need(pcsr_handle_t h, int32_t K)
{
    if (!h->host.S || (h->flags & PCSR_FLAG_ATOMIC_SPLIT)) return 0;
    return h->n_split_items * (int64_t)h->host.V * (int64_t)K * (int64_t)sizeof(float);
}

// Checks shared by the SpMM entry points; resolves the launch shape.
static int spmm_check(pcsr_handle_t h, const float *B, float *C, int32_t K, pcsr::LaunchShape *ls)
{
    if (!valid(h)) return PCSR_E_INVALID_ARG;
    if (h->host_only) return PCSR_E_UNSUPPORTED;
    if (K <= 0) return PCSR_E_UNSUPPORTED;
    if (!C && h->host.n_rows > 0) return PCSR_E_INVALID_ARG;
    if (!B && h->host.n_cols > 0 && h->host.nnz_v > 0) return PCSR_E_INVALID_ARG;
    int rc = resolve_launch(h, K, ls);
    if (rc != PCSR_OK) return rc;
    const uintptr_t align = 4u * (unsigned)ls->vec;
    if ((reinterpret_cast<uintptr_t>(B) % align) || (reinterpret_cast<uintptr_t>(C) % align))
        return PCSR_E_INVALID_ARG;
    if (h->host.n_rows == 0) return PCSR_OK;
    // B and C may not overlap: the kernel reads B while other workgroups write C
    const uintptr_t b0 = reinterpret_cast<uintptr_t>(B), c0 = reinterpret_cast<uintptr_t>(C);
    const uintptr_t b1 = b0 + (uintptr_t)h->host.n_cols * (uintptr_t)K * 4u;
    const uintptr_t c1 = c0 + (uintptr_t)h->host.n_rows * (uintptr_t)K * 4u;
    if (b0 < c1 && c0 < b1 && h->host.n_cols > 0) return PCSR_E_INVALID_ARG;
    // the handle's arrays live on the device that was current at pcsr_build
    int dev = -1;
    if (!hip_ok(hipGetDevice(&dev))) return PCSR_E_HIP;
    if (dev != h->device) return PCSR_E_INVALID_ARG;
    return PCSR_OK;
}

// Enqueues the kernels of one SpMM.  ws: workspace of at least workspace_need(h, K) bytes
// (ignored when that is 0).
static int spmm_enqueue(pcsr_handle_t h, const float *B, float *C, int32_t K, const pcsr::LaunchShape &ls,
                        float *ws, hipStream_t s)
{
    const bool two_pass = workspace_need(h, K) > 0;
    if (h->host.S && h->n_split > 0 && !two_pass) {
        if (!hip_ok(pcsr::launch_zero_panels(h->d_split, h->n_split, h->host.V, C,
                                             (int32_t)h->host.n_rows, K, s)))
            return PCSR_E_HIP;
    }
    pcsr::SpmmArgs a;
    a.rowptr = h->d_rowptr;
    a.colidx = h->d_colidx;
    a.val = h->d_val;
    a.trow = h->d_trow;
    a.B = B;
    a.C = C;
    a.M = (int32_t)h->host.M;
    a.n_rows = (int32_t)h->host.n_rows;
    a.K = K;
    a.nblk = ls.grid_x;
    a.xcd_remap = (h->flags & PCSR_FLAG_NO_XCD_REMAP) ? 0 : 1;
    for (int x = 0; x < 9; ++x) a.xb[x] = h->host.xcd_bounds[x];
    a.ws = two_pass ? ws : nullptr;
    a.item_slot = h->d_item_slot;
    a.sched = reinterpret_cast<const int4 *>(h->d_sched);
    a.win_start = h->d_win;
    a.win_cols = h->host.win_cols;
    a.win_ptr = h->d_win_ptr;
    a.win_lo = h->d_win_lo;
    a.win_hi = h->d_win_hi;
    a.n_cols = (int32_t)h->host.n_cols;
    if (!hip_ok(pcsr::launch_spmm(h->host.V, h->host.S, ls, a, s))) return PCSR_E_HIP;
    if (two_pass) {
        if (!hip_ok(pcsr::launch_reduce_split(h->d_split, h->d_split_slot, h->n_split, h->d_long, h->n_long, h->host.V, ws, C,
                                              (int32_t)h->host.n_rows, K, s)))
            return PCSR_E_HIP;
    }
    return PCSR_OK;
}

// Makes the handle's own workspace at least `need` bytes.  Allocates, so not for use
// under stream capture.
static int grow_workspace(pcsr_handle_t h, int64_t need)
{
    if (need <= (int64_t)h->ws_bytes) return PCSR_OK;
    if (h->d_ws) {
        // hipFree waits for the device, so no earlier SpMM still uses the old block
        if (!hip_ok(hipFree(h->d_ws))) return PCSR_E_HIP;
        h->d_ws = nullptr;
        h->ws_bytes = 0;
    }
    hipError_t e = hipMalloc((void **)&h->d_ws, (size_t)need);
    if (e == hipErrorOutOfMemory) {
        (void)hipGetLastError();
        h->d_ws = nullptr;
        return PCSR_E_OOM;
    }
    if (!hip_ok(e)) {
        h->d_ws = nullptr;
        return PCSR_E_HIP;
    }
    h->ws_bytes = (size_t)need;
    return PCSR_OK;
}

int pcsr_spmm(pcsr_handle_t h, const float *B, float *C, int32_t K, void *stream)
{
    pcsr::LaunchShape ls;
    int rc = spmm_check(h, B, C, K, &ls);
    if (rc != PCSR_OK) return rc;
    if (h->host.n_rows == 0) return PCSR_OK;
    rc = grow_workspace(h, workspace_need(h, K));
    if (rc != PCSR_OK) return rc;
    return spmm_enqueue(h, B, C, K, ls, h->d_ws, static_cast<hipStream_t>(stream));
}

int pcsr_spmm_static(pcsr_handle_t h, const float *B, float *C, int32_t K, void *stream)
{
    pcsr::LaunchShape ls;
    int rc = spmm_check(h, B, C, K, &ls);
    if (rc != PCSR_OK) return rc;
    if (h->host.n_rows == 0) return PCSR_OK;
    if (workspace_need(h, K) > (int64_t)pcsr::kStaticScratchBytes) return PCSR_E_TOO_LARGE;
    void *ws = nullptr;
    if (!hip_ok(pcsr::static_scratch(&ws))) return PCSR_E_HIP;
    return spmm_enqueue(h, B, C, K, ls, static_cast<float *>(ws), static_cast<hipStream_t>(stream));
}

int64_t pcsr_static_scratch_bytes(void) { return (int64_t)pcsr::kStaticScratchBytes; }

int pcsr_workspace_bytes(pcsr_handle_t h, int32_t K, int64_t *bytes)
{
    if (!valid(h) || !bytes) return PCSR_E_INVALID_ARG;
    if (K <= 0) return PCSR_E_UNSUPPORTED;
    *bytes = workspace_need(h, K);
    return PCSR_OK;
}

int pcsr_reserve_workspace(pcsr_handle_t h, int32_t K)
{
    if (!valid(h)) return PCSR_E_INVALID_ARG;
    if (h->host_only || K <= 0) return PCSR_E_UNSUPPORTED;
    int dev = -1;
    if (!hip_ok(hipGetDevice(&dev))) return PCSR_E_HIP;
    if (dev != h->device) return PCSR_E_INVALID_ARG;
    return grow_workspace(h, workspace_need(h, K));
}

int pcsr_free(pcsr_handle_t h)
{
    if (!h) return PCSR_OK;
    if (!valid(h)) return PCSR_E_INVALID_ARG;
    release_device(h);
    h->magic = 0;
    delete h;
    return PCSR_OK;
}

int pcsr_set_kernel_params(pcsr_handle_t h, int32_t lanes_per_row, int32_t vec, int32_t rep,
                           int32_t waves_per_wg, int32_t items_per_group, int32_t flags)
{
    if (!valid(h)) return PCSR_E_INVALID_ARG;
    int rc = check_kernel_params(lanes_per_row, vec, rep, waves_per_wg, items_per_group);
    if (rc != PCSR_OK) return rc;
    h->lpr = lanes_per_row;
    h->vec = vec;
    h->rep = rep;
    h->waves = waves_per_wg;
    h->ipg = items_per_group;
    constexpr int32_t kLaunchFlags = PCSR_FLAG_NO_XCD_REMAP | PCSR_FLAG_ATOMIC_SPLIT;
    h->flags = (h->flags & ~kLaunchFlags) | (flags & kLaunchFlags);
    return PCSR_OK;
}

int pcsr_query_launch(pcsr_handle_t h, int32_t K, int32_t out[8])
{
    if (!valid(h) || !out) return PCSR_E_INVALID_ARG;
    pcsr::LaunchShape ls;
    int rc = resolve_launch(h, K, &ls);
    if (rc != PCSR_OK) return rc;
    out[0] = ls.lpr;
    out[1] = ls.vec;
    out[2] = ls.rep;
    out[3] = ls.waves;
    out[4] = ls.grid_x;
    out[5] = ls.grid_y;
    out[6] = ls.ipg;
    out[7] = ls.lds_bytes;
    return PCSR_OK;
}

int pcsr_window_stats(pcsr_handle_t h, double out[3])
{
    if (!valid(h) || !out) return PCSR_E_INVALID_ARG;
    out[0] = (double)h->host.win_cols;
    out[1] = h->n_win_blocks ? (double)h->host.M / (double)h->n_win_blocks : 0.0;
    out[2] = h->host.win_hit;
    return PCSR_OK;
}

int pcsr_export(pcsr_handle_t h, int64_t sizes[6], int32_t *rowptr, int32_t *colidx, float *val,
                int32_t *trow)
{
    if (!valid(h)) return PCSR_E_INVALID_ARG;
    const pcsr::HostPcsr &m = h->host;
    if (sizes) {
        sizes[0] = m.P;
        sizes[1] = m.M;
        sizes[2] = m.nnz_v;
        sizes[3] = m.V;
        sizes[4] = m.SG;
        sizes[5] = m.S ? 1 : 0;
    }
    auto fetch = [&](void *dst, const void *host_src, const void *dev_src, size_t bytes) -> int {
        if (!dst || bytes == 0) return PCSR_OK;
        if (h->host_only) {
            std::memcpy(dst, host_src, bytes);
            return PCSR_OK;
        }
        return hip_ok(hipMemcpy(dst, dev_src, bytes, hipMemcpyDeviceToHost)) ? PCSR_OK : PCSR_E_HIP;
    };
    int rc = fetch(rowptr, m.rowptr.data(), h->d_rowptr, sizeof(int32_t) * (m.M + 1));
    if (rc == PCSR_OK) rc = fetch(colidx, m.colidx.data(), h->d_colidx, sizeof(int32_t) * m.nnz_v);
    if (rc == PCSR_OK) rc = fetch(val, m.val.data(), h->d_val, sizeof(float) * m.nnz_v * m.V);
    if (rc == PCSR_OK && m.S) rc = fetch(trow, m.trow.data(), h->d_trow, sizeof(int32_t) * m.M);
    return rc;
}

int pcsr_export_schedule(pcsr_handle_t h, int64_t *n_positions, int32_t *sched, int32_t xcd_bounds[9])
{
    if (!valid(h)) return PCSR_E_INVALID_ARG;
    const bool has = h->host_only ? !h->host.sched.empty() : h->d_sched != nullptr;
    if (n_positions) *n_positions = has ? h->host.M : 0;
    if (xcd_bounds)
        for (int x = 0; x < 9; ++x) xcd_bounds[x] = h->host.xcd_bounds[x];
    if (!sched || !has || h->host.M == 0) return PCSR_OK;
    const size_t bytes = sizeof(int32_t) * 4 * (size_t)h->host.M;
    if (h->host_only) {
        std::memcpy(sched, h->host.sched.data(), bytes);
        return PCSR_OK;
    }
    return hip_ok(hipMemcpy(sched, h->d_sched, bytes, hipMemcpyDeviceToHost)) ? PCSR_OK : PCSR_E_HIP;
}

int pcsr_features(int64_t n_rows, int64_t n_cols, int64_t nnz, const int32_t *rowptr,
                  const int32_t *colidx, int32_t omega, double *out, int32_t n_out)
{
    if (!out || n_out < PCSR_N_FEATURES || !rowptr || omega < 0) return PCSR_E_INVALID_ARG;
    int rc = pcsr::validate_csr(n_rows, n_cols, nnz, rowptr, colidx);
    if (rc != PCSR_OK) return rc;
    try {
        return pcsr::features_host(n_rows, n_cols, nnz, rowptr, colidx, omega, out);
    } catch (const std::bad_alloc &) {
        return PCSR_E_OOM;
    }
}

int pcsr_features_device(int64_t n_rows, int64_t n_cols, int64_t nnz, const int32_t *rowptr,
                         const int32_t *colidx, int32_t omega, double *out, int32_t n_out)
{
    if (!out || n_out < PCSR_N_FEATURES || !rowptr || omega < 0 || n_rows < 0 || n_cols < 0 || nnz < 0)
        return PCSR_E_INVALID_ARG;
    if (nnz > 0 && !colidx) return PCSR_E_INVALID_ARG;
    if (nnz >= (int64_t(1) << 31) || n_rows >= (int64_t(1) << 31) - 1) return PCSR_E_TOO_LARGE;
    int herr = 0;
    int rc = pcsr::features_device(n_rows, n_cols, nnz, rowptr, colidx, omega, out, &herr);
    if (rc == PCSR_E_HIP) g_last_hip = herr;
    return rc;
}

int pcsr_select(const double *f, int32_t K, pcsr_params_t *out)
{
    if (!f || !out) return PCSR_E_INVALID_ARG;
    if (K <= 0) return PCSR_E_UNSUPPORTED;
    pcsr_params_t p;
    std::memset(&p, 0, sizeof(p));
    const double d_hat = f[5], d_max = f[6], cv = f[7], pr2 = f[15];

    // Balancing (Section 3.2) pays when a few rows dwarf the average one.  On MI355X the
    // recorded sweeps then prefer short items (32 vectors with slices of up to 64 columns, 64
    // vectors with 128-column slices) run in column order: the items of
    // the long rows, sorted by first column, make the wavefronts of an XCD gather the same B
    // rows at about the same time (R-MAT scale 22: 1.6-2x over the best index-order tuple at
    // every width from 16 to 512; neutral on small or uniform inputs).
    const bool skewed = cv > 1.5 && d_max > 256.0;
    // Loads per lane: the widest vector that divides K, except where fewer rows per
    // wavefront pay more than wide loads.  A wavefront runs until the longest of its work
    // items ends, so with rows of varying length every further item per wavefront costs
    // lane time.  K of 9..16: one dword per lane, 16 lanes per row (4 items per wavefront
    // instead of 16: 11-18 % faster on every input but road-like ones, whose rows of 3 want
    // many rows per wavefront).
    int vec = K % 4 == 0 ? 4 : (K % 2 == 0 ? 2 : 1);
    if (K > 8 && K <= 16 && d_hat >= 8.0) vec = 1;
    // Rows that gather from a neighbourhood of their own index are served from LDS instead
    // (see the column window below), from K = 64 (at 32 it ties with the plain kernel) and if
    // the product is large enough to give every compute unit a few window blocks: a block
    // occupies a whole compute unit, and with too few rounds of blocks the last one leaves
    // most of the chip idle (90,000 rows in communities of 300: 0.55x of the plain kernel
    // at K = 32, 0.81x at K = 128; 200,000 rows at K = 64: 1.1x).
    const double n = f[0];
    // Rows that share most columns with their neighbour (padding below 30 %) do better
    // paired, V = 2, than from LDS (cliques of 48, K = 128: 0.98 against 0.82 of the best).
    const bool windowed = !skewed && f[16] >= 0.6 && d_hat >= 40.0 && vec == 4 && pr2 >= 0.3 && K >= 64 &&
                          n * (double)((K + 63) / 64) >= 200000.0;
    // Uniformly long rows with scattered columns (mean length 40 or more, no more nonzeros
    // near the diagonal than four times what uniform columns would put there).  From
    // K = 64 the same column-ordered schedule, with items of 32, turns the split into a
    // column partition of A, each XCD gathering from its own range of B rows (uniform
    // random columns, 96 per row, K = 128: 1.5x; 48 per row, K = 256: 1.13x; at 32 per
    // row the second items are too short and it loses 15 %).  Narrower B rows are cached
    // well enough as they are; there pairing rows (V = 2) wins, by doubling the gathers a
    // lane group has in flight.  Rows with local columns lose up to half their speed under
    // the column order (it gives up the reuse between neighbouring rows).
    const bool scattered = f[16] < 4.0 * 1025.0 / (n > 1.0 ? n : 1.0);
    // K of 17..32 with scattered columns and a B beyond 16 MB (rows gathered from the
    // memory side, not from L2): one dword per lane again, a row per half wavefront
    // (uniform random columns, 16 to 64 per row, 150,000 rows or more: 7-24 % faster than
    // the best 16-byte shape; slower when B is small or the columns are local).
    const bool wide_scatter = !skewed && scattered && d_hat >= 12.0 && K > 16 && K <= 32 &&
                              n * (double)K * 4.0 > 16.0 * 1048576.0;
    if (wide_scatter) vec = 1;
    const bool long_uniform = !skewed && !windowed && !wide_scatter && d_hat >= 40.0 && scattered;
    const bool long_uniform_wide = long_uniform && K >= 64;
    p.S = (skewed || long_uniform_wide) ? 1 : 0;
    p.SG = p.S ? 32 : 0; // power-law inputs: raised to 64 below for 128-column slices
    p.omega = 64;
    if (p.S) p.flags |= PCSR_FLAG_COLUMN_ORDER;
    // Vector size 2 (Section 3.1) when adjacent rows share columns, and for short rows, where
    // pairing rows doubles the gathers a lane group keeps in flight.  The paper's A6000 data
    // puts the break-even near 30 % padding; on MI355X clique-like inputs win at 11 %
    // padding (1.23x at K=128) and lose at 27 %, because adjacent rows of one wavefront
    // already share their B lines in L1.  Power-law inputs: V = 2 ties or loses in the sweeps.
    // Long scattered rows at K below 64 (above): paired as well, unless the matrix is so small
    // that halving the number of work items leaves wavefront slots empty (30,000 rows of
    // 160, K = 32: V = 2 runs at 0.55 of V = 1).
    const bool pair_long = long_uniform && n * (double)(K < 32 ? 4 : 8) / 128.0 >= 3500.0;
    p.V = (!p.S && (d_hat < 6.0 || (d_hat < 12.0 && pr2 < 0.45) || pr2 < 0.20 || pair_long)) ? 2 : 1;

    // Launch shape: the widest vector load that divides K, one lane group spanning the
    // whole row of C when it fits a wavefront, repeats beyond that.
    // Balanced power-law inputs do best without repeats and, once B outgrows the 256 MB
    // memory-side cache, with 64-column slices (four items per wavefront; grid.y covers
    // wider rows), which shrinks the bytes a cached B row occupies; a smaller B is gathered
    // in 128-column slices.
    const double b_bytes = f[0] * (double)K * 4.0;
    const int lpr_cap = p.S ? ((long_uniform_wide || b_bytes > 192.0 * 1048576.0) ? 16 : 32) : 64;
    int lpr = 4;
    while (lpr * vec < K && lpr < lpr_cap) lpr <<= 1;
    int rep = 1;
    while (!p.S && lpr * vec * rep < K && rep < 4) rep <<= 1;
    if (!p.S && p.V == 1 && d_hat < 8.0 && lpr >= 32 && rep == 1) {
        lpr >>= 1; // short rows: more rows per wavefront, two loads per lane
        rep = 2;
    }
    // Scattered columns, rows of 8 to 40, K from 64: a 64-column slice per half wavefront
    // with dwordx2 loads (uniform random columns, 8 to 32 per row, K = 64 and 128: 3-7 %
    // over the best 16-byte shape; local columns keep the 16-byte shapes).
    if (!skewed && !windowed && !long_uniform && scattered && d_hat >= 8.0 && K >= 64 && K % 2 == 0) {
        lpr = 32;
        vec = 2;
        rep = 1;
    }
    // K of 17..32, rows of 32 and more that are neither split nor paired: 16 lanes of one
    // dword, two loads per lane (4 items per wavefront instead of 8): 9-19 % faster than
    // 8 lanes x dwordx4 on the community and clique inputs of the validation sets; rows
    // of 20-27 and road-like inputs keep the 16-byte shape.
    if (!p.S && !wide_scatter && !pair_long && d_hat >= 32.0 && K > 16 && K <= 32) {
        lpr = 16;
        vec = 1;
        rep = 2;
    }
    p.lanes_per_row = lpr;
    p.vec = vec;
    p.rep = rep;
    if (skewed && lpr * vec > 64) p.SG = 64;
    // Workgroup size: four wavefronts, two for short rows and for paired long rows (eight
    // were 4-7 % slower than four on every unsplit input of the later validation sets).
    p.waves_per_wg = p.S ? 4 : (d_hat >= 16.0 && !pair_long ? 4 : 2);
    p.items_per_group = 1;
    p.col_window = 0;
    // Column-window blocking: rows that gather from a neighbourhood of their own index (most
    // nonzeros within 512 columns of the diagonal) and are long enough that every staged row
    // of B is used dozens of times.  A 500-node community graph of degree 48 runs 1.1x
    // (K = 64) to 1.4x (K = 512) faster from LDS than from L2; cliques of 25 or blocks of 50
    // nodes do not repay the staging.  The build drops the window again if the blocks it
    // finds are poor.
    if (windowed) {
        p.V = 1;
        p.col_window = 512;
        p.flags |= PCSR_FLAG_WINDOW_IF_USEFUL;
        p.lanes_per_row = 16; // 64-column slices of the window (136 KiB of LDS)
        p.rep = 1;
        p.waves_per_wg = 16;
    }
    *out = p;
    return PCSR_OK;
}

int32_t pcsr_mac_job_gap(int32_t dim, int32_t F, int32_t omega)
{
    if (dim <= 0 || F <= 0 || omega <= 0) return -1;
    const int64_t span = (int64_t)F * omega;
    const int64_t tn = dim < span ? dim : span;
    const int64_t tr = dim % span;
    return tr == 0 ? 0 : (int32_t)(tn - tr);
}

const char *pcsr_strerror(int code)
{
    switch (code) {
    case PCSR_OK: return "ok";
    case PCSR_E_INVALID_ARG: return "invalid argument";
    case PCSR_E_BAD_CSR: return "malformed CSR (rowptr not monotone, column out of range, unsorted or duplicate columns)";
    case PCSR_E_UNSUPPORTED: return "unsupported parameter value";
    case PCSR_E_TOO_LARGE: return "size does not fit 32-bit indexing, or the fixed workspace";
    case PCSR_E_OOM: return "out of memory";
    case PCSR_E_HIP: return "HIP runtime error";
    }
    return "unknown error";
}

int pcsr_last_hip_error(void) { return g_last_hip; }

} // extern "C"
