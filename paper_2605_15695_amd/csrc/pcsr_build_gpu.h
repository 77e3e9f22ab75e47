// PCSR generation on the GPU (internal to the library).
#pragma once
#include <cstdint>

namespace pcsr {

// Device arrays produced by build_device; ownership passes to the caller (hipFree).
struct DeviceBuild {
    int32_t *rowptr = nullptr; // M+1
    int32_t *colidx = nullptr; // nnz_v
    float *val = nullptr;      // nnz_v * V
    int32_t *trow = nullptr;   // M (S only)
    int32_t *split = nullptr;  // panels with more than one item (S only), ascending, n_split entries
    int32_t *item_slot = nullptr;   // per item (S only): workspace slot, -1 for a sole item
    int32_t *split_slot = nullptr;  // first workspace slot of each of them, n_split + 1 entries
    int32_t *sched = nullptr;       // column-ordered schedule, 4 int32 per launch position (or null)
    int64_t P = 0, M = 0, nnz_v = 0, n_split = 0, n_split_items = 0, max_item_len = 0;
    int32_t SG = 0;
    int32_t xcd_bounds[9] = {0, 0, 0, 0, 0, 0, 0, 0, 0};
};

// d_rowptr / d_colidx / d_vals are device pointers.  Returns PCSR_OK or a PCSR_E_* code;
// on PCSR_E_HIP *hip_err holds the hipError_t.  Synchronous.
int build_device(int64_t n_rows, int64_t n_cols, int64_t nnz, const int32_t *d_rowptr,
                 const int32_t *d_colidx, const float *d_vals, int32_t V, int32_t S, int32_t SG,
                 int32_t omega, bool validate, bool column_order, DeviceBuild *out, int *hip_err);

// Table 3 features (order as in pcsr.h) from CSR arrays in device memory.  The CSR is
// assumed valid (pcsr_build validates).  Synchronous.
int features_device(int64_t n_rows, int64_t n_cols, int64_t nnz, const int32_t *d_rowptr,
                    const int32_t *d_colidx, int32_t omega, double *out, int *hip_err);

} // namespace pcsr
