// Host-side PCSR construction and matrix features (internal to the library).
#pragma once
#include <cstdint>
#include <vector>

namespace pcsr {

// The four PCSR arrays of Section 4.2 plus the bookkeeping the launcher needs.
struct HostPcsr {
    int64_t n_rows = 0, n_cols = 0, nnz = 0;
    int64_t P = 0;     // row panels = ceil(n_rows / V)
    int64_t M = 0;     // work items (== P when S is off)
    int64_t nnz_v = 0; // nonzero vectors
    int32_t V = 1, S = 0, SG = 0;
    std::vector<int32_t> rowptr; // M+1
    std::vector<int32_t> colidx; // nnz_v
    std::vector<float> val;      // nnz_v * V, padding slots +0.0f
    std::vector<int32_t> trow;   // M when S, else empty
    // Not part of the format: panels that own more than one work item.  Their C rows
    // are cleared before the kernel accumulates into them.
    std::vector<int32_t> split_panels;
    // For the q-th such panel: the first of the consecutive workspace slots its items
    // write their partial rows to (one more entry at the end: the total number of items
    // that belong to split panels); and per work item its slot, -1 for an item that is
    // the only one of its panel.
    std::vector<int32_t> split_slot, item_slot;
    // Column-ordered schedule (empty = items run in index order): four entries per launch
    // position - first vector, vector count, panel, workspace slot or -1 - of the item
    // that runs there.  With it, xcd_bounds are positions.
    std::vector<int32_t> sched;
    int64_t max_item_len = 0;
    // Not part of the format: item boundaries that cut the item sequence into 8 contiguous
    // ranges of equal work (vectors plus a per-item overhead), one per XCD.
    int32_t xcd_bounds[9] = {0, 0, 0, 0, 0, 0, 0, 0, 0};
    // Column-window blocking (not part of the format): consecutive items are grouped into
    // blocks [win_ptr[b], win_ptr[b+1]) of at most win_cols items that gather from the same
    // stretch of columns; win_start[b] is the first column of block b's LDS-resident
    // window, or -1 when no window is worth staging for that block.
    int32_t win_cols = 0;
    std::vector<int32_t> win_ptr, win_start;
    // per item: its vectors [win_lo, win_hi) have their column inside the block's window
    // (the columns of an item ascend, so they form one run)
    std::vector<int32_t> win_lo, win_hi;
    double win_hit = 0.0; // fraction of nonzero vectors that fall inside their window
};

// Returns PCSR_OK or PCSR_E_BAD_CSR / PCSR_E_TOO_LARGE / PCSR_E_INVALID_ARG.
int validate_csr(int64_t n_rows, int64_t n_cols, int64_t nnz, const int32_t *rowptr,
                 const int32_t *colidx);

// Vectorised blocking followed by the optional workload split.
int build_host(int64_t n_rows, int64_t n_cols, int64_t nnz, const int32_t *rowptr,
               const int32_t *colidx, const float *vals, int32_t V, int32_t S, int32_t SG,
               int32_t omega, HostPcsr *out);

// Column-ordered schedule for a balanced handle (needs rowptr / colidx / item_slot on the
// host): the items of split panels in ascending order of their first column, the other
// items in index order, both dealt to the 8 XCDs in contiguous equal-work slices.
int schedule_by_column(HostPcsr *h);

// Cuts the items into blocks that share a window of win_cols consecutive columns and picks
// each block's window (needs h->rowptr / h->colidx on the host).
int choose_windows(HostPcsr *h, int32_t win_cols);

// Table 3 features in the order documented in pcsr.h.
int features_host(int64_t n_rows, int64_t n_cols, int64_t nnz, const int32_t *rowptr,
                  const int32_t *colidx, int32_t omega, double *out);

} // namespace pcsr
