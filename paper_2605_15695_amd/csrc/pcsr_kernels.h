// Launchers of the HIP SpMM kernel family (internal to the library).
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace pcsr {

struct SpmmArgs {
    const int32_t *rowptr; // M+1, device
    const int32_t *colidx; // nnz_v, device
    const float *val;      // nnz_v * V, device
    const int32_t *trow;   // M (S only), device
    const float *B;
    float *C;
    int32_t M;      // work items
    int32_t n_rows; // rows of C
    int32_t K;
    int32_t nblk;      // grid.x
    int32_t xcd_remap; // 1: one contiguous, work-balanced item range per XCD
    int32_t xb[9];     // item range [xb[x], xb[x+1]) of XCD x (xcd_remap only)
    // Balanced handles, deterministic write-back: an item of a panel that was split over
    // several items stores its partial rows in `ws` (slot-major: (slot*V + v)*K + k) and
    // reduce_split adds them in item order.  ws == nullptr selects the atomic write-back.
    float *ws;
    const int32_t *item_slot; // M (S only): workspace slot of an item of a split panel, -1 for
                              // an item that is the only one of its panel
    // Column-ordered schedule (S only, may be null): for launch position i the record
    // {first vector, vector count, panel (TRow), workspace slot or -1} of the work item
    // that runs there.  xb then bounds positions, not items.
    const int4 *sched;
    // column-window blocking (window kernel only)
    const int32_t *win_ptr;   // item range [win_ptr[b], win_ptr[b+1]) of block b (= workgroup b)
    const int32_t *win_start; // per item block: first column of the staged window or -1
    const int32_t *win_lo;    // per item: its vectors [win_lo, win_hi) lie inside the block's
    const int32_t *win_hi;    // window (an empty range when the block has none)
    int32_t win_cols;         // rows of B staged in LDS
    int32_t n_cols;
};

// Resolved launch shape.
struct LaunchShape {
    int32_t lpr, vec, rep, waves;
    int32_t ipg; // work items per lane group (1 = one item per group)
    int32_t window; // 1: column-window kernel (one workgroup per item block, B window in LDS)
    int32_t lds_bytes;
    int32_t grid_x, grid_y;
};

bool kernel_exists(int V, int S, int lpr, int vec, int rep, int ipg);
bool window_kernel_exists(int V, int lpr, int vec, int rep);

// Enqueues the SpMM kernel <V,S,lpr,vec,rep> with `waves` wavefronts per workgroup.
hipError_t launch_spmm(int V, int S, const LaunchShape &ls, const SpmmArgs &args,
                       hipStream_t stream);

// Clears the C rows of the listed panels (rows panel*V .. panel*V+V-1, K floats each).
hipError_t launch_zero_panels(const int32_t *panels, int64_t n_panels, int V, float *C,
                              int32_t n_rows, int32_t K, hipStream_t stream);

// Second pass of the deterministic balanced write-back: for every split panel q and
// v < V, C[panel*V + v][:] = sum over its items of the partial rows the SpMM kernel left
// in ws.  Panels with at most kLongPanelSlots items are added in item order by one thread
// per vector of C; the others (indices into the split tables listed in long_panels,
// n_long of them) by kLongReduceLanes threads per vector, thread j taking items j,
// j + kLongReduceLanes, ... in order, the partial sums then added in ascending j.
constexpr int kLongPanelSlots = 64;
constexpr int kLongReduceLanes = 16;
hipError_t launch_reduce_split(const int32_t *split_panels, const int32_t *split_slot, int64_t n_split,
                               const int32_t *long_panels, int64_t n_long, int V, const float *ws, float *C,
                               int32_t n_rows, int32_t K, hipStream_t stream);

// Fixed workspace for callers that cannot allocate: one block of kStaticScratchBytes
// bytes per GPU, part of the library's device image and held until the process ends.
// static_scratch returns its address on the current device (looked up once per device).
constexpr size_t kStaticScratchBytes = size_t(64) << 20;
hipError_t static_scratch(void **ptr);

} // namespace pcsr
