/*
 * pcsr.h - C ABI of the PCSR SpMM library for AMD MI355X (gfx950).
 *
 * Computes C = A * B where A (n_rows x n_cols, sparse) is held in the paper's
 * Parameterized CSR form and B (n_cols x K) and C (n_rows x K) are dense, row-major,
 * fp32 (problem statement: Section 2, "Background"; format: Section 4.2; kernel:
 * Algorithm 2 in Section 4.3).
 *
 * Conventions for every entry point
 *   - return value: PCSR_OK (0) or a negative PCSR_E_* code; nothing is thrown across
 *     the ABI; output arguments are left untouched on failure.
 *   - "host" / "device" in an argument's description says where the memory must live.
 *   - the library never synchronises the caller's stream unless stated.
 */
#ifndef PCSR_H
#define PCSR_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    PCSR_OK = 0,
    PCSR_E_INVALID_ARG = -1, /* null pointer, negative size, misaligned B/C, bad handle      */
    PCSR_E_BAD_CSR = -2,     /* rowptr not monotone / not starting at 0 / not ending at nnz,
                                column out of range, columns of a row not strictly ascending  */
    PCSR_E_UNSUPPORTED = -3, /* V not in {1,2}, K <= 0, vec does not divide K, bad kernel
                                parameter, SpMM on a host-only handle                        */
    PCSR_E_TOO_LARGE = -4,   /* nnz, n_rows or the item count does not fit int32; workspace
                                need beyond the fixed block of pcsr_spmm_static             */
    PCSR_E_OOM = -5,         /* host or device allocation failed                             */
    PCSR_E_HIP = -6          /* a HIP runtime call failed (see pcsr_last_hip_error)          */
};

enum {
    PCSR_FLAG_DEVICE_CSR = 1,  /* rowptr/colidx/vals passed to pcsr_build are device pointers */
    PCSR_FLAG_NO_VALIDATE = 2, /* trust the CSR (skips the O(nnz) check)                      */
    PCSR_FLAG_NO_XCD_REMAP = 4,/* keep the hardware's round-robin workgroup -> XCD order      */
    PCSR_FLAG_HOST_ONLY = 8,   /* build the arrays on the host only (no GPU needed); the
                                  handle serves pcsr_export but not pcsr_spmm                 */
    PCSR_FLAG_GPU_BUILD = 16,  /* generate the PCSR arrays with GPU kernels (host CSR arrays
                                  are uploaded first).  CSR arrays given in device memory are
                                  always built this way.  With col_window the flag is ignored:
                                  windows are chosen on the host, and CSR arrays given in
                                  device memory are copied to the host for that build        */
    PCSR_FLAG_COLUMN_ORDER = 64,/* S = 1 only: column-ordered schedule.  The work items of
                                  panels that were split run in ascending order of their first
                                  column, dealt to the 8 XCDs as 8 contiguous column ranges,
                                  so that the wavefronts of one XCD gather the same rows of B
                                  at about the same time; all other items run in index order.
                                  The PCSR arrays do not change                                */
    PCSR_FLAG_WINDOW_IF_USEFUL = 128, /* with col_window: keep the window blocks only if the build
                                  finds the structure they need (at least half of the nonzero
                                  vectors inside their block's window and blocks of 128 items or
                                  more on average); otherwise the handle is built as if
                                  col_window were 0 and its kernel parameters are set to auto */
    PCSR_FLAG_ATOMIC_SPLIT = 32 /* S = 1 only: panels that were split accumulate into C with
                                  fp32 atomics, as Algorithm 2 prints it, instead of the
                                  default two-pass write-back (see pcsr_spmm)                 */
};

/*
 * The configuration tuple of Section 3.4 / 4.1, re-expressed for 64-lane wavefronts.
 *   Format parameters (change the PCSR arrays):
 *     V      vector size: rows per panel, 1 or 2 (Section 3.1 limits V to {1,2}).
 *     S      0/1 workload balancing (Section 3.2): cap every work item at SG vectors.
 *     SG     split granularity; 0 = Eq. (3) with `omega`, > 0 = use as given.
 *     omega  lane count used by Eq. (3); 0 = 64 (wavefront).  32 gives the paper's SG.
 *     col_window  column-window blocking: 0 = off, else 256, 512, 1024 or 2048.  Consecutive
 *            work items are cut into blocks of at most col_window items: a block ends
 *            where the rows stop gathering from the stretch of col_window consecutive
 *            columns its first rows use (a community of a clustered graph becomes one
 *            block).  For each block the build picks the window of col_window columns
 *            that holds most of its nonzeros; the kernel stages that window of B (one
 *            grid.y column slice of it) in LDS and gathers from there, and nonzeros
 *            outside the window are gathered from memory as usual.  The PCSR arrays
 *            themselves do not change.  Needs S = 0 and
 *            (col_window + 1)*(lanes_per_row*vec*rep + 4)*4 bytes of LDS <= 160 KiB at launch.
 *   Kernel parameters (launch shape only; the paper's F and W):
 *     lanes_per_row  lanes cooperating on one work item: 4, 8, 16, 32 or 64; 0 = auto.
 *     vec            fp32 values per lane per B load: 1, 2 or 4; must divide K; 0 = auto
 *                    (the widest that divides K; 1 for K of 9..16 when lanes_per_row is
 *                    auto too and rows average 8 vectors or more).
 *     rep            column tiles per lane (the coarsening factor F): 1, 2 or 4; 0 = auto.
 *                    One work item covers lanes_per_row*vec*rep columns of C per grid.y
 *                    slice; wider K is covered by more grid.y slices.
 *     waves_per_wg   wavefronts per workgroup (the paper's W): 1, 2, 4, 8 or 16; 0 = auto.
 *     items_per_group  consecutive work items one lane group walks in a single pass,
 *                    gathering for all of them before any result is needed: 1, 2 or 4;
 *                    0 = auto.  Values above 1 need S = 0, items_per_group <
 *                    lanes_per_row, no work item longer than 1024 vectors and
 *                    V*vec*rep*items_per_group <= 32.
 *   flags   PCSR_FLAG_* bits.
 */
typedef struct {
    int32_t V;
    int32_t S;
    int32_t SG;
    int32_t omega;
    int32_t lanes_per_row;
    int32_t vec;
    int32_t rep;
    int32_t waves_per_wg;
    int32_t flags;
    int32_t items_per_group;
    int32_t col_window;
    int32_t reserved[1]; /* must be 0 */
} pcsr_params_t;

typedef struct pcsr_handle_s *pcsr_handle_t;

/*
 * PCSR generation (Section 4.2, "PCSR Generation"): vectorised blocking of the CSR
 * matrix into V x 1 nonzero vectors, then, if S, the workload split that rewrites
 * rowPtr and emits TRow.
 *   n_rows, n_cols, nnz : shape of A and its stored nonzeros (nnz < 2^31).
 *   rowptr  int32[n_rows+1], colidx int32[nnz], vals fp32[nnz]: host memory, or device
 *           memory when PCSR_FLAG_DEVICE_CSR is set.  Columns of each row must be
 *           strictly ascending (sorted, no duplicates); explicit zeros are kept.
 *   p       parameters; NULL = all defaults (V=1, S=0).
 *   out     receives the handle.  The handle owns device copies of the PCSR arrays on
 *           the device that is current at the call; the caller keeps ownership of the
 *           CSR arrays and may free them on return.
 * Errors: INVALID_ARG, BAD_CSR, UNSUPPORTED, TOO_LARGE, OOM, HIP.  Synchronous.
 */
int pcsr_build(int64_t n_rows, int64_t n_cols, int64_t nnz, const int32_t *rowptr,
               const int32_t *colidx, const float *vals, const pcsr_params_t *p,
               pcsr_handle_t *out);

/*
 * SpMM computing engine (Algorithm 2): C = A * B, overwriting C whatever it held.
 *   B  device, fp32[n_cols x K] row-major, leading dimension K, aligned to 4*vec bytes.
 *   C  device, fp32[n_rows x K] row-major, leading dimension K, same alignment; must
 *      not overlap B.
 *   K  > 0.  One handle serves any K.
 *   stream  a hipStream_t (NULL = the null stream).  The work is enqueued there; the
 *      call does not wait for it.
 * Write-back (Algorithm 2, last block).  S = 0: one plain store per row of C.  S = 1: a
 * panel that the workload split left whole is stored the same way; the items of a panel
 * that was split each leave their partial rows in a workspace owned by the handle
 * (V*K floats per such item) and a second pass adds them and stores the row once: in
 * item order for a panel of up to 64 items; for a longer panel 16 threads per element
 * each add every 16th item in order and the 16 partial sums are then added in order (the
 * order depends on the item numbers alone, not on the launch or the schedule).  No atomics, no clearing of C: for a given handle, kernel parameters and K the
 * result is the same bits on every run, for S = 0 and S = 1 alike.  With
 * PCSR_FLAG_ATOMIC_SPLIT the split panels are cleared and accumulated with fp32 atomics
 * instead (no workspace; summation order, hence the last bits, may vary between runs).
 * Allocation: none, except that an S = 1 handle grows its workspace (a hipMalloc, after
 * a hipFree that waits for the device) on the first call whose K needs more than any
 * call before; pcsr_reserve_workspace does that ahead of time, e.g. before the stream
 * is captured into a HIP graph.  Because of the workspace, SpMMs of one S = 1 handle must
 * not overlap in time (two streams); different handles may.
 * Errors: INVALID_ARG (null or misaligned or overlapping B / C, handle built on another
 * device than the current one), UNSUPPORTED, OOM, HIP.
 */
int pcsr_spmm(pcsr_handle_t h, const float *B, float *C, int32_t K, void *stream);

/*
 * pcsr_spmm for callers that cannot allocate device memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same
 * kernels and bit-identical results, but the workspace of the balanced write-back is a
 * fixed block of pcsr_static_scratch_bytes() bytes (64 MiB) inside the library's device
 * image, one per GPU, held until the process ends; the call never allocates or frees.
 * A call whose workspace need (pcsr_workspace_bytes) exceeds that block returns
 * PCSR_E_TOO_LARGE and enqueues nothing.  Every call on a GPU, from any handle, shares
 * that GPU's block: calls that overlap in time on one GPU (two streams, two threads)
 * race; serialise them.  Nothing in the block has to be cleared between calls (every
 * slot that is read was written earlier in the same call).  The first call on a device
 * looks the block's address up and should be made outside stream capture.
 * Errors: as pcsr_spmm, plus TOO_LARGE; never OOM.
 */
int pcsr_spmm_static(pcsr_handle_t h, const float *B, float *C, int32_t K, void *stream);
int64_t pcsr_static_scratch_bytes(void);

/*
 * Workspace of the balanced write-back (see pcsr_spmm): bytes an SpMM of width K needs
 * (0 for S = 0 handles and under PCSR_FLAG_ATOMIC_SPLIT), and a call that makes the
 * handle's workspace at least that large now.  bytes: host.  pcsr_reserve_workspace
 * allocates and may wait for the device; it must run on the handle's device.
 * Errors: INVALID_ARG, UNSUPPORTED (K <= 0, host-only handle), OOM, HIP.
 */
int pcsr_workspace_bytes(pcsr_handle_t h, int32_t K, int64_t *bytes);
int pcsr_reserve_workspace(pcsr_handle_t h, int32_t K);

/* Releases the handle and its device arrays.  NULL is a no-op.  The caller must make
 * sure no pcsr_spmm using the handle is still running. */
int pcsr_free(pcsr_handle_t h);

/*
 * Changes the kernel-only parameters (lanes_per_row, vec, rep, waves_per_wg,
 * items_per_group, and the PCSR_FLAG_NO_XCD_REMAP and PCSR_FLAG_ATOMIC_SPLIT bits of
 * flags) of an existing handle; 0 = auto.  The PCSR
 * arrays are untouched, so one build can be timed under many launch shapes (the
 * exhaustive sweep that stands in for the training data of Section 5.2).
 * Errors: INVALID_ARG, UNSUPPORTED.
 */
int pcsr_set_kernel_params(pcsr_handle_t h, int32_t lanes_per_row, int32_t vec, int32_t rep,
                           int32_t waves_per_wg, int32_t items_per_group, int32_t flags);

/*
 * Reports the launch shape pcsr_spmm would use for width K with the handle's current
 * kernel parameters (after "auto" resolution): out[0..7] = lanes_per_row, vec, rep,
 * waves_per_wg, grid.x, grid.y, items_per_group, dynamic LDS bytes (0 unless the
 * column-window kernel runs).  Host memory.  Errors: INVALID_ARG, UNSUPPORTED.
 */
int pcsr_query_launch(pcsr_handle_t h, int32_t K, int32_t out[8]);

/*
 * Column-window blocking as built into the handle (host, fp64[3]): col_window, average
 * work items per block, fraction of nonzero vectors that fall inside their block's window
 * (0 when col_window is off).  Errors: INVALID_ARG.
 */
int pcsr_window_stats(pcsr_handle_t h, double out[3]);

/*
 * Copies the PCSR arrays (Section 4.2, "Data Representation") out of the handle for
 * inspection.  sizes (host, int64[6]) receives P (panels), M (work items), nnz_V
 * (vectors), V, SG, has_TRow.  Each of rowptr int32[M+1], colidx int32[nnz_V],
 * val fp32[nnz_V*V], trow int32[M] (host) is filled when non-NULL; pass NULLs first
 * to learn the sizes.  Synchronous (device -> host copies).  Errors: INVALID_ARG, HIP.
 */
int pcsr_export(pcsr_handle_t h, int64_t sizes[6], int32_t *rowptr, int32_t *colidx, float *val,
                int32_t *trow);

/*
 * Launch schedule of the handle, for inspection.  xcd_bounds (host, int32[9], may be NULL):
 * XCD x processes launch positions [xcd_bounds[x], xcd_bounds[x+1]).  Without
 * PCSR_FLAG_COLUMN_ORDER position i is work item i and *n_positions is set to 0.  With it
 * *n_positions = M and sched (host, int32[4*M], may be NULL) receives for every position the
 * record {first vector, vector count, panel, workspace slot or -1} of the item that runs
 * there.  Synchronous.  Errors: INVALID_ARG, HIP.
 */
int pcsr_export_schedule(pcsr_handle_t h, int64_t *n_positions, int32_t *sched, int32_t xcd_bounds[9]);

/*
 * Sparse-matrix features of Table 3, in this order (host, fp64[PCSR_N_FEATURES]):
 *   n, n_hat, nnz, delta, d, d_hat, d_max, CV, CV_hat, SR_1, SR_2, rho, b, b_max,
 *   PR_1, PR_2      (SR: Eq. (4) under S with Eq. (3)'s SG; PR: Eq. (2)),
 * followed by one feature that is not in the paper:
 *   near_512        share of the nonzeros with |column - row| < 512 (0 for nnz = 0).
 * rowptr/colidx: host.  omega as in pcsr_params_t (0 = 64).
 * Errors: INVALID_ARG (n_out < PCSR_N_FEATURES, nulls), BAD_CSR.
 */
#define PCSR_N_FEATURES 17
int pcsr_features(int64_t n_rows, int64_t n_cols, int64_t nnz, const int32_t *rowptr,
                  const int32_t *colidx, int32_t omega, double *out, int32_t n_out);

/*
 * The same features computed by GPU kernels from CSR arrays that already live in device
 * memory (rowptr, colidx: device; out: host).  The CSR is not validated here (pcsr_build
 * does that); values agree with pcsr_features up to the rounding order of the fp64 sums.
 * Synchronous.  Errors: INVALID_ARG, TOO_LARGE, OOM, HIP.
 */
int pcsr_features_device(int64_t n_rows, int64_t n_cols, int64_t nnz, const int32_t *rowptr,
                         const int32_t *colidx, int32_t omega, double *out, int32_t n_out);

/*
 * Configuration prediction (the role of the SpMM-decider, Section 5.2): maps the
 * feature vector and K to a full parameter tuple with a rule distilled from recorded
 * exhaustive sweeps on MI355X.  features: host fp64[PCSR_N_FEATURES]; out: host.
 * Errors: INVALID_ARG, UNSUPPORTED (K <= 0).
 */
int pcsr_select(const double *features, int32_t K, pcsr_params_t *out);

/*
 * Locality reordering pre-step (Section 4.4: a community-based relabelling of the nodes
 * is the default first step of the pipeline and is amortised over many SpMMs).  Own
 * scheme: up to max_rounds (0 = 8) rounds of synchronous label propagation over the
 * pattern of a square matrix, then clusters are numbered one after the other, members
 * in their original order.  Deterministic.
 *   rowptr int32[n+1], colidx int32[nnz]: host.  perm (host, int32[n]) receives the new
 *   id of every node: perm[old] = new.  n_clusters (host, may be NULL) receives the
 *   number of clusters found.
 * The caller applies it: A' = P A P^T (pcsr_permute_csr), B' = P B, and reads C = P^T C'.
 * Errors: INVALID_ARG, BAD_CSR (column >= n), TOO_LARGE, OOM.
 */
int pcsr_reorder(int64_t n, const int32_t *rowptr, const int32_t *colidx, int32_t max_rounds,
                 int32_t *perm, int64_t *n_clusters);

/*
 * Second relabelling for the same pre-step (Section 4.4), meant for power-law inputs, which
 * have hubs rather than communities: nodes are numbered by descending in-degree (how often
 * their row of B is gathered), ties in original order.  The most-gathered rows of B then
 * sit at the lowest ids, so in every row of A the hub columns come first, and a
 * column-ordered schedule (PCSR_FLAG_COLUMN_ORDER) runs the hub-only work items together.
 *   rowptr int32[n+1], colidx int32[nnz]: host.  perm (host, int32[n]): perm[old] = new.
 * Errors: INVALID_ARG, BAD_CSR (column >= n), TOO_LARGE, OOM.
 */
int pcsr_reorder_by_degree(int64_t n, const int32_t *rowptr, const int32_t *colidx, int32_t *perm);

/*
 * Symmetric relabelling of a square CSR matrix: row perm[i] of the output holds row i of
 * the input with every column c replaced by perm[c], columns sorted ascending.
 * All arrays host; outputs sized like the inputs (int32[n+1], int32[nnz], fp32[nnz]).
 * Errors: INVALID_ARG (nulls, perm not a permutation), OOM.
 */
int pcsr_permute_csr(int64_t n, const int32_t *rowptr, const int32_t *colidx, const float *vals,
                     const int32_t *perm, int32_t *out_rowptr, int32_t *out_colidx, float *out_vals);

/*
 * CSR of the transpose (n_cols x n_rows), columns of every output row ascending; used
 * for the backward pass dB = A^T dC when A is embedded in GNN training (Section 6.5).
 * All arrays host; out_rowptr int32[n_cols+1], out_colidx int32[nnz], out_vals fp32[nnz].
 * Errors: INVALID_ARG, BAD_CSR (column out of range), OOM.
 */
int pcsr_transpose_csr(int64_t n_rows, int64_t n_cols, const int32_t *rowptr, const int32_t *colidx,
                       const float *vals, int32_t *out_rowptr, int32_t *out_colidx, float *out_vals);

/* MAC-job gap of Eq. (1) for width dim, coarsening F and lane count omega (0 when dim
 * is a multiple of F*omega, as Table 2 prints).  Returns -1 on non-positive input. */
int32_t pcsr_mac_job_gap(int32_t dim, int32_t F, int32_t omega);

/* Static, never-freed description of an error code. */
const char *pcsr_strerror(int code);

/* hipError_t value of the last failing HIP call seen by this thread (0 if none). */
int pcsr_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* PCSR_H */
