// PCSR generation on the GPU (Section 4.2, "PCSR Generation"): the same two steps as the
// host builder - vectorised blocking into V x 1 nonzero vectors, then the optional
// workload split - but with the CSR arrays already in device memory, so nothing crosses
// PCIe except a handful of scalars.  The arrays it produces are bit-identical to the
// host builder's.
#include <hip/hip_runtime.h>
#include <hipcub/hipcub.hpp>

#include <cmath>
#include <cstdint>
#include <cstring>

#include "../../include/pcsr.h"
#include "pcsr_build_gpu.h"

namespace pcsr {
namespace {

constexpr int kThreads = 256;

inline unsigned blocks_for(int64_t n) { return (unsigned)((n + kThreads - 1) / kThreads); }

// one thread per row: monotone row pointer, columns in range and strictly ascending
__global__ void validate_kernel(int64_t n_rows, int64_t n_cols, int64_t nnz, const int32_t *rowptr,
                                const int32_t *colidx, int *bad)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_rows) return;
    const int64_t s = rowptr[i], e = rowptr[i + 1];
    if (s > e || s < 0 || e > nnz) {
        *bad = 1;
        return;
    }
    int64_t prev = -1;
    for (int64_t p = s; p < e; ++p) {
        const int64_t c = colidx[p];
        if (c <= prev || c >= n_cols) {
            *bad = 1;
            return;
        }
        prev = c;
    }
}

// V = 2, one thread per nonzero, so that a row of 100,000 nonzeros is merged by 100,000
// threads and not by one.  The vectors of panel p are the sorted union of the columns of
// rows 2p ("even") and 2p+1 ("odd"); an element's place in the union follows from two
// counts: the elements of its own row before it, and those of the other row that are
// smaller and not already counted (columns present in both rows are counted with the even
// row).

// index of the row that holds nonzero t: the last r with rowptr[r] <= t
__device__ __forceinline__ int64_t row_of_nonzero(const int32_t *rowptr, int64_t n_rows, int64_t t)
{
    int64_t lo = 0, hi = n_rows; // rowptr[lo] <= t < rowptr[hi]
    while (hi - lo > 1) {
        const int64_t mid = (lo + hi) >> 1;
        if (rowptr[mid] <= t)
            lo = mid;
        else
            hi = mid;
    }
    return lo;
}

// number of entries of colidx[b, e) smaller than c
__device__ __forceinline__ int64_t count_below(const int32_t *colidx, int64_t b, int64_t e, int32_t c)
{
    int64_t lo = b, hi = e;
    while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        if (colidx[mid] < c)
            lo = mid + 1;
        else
            hi = mid;
    }
    return lo - b;
}

// shared[t] = 1 for a nonzero of an odd row whose column also occurs in the even row of
// its panel, else 0; shared[nnz] = 0 (scanned together with the rest)
__global__ void union_shared_kernel(int64_t n_rows, int64_t nnz, const int32_t *rowptr, const int32_t *colidx,
                                    int32_t *shared)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t > nnz) return;
    int32_t flag = 0;
    if (t < nnz) {
        const int64_t r = row_of_nonzero(rowptr, n_rows, t);
        if (r & 1) {
            const int64_t a0 = rowptr[r - 1], a1 = rowptr[r];
            const int32_t c = colidx[t];
            const int64_t k = count_below(colidx, a0, a1, c);
            flag = (a0 + k < a1 && colidx[a0 + k] == c) ? 1 : 0;
        }
    }
    shared[t] = flag;
}

// vectors per panel: both rows' nonzeros minus the columns they share; cnt[P] = 0
__global__ void union_count_kernel(int64_t P, int64_t n_rows, const int32_t *rowptr, const int32_t *shared_scan,
                                   int32_t *cnt)
{
    const int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p > P) return;
    if (p == P) {
        cnt[P] = 0; // scanned together with the panels: prow[P] becomes the total
        return;
    }
    const int64_t r0 = 2 * p;
    const int64_t a0 = rowptr[r0], a1 = rowptr[r0 + 1];
    const int64_t b1 = (r0 + 1 < n_rows) ? rowptr[r0 + 2] : a1;
    cnt[p] = (int32_t)((b1 - a0) - (shared_scan[b1] - shared_scan[a1]));
}

// every nonzero writes its vector (ascending column, +0.0f padding); a column that both
// rows hold is written by the even row's nonzero
__global__ void union_fill_kernel(int64_t n_rows, int64_t nnz, const int32_t *rowptr, const int32_t *colidx,
                                  const float *vals, const int32_t *shared_scan, const int32_t *prow,
                                  int32_t *out_col, float *out_val)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= nnz) return;
    const int64_t r = row_of_nonzero(rowptr, n_rows, t);
    const int64_t p = r >> 1;
    const int32_t c = colidx[t];
    const int64_t a0 = rowptr[2 * p], a1 = rowptr[2 * p + 1];
    const int64_t b1 = (2 * p + 1 < n_rows) ? rowptr[2 * p + 2] : a1;
    if (!(r & 1)) {
        const int64_t k = count_below(colidx, a1, b1, c);                // odd-row columns below c
        const int64_t both = shared_scan[a1 + k] - shared_scan[a1];       // of which also in this row
        const int64_t o = prow[p] + (t - a0) + (k - both);
        const bool twin = a1 + k < b1 && colidx[a1 + k] == c;
        if (o >= prow[p + 1]) return; // only with rows that are not sorted (validation skipped)
        out_col[o] = c;
        out_val[2 * o] = vals[t];
        out_val[2 * o + 1] = twin ? vals[a1 + k] : 0.0f;
    } else if (shared_scan[t + 1] == shared_scan[t]) {                    // not shared
        const int64_t k = count_below(colidx, a0, a1, c);                // even-row columns below c
        const int64_t o = prow[p] + k + ((t - a1) - (shared_scan[t] - shared_scan[a1]));
        if (o >= prow[p + 1]) return;
        out_col[o] = c;
        out_val[2 * o] = 0.0f;
        out_val[2 * o + 1] = vals[t];
    }
}

// stats[0] = non-empty panels, stats[1] = longest panel
__global__ void panel_stats_kernel(int64_t P, const int32_t *prow, unsigned long long *nonempty, int *longest)
{
    const int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int len = 0;
    if (p < P) len = prow[p + 1] - prow[p];
    typedef hipcub::BlockReduce<int, kThreads> Reduce;
    __shared__ typename Reduce::TempStorage t1, t2;
    const int ne = Reduce(t1).Sum(len > 0 ? 1 : 0);
    const int mx = Reduce(t2).Reduce(len, hipcub::Max());
    if (threadIdx.x == 0) {
        if (ne) atomicAdd(nonempty, (unsigned long long)ne);
        if (mx) atomicMax(longest, mx);
    }
}

// work items per panel: max(1, ceil(len / SG))
__global__ void items_kernel(int64_t P, const int32_t *prow, int32_t sg, int32_t *items)
{
    const int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p > P) return;
    if (p == P) {
        items[P] = 0;
        return;
    }
    const int len = prow[p + 1] - prow[p];
    const int it = (int)(((long)len + sg - 1) / sg);
    items[p] = it > 1 ? it : 1;
}

// Panels that own more than one item, in ascending order (positions come from scans, so
// the tables are the same on every run): mark[p] = 1 and cnt[p] = items for such a panel.
__global__ void split_marks_kernel(int64_t P, const int32_t *items, int32_t *mark, int32_t *cnt)
{
    const int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p > P) return;
    const int it = p < P ? items[p] : 0;
    mark[p] = it > 1 ? 1 : 0;
    cnt[p] = it > 1 ? it : 0;
}

// rewritten rowPtr, TRow and the workspace slot of every item (first / slotbase: exclusive
// scans of items / cnt)
__global__ void split_fill_kernel(int64_t P, const int32_t *prow, const int32_t *first,
                                  const int32_t *slotbase, int32_t sg, int32_t *out_rowptr,
                                  int32_t *out_trow, int32_t *out_slot)
{
    const int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= P) return;
    int64_t start = prow[p];
    const int i0 = first[p], i1 = first[p + 1];
    int slot = i1 - i0 > 1 ? slotbase[p] : -1;
    for (int it = i0; it < i1; ++it) {
        out_rowptr[it] = (int32_t)start;
        out_trow[it] = (int32_t)p;
        out_slot[it] = slot;
        if (slot >= 0) ++slot;
        start += sg;
    }
    if (p == P - 1) out_rowptr[i1] = prow[P];
}

// qpos / slotbase: exclusive scans of mark / cnt over P + 1 entries
__global__ void split_tables_kernel(int64_t P, const int32_t *items, const int32_t *qpos,
                                    const int32_t *slotbase, int32_t *split_panels, int32_t *split_slot)
{
    const int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p > P) return;
    if (p == P) {
        split_slot[qpos[P]] = slotbase[P];
        return;
    }
    if (items[p] > 1) {
        const int q = qpos[p];
        split_panels[q] = (int32_t)p;
        split_slot[q] = slotbase[p];
    }
}

// ---- column-ordered schedule (same result as the host builder's schedule_by_column)

// flag[it] = 1 for an item of a split panel (one extra trailing 0 so the scan yields the total)
__global__ void sched_flag_kernel(int64_t M, const int32_t *item_slot, int32_t *flag)
{
    const int64_t it = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (it > M) return;
    flag[it] = (it < M && item_slot[it] >= 0) ? 1 : 0;
}

// long items keyed by their first column (in slot order = item order); the others listed in
// item order.  lrank: exclusive scan of flag.
__global__ void sched_lists_kernel(int64_t M, const int32_t *rowptr, const int32_t *colidx,
                                   const int32_t *item_slot, const int32_t *lrank, int32_t *long_key,
                                   int32_t *long_item, int32_t *short_item)
{
    const int64_t it = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (it >= M) return;
    const int slot = item_slot[it];
    if (slot >= 0) {
        long_key[slot] = colidx[rowptr[it]]; // items of split panels are never empty
        long_item[slot] = (int32_t)it;
    } else {
        short_item[it - lrank[it]] = (int32_t)it;
    }
}

// w[i] = vectors of list[i] + 8 (the per-item cost), w[n] = 0
__global__ void sched_weights_kernel(int64_t n, const int32_t *list, const int32_t *rowptr, long long *w)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i > n) return;
    w[i] = i < n ? (long long)(rowptr[list[i] + 1] - rowptr[list[i]]) + 8 : 0;
}

// 8 contiguous equal-work slices of both lists; cum*: exclusive scans of the weights (n + 1
// entries, the last one the total).  out: lb[9], sb[9], xb[9].
__global__ void sched_bounds_kernel(long nl, const long long *cum_l, long ns, const long long *cum_s,
                                    int32_t *out)
{
    const int x = threadIdx.x;
    if (x > 8) return;
    auto lower = [](const long long *cum, long n, long long target) {
        long lo = 0, hi = n + 1; // first index in [0, n] with cum[index] >= target
        while (lo < hi) {
            const long mid = (lo + hi) / 2;
            if (cum[mid] >= target)
                hi = mid;
            else
                lo = mid + 1;
        }
        return lo > n ? n : lo;
    };
    const long l = x == 0 ? 0 : (x == 8 ? nl : lower(cum_l, nl, cum_l[nl] * x / 8));
    const long sh = x == 0 ? 0 : (x == 8 ? ns : lower(cum_s, ns, cum_s[ns] * x / 8));
    out[x] = (int32_t)l;
    out[9 + x] = (int32_t)sh;
    out[18 + x] = (int32_t)(l + sh);
}

// one record per launch position: XCD x runs its slice of the column-ordered list, then
// its slice of the others
__global__ void sched_emit_kernel(int64_t n, const int32_t *list, int is_short, const int32_t *bounds,
                                  const int32_t *rowptr, const int32_t *trow, const int32_t *item_slot,
                                  int4 *sched)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const int32_t *lb = bounds, *sb = bounds + 9;
    const int32_t *mine = is_short ? sb : lb;
    int x = 0;
    while (x < 7 && i >= mine[x + 1]) ++x;
    const int64_t pos = is_short ? (int64_t)lb[x + 1] + i : (int64_t)sb[x] + i;
    const int it = list[i];
    const int start = rowptr[it];
    sched[pos] = make_int4(start, rowptr[it + 1] - start, trow[it], item_slot[it]);
}

// 8 contiguous item ranges of equal work (vectors + 8 per item); same rule as the host builder
__global__ void xcd_bounds_kernel(int32_t M, const int32_t *rowptr, int32_t *xb)
{
    const int x = threadIdx.x;
    if (x > 8) return;
    if (x == 0) {
        xb[0] = 0;
        return;
    }
    if (x == 8) {
        xb[8] = M;
        return;
    }
    const long total = (long)rowptr[M] + 8L * M;
    const long target = total * x / 8;
    long lo = 0, hi = M;
    while (lo < hi) {
        const long mid = (lo + hi) / 2;
        if ((long)rowptr[mid] + 8L * mid >= target)
            hi = mid;
        else
            lo = mid + 1;
    }
    xb[x] = (int32_t)lo;
}


// ---- Table 3 features on the GPU (two passes over the row pointer, one over colIdx)
struct FeatAcc {
    unsigned long long n_hat, nnz2, nonempty2, M1, M2, near;
    int d_max;
    int pad;
    double bw_sum, bw_max, ss, ss_hat;
};

__device__ inline void atomic_max_double(double *addr, double v)
{
    unsigned long long *a = reinterpret_cast<unsigned long long *>(addr);
    unsigned long long old = *a;
    while (__longlong_as_double((long long)old) < v) {
        const unsigned long long assumed = old;
        old = atomicCAS(a, assumed, (unsigned long long)__double_as_longlong(v));
        if (old == assumed) break;
    }
}

// pass 1: one thread per row (degree, bandwidth) and, for even rows, the V = 2 panel length
__global__ void features_pass1_kernel(int64_t n_rows, const int32_t *rowptr, const int32_t *colidx,
                                      int32_t *len2, FeatAcc *acc)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int nh = 0, dmax = 0, ne2 = 0;
    long l2 = 0, near = 0;
    double bw = 0.0;
    if (i < n_rows) {
        const int64_t s = rowptr[i], e = rowptr[i + 1];
        const int l = (int)(e - s);
        if (l > 0) {
            nh = 1;
            dmax = l;
            bw = (double)colidx[e - 1] - (double)colidx[s];
            // nonzeros with |column - row| < 512: two binary searches in the ascending row
            auto lower = [&](int64_t key) {
                int64_t lo = s, hi = e;
                while (lo < hi) {
                    const int64_t mid = (lo + hi) / 2;
                    if (colidx[mid] < key)
                        lo = mid + 1;
                    else
                        hi = mid;
                }
                return lo;
            };
            near = lower(i + 512) - lower(i - 511);
        }
        if ((i & 1) == 0) {
            int64_t a = s, ae = e, b = e, be = (i + 1 < n_rows) ? rowptr[i + 2] : e, n = 0;
            while (a < ae && b < be) {
                const int32_t ca = colidx[a], cb = colidx[b];
                a += (ca <= cb);
                b += (cb <= ca);
                ++n;
            }
            l2 = n + (ae - a) + (be - b);
            len2[i >> 1] = (int32_t)l2;
            ne2 = l2 > 0;
        }
    }
    typedef hipcub::BlockReduce<int, kThreads> RI;
    typedef hipcub::BlockReduce<long, kThreads> RL;
    typedef hipcub::BlockReduce<double, kThreads> RD;
    __shared__ typename RI::TempStorage ti;
    __shared__ typename RL::TempStorage tl;
    __shared__ typename RD::TempStorage td;
    const int s_nh = RI(ti).Sum(nh);
    __syncthreads();
    const int s_dmax = RI(ti).Reduce(dmax, hipcub::Max());
    __syncthreads();
    const int s_ne2 = RI(ti).Sum(ne2);
    const long s_l2 = RL(tl).Sum(l2);
    __syncthreads();
    const long s_near = RL(tl).Sum(near);
    const double s_bw = RD(td).Sum(bw);
    __syncthreads();
    const double m_bw = RD(td).Reduce(bw, hipcub::Max());
    if (threadIdx.x == 0) {
        if (s_nh) atomicAdd(&acc->n_hat, (unsigned long long)s_nh);
        if (s_dmax) atomicMax(&acc->d_max, s_dmax);
        if (s_ne2) atomicAdd(&acc->nonempty2, (unsigned long long)s_ne2);
        if (s_l2) atomicAdd(&acc->nnz2, (unsigned long long)s_l2);
        if (s_near) atomicAdd(&acc->near, (unsigned long long)s_near);
        if (s_bw != 0.0) atomicAdd(&acc->bw_sum, s_bw);
        if (m_bw > 0.0) atomic_max_double(&acc->bw_max, m_bw);
    }
}

// pass 2: squared deviations of the degrees and the item counts under Eq. (3)'s SG
__global__ void features_pass2_kernel(int64_t n_rows, const int32_t *rowptr, const int32_t *len2, double d,
                                      double d_hat, long sg1, long sg2, FeatAcc *acc)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    double ss = 0.0, ssh = 0.0;
    long m1 = 0, m2 = 0;
    if (i < n_rows) {
        const long l = rowptr[i + 1] - rowptr[i];
        ss = ((double)l - d) * ((double)l - d);
        if (l > 0) ssh = ((double)l - d_hat) * ((double)l - d_hat);
        m1 = (l + sg1 - 1) / sg1;
        if (m1 < 1) m1 = 1;
        if ((i & 1) == 0) {
            m2 = (len2[i >> 1] + sg2 - 1) / sg2;
            if (m2 < 1) m2 = 1;
        }
    }
    typedef hipcub::BlockReduce<long, kThreads> RL;
    typedef hipcub::BlockReduce<double, kThreads> RD;
    __shared__ typename RL::TempStorage tl;
    __shared__ typename RD::TempStorage td;
    const double s_ss = RD(td).Sum(ss);
    __syncthreads();
    const double s_ssh = RD(td).Sum(ssh);
    const long s_m1 = RL(tl).Sum(m1);
    __syncthreads();
    const long s_m2 = RL(tl).Sum(m2);
    if (threadIdx.x == 0) {
        atomicAdd(&acc->ss, s_ss);
        atomicAdd(&acc->ss_hat, s_ssh);
        atomicAdd(&acc->M1, (unsigned long long)s_m1);
        atomicAdd(&acc->M2, (unsigned long long)s_m2);
    }
}

struct Scratch { // frees everything it still owns on scope exit
    void *p[32] = {};
    int n = 0;
    hipError_t alloc(void **out, size_t bytes)
    {
        if (n >= 32) return hipErrorOutOfMemory;
        hipError_t e = hipMalloc(out, bytes ? bytes : 16);
        if (e == hipSuccess) p[n++] = *out;
        return e;
    }
    void release(void *q)
    {
        for (int i = 0; i < n; ++i)
            if (p[i] == q) p[i] = nullptr;
    }
    ~Scratch()
    {
        for (int i = 0; i < n; ++i)
            if (p[i]) (void)hipFree(p[i]);
    }
};

#define HIP_TRY(expr)                  \
    do {                               \
        hipError_t e_ = (expr);        \
        if (e_ != hipSuccess) {        \
            *hip_err = (int)e_;        \
            (void)hipGetLastError();   \
            return e_ == hipErrorOutOfMemory ? PCSR_E_OOM : PCSR_E_HIP; \
        }                              \
    } while (0)

hipError_t exclusive_scan(const int32_t *in, int32_t *out, int64_t n, Scratch &sc)
{
    size_t bytes = 0;
    hipError_t e = hipcub::DeviceScan::ExclusiveSum(nullptr, bytes, in, out, (int)n);
    if (e != hipSuccess) return e;
    void *tmp = nullptr;
    e = sc.alloc(&tmp, bytes);
    if (e != hipSuccess) return e;
    e = hipcub::DeviceScan::ExclusiveSum(tmp, bytes, in, out, (int)n);
    return e;
}

hipError_t exclusive_scan64(const long long *in, long long *out, int64_t n, Scratch &sc)
{
    size_t bytes = 0;
    hipError_t e = hipcub::DeviceScan::ExclusiveSum(nullptr, bytes, in, out, (int)n);
    if (e != hipSuccess) return e;
    void *tmp = nullptr;
    e = sc.alloc(&tmp, bytes);
    if (e != hipSuccess) return e;
    return hipcub::DeviceScan::ExclusiveSum(tmp, bytes, in, out, (int)n);
}

// Column-ordered schedule from the balanced arrays (all device pointers): fills *sched_out
// (4 int32 per launch position, ownership to the caller) and the position bounds per XCD.
int schedule_by_column_device(int64_t M, int64_t n_long, const int32_t *rowptr, const int32_t *colidx,
                              const int32_t *trow, const int32_t *item_slot, int32_t **sched_out,
                              int32_t xcd_bounds[9], int *hip_err)
{
    Scratch sc;
    const int64_t n_short = M - n_long;
    int32_t *flag = nullptr, *lrank = nullptr, *long_key = nullptr, *long_item = nullptr, *short_item = nullptr;
    int32_t *key_sorted = nullptr, *long_sorted = nullptr, *d_bounds = nullptr, *sched = nullptr;
    long long *w_l = nullptr, *w_s = nullptr, *cum_l = nullptr, *cum_s = nullptr;
    HIP_TRY(sc.alloc((void **)&flag, sizeof(int32_t) * (M + 1)));
    HIP_TRY(sc.alloc((void **)&lrank, sizeof(int32_t) * (M + 1)));
    HIP_TRY(sc.alloc((void **)&long_key, sizeof(int32_t) * (n_long + 1)));
    HIP_TRY(sc.alloc((void **)&long_item, sizeof(int32_t) * (n_long + 1)));
    HIP_TRY(sc.alloc((void **)&key_sorted, sizeof(int32_t) * (n_long + 1)));
    HIP_TRY(sc.alloc((void **)&long_sorted, sizeof(int32_t) * (n_long + 1)));
    HIP_TRY(sc.alloc((void **)&short_item, sizeof(int32_t) * (n_short + 1)));
    HIP_TRY(sc.alloc((void **)&w_l, sizeof(long long) * (n_long + 1)));
    HIP_TRY(sc.alloc((void **)&w_s, sizeof(long long) * (n_short + 1)));
    HIP_TRY(sc.alloc((void **)&cum_l, sizeof(long long) * (n_long + 1)));
    HIP_TRY(sc.alloc((void **)&cum_s, sizeof(long long) * (n_short + 1)));
    HIP_TRY(sc.alloc((void **)&d_bounds, sizeof(int32_t) * 27));
    HIP_TRY(sc.alloc((void **)&sched, sizeof(int32_t) * 4 * (M + 1)));

    hipLaunchKernelGGL(sched_flag_kernel, dim3(blocks_for(M + 1)), dim3(kThreads), 0, 0, M, item_slot, flag);
    HIP_TRY(hipGetLastError());
    HIP_TRY(exclusive_scan(flag, lrank, M + 1, sc));
    if (M > 0) {
        hipLaunchKernelGGL(sched_lists_kernel, dim3(blocks_for(M)), dim3(kThreads), 0, 0, M, rowptr, colidx,
                           item_slot, lrank, long_key, long_item, short_item);
        HIP_TRY(hipGetLastError());
    }
    if (n_long > 0) {
        // stable: equal first columns stay in item order, as on the host
        size_t bytes = 0;
        HIP_TRY(hipcub::DeviceRadixSort::SortPairs(nullptr, bytes, long_key, key_sorted, long_item, long_sorted,
                                                   (int)n_long));
        void *tmp = nullptr;
        HIP_TRY(sc.alloc(&tmp, bytes));
        HIP_TRY(hipcub::DeviceRadixSort::SortPairs(tmp, bytes, long_key, key_sorted, long_item, long_sorted,
                                                   (int)n_long));
    }
    hipLaunchKernelGGL(sched_weights_kernel, dim3(blocks_for(n_long + 1)), dim3(kThreads), 0, 0, n_long,
                       long_sorted, rowptr, w_l);
    HIP_TRY(hipGetLastError());
    hipLaunchKernelGGL(sched_weights_kernel, dim3(blocks_for(n_short + 1)), dim3(kThreads), 0, 0, n_short,
                       short_item, rowptr, w_s);
    HIP_TRY(hipGetLastError());
    HIP_TRY(exclusive_scan64(w_l, cum_l, n_long + 1, sc));
    HIP_TRY(exclusive_scan64(w_s, cum_s, n_short + 1, sc));
    hipLaunchKernelGGL(sched_bounds_kernel, dim3(1), dim3(64), 0, 0, (long)n_long, cum_l, (long)n_short, cum_s,
                       d_bounds);
    HIP_TRY(hipGetLastError());
    if (n_long > 0) {
        hipLaunchKernelGGL(sched_emit_kernel, dim3(blocks_for(n_long)), dim3(kThreads), 0, 0, n_long, long_sorted,
                           0, d_bounds, rowptr, trow, item_slot, reinterpret_cast<int4 *>(sched));
        HIP_TRY(hipGetLastError());
    }
    if (n_short > 0) {
        hipLaunchKernelGGL(sched_emit_kernel, dim3(blocks_for(n_short)), dim3(kThreads), 0, 0, n_short, short_item,
                           1, d_bounds, rowptr, trow, item_slot, reinterpret_cast<int4 *>(sched));
        HIP_TRY(hipGetLastError());
    }
    int32_t h_bounds[27];
    HIP_TRY(hipMemcpy(h_bounds, d_bounds, sizeof(h_bounds), hipMemcpyDeviceToHost));
    for (int x = 0; x < 9; ++x) xcd_bounds[x] = h_bounds[18 + x];
    HIP_TRY(hipDeviceSynchronize());
    *sched_out = sched;
    sc.release(sched);
    return PCSR_OK;
}

} // namespace

int build_device(int64_t n_rows, int64_t n_cols, int64_t nnz, const int32_t *d_rowptr,
                 const int32_t *d_colidx, const float *d_vals, int32_t V, int32_t S, int32_t SG,
                 int32_t omega, bool validate, bool column_order, DeviceBuild *out, int *hip_err)
{
    if (V != 1 && V != 2) return PCSR_E_UNSUPPORTED;
    if (omega == 0) omega = 64;
    Scratch sc;
    const int64_t P = (n_rows + V - 1) / V;

    // the row pointer must start at 0 and end at nnz
    int32_t ends[2] = {0, 0};
    HIP_TRY(hipMemcpy(&ends[0], d_rowptr, sizeof(int32_t), hipMemcpyDeviceToHost));
    HIP_TRY(hipMemcpy(&ends[1], d_rowptr + n_rows, sizeof(int32_t), hipMemcpyDeviceToHost));
    if (ends[0] != 0 || ends[1] != nnz) return PCSR_E_BAD_CSR;

    int *d_flags = nullptr; // [0] bad csr, [1] longest panel; [4..5] nonempty (64 bit)
    HIP_TRY(sc.alloc((void **)&d_flags, 8 * sizeof(int)));
    HIP_TRY(hipMemset(d_flags, 0, 8 * sizeof(int)));
    if (validate && n_rows > 0) {
        hipLaunchKernelGGL(validate_kernel, dim3(blocks_for(n_rows)), dim3(kThreads), 0, 0, n_rows, n_cols,
                           nnz, d_rowptr, d_colidx, d_flags);
        HIP_TRY(hipGetLastError());
        int bad = 0;
        HIP_TRY(hipMemcpy(&bad, d_flags, sizeof(int), hipMemcpyDeviceToHost));
        if (bad) return PCSR_E_BAD_CSR;
    }

    // ---- vectorised blocking
    int32_t *prow = nullptr, *pcol = nullptr;
    float *pval = nullptr;
    int64_t nnz_v = nnz;
    HIP_TRY(sc.alloc((void **)&prow, sizeof(int32_t) * (P + 1)));
    if (V == 1) {
        HIP_TRY(hipMemcpy(prow, d_rowptr, sizeof(int32_t) * (n_rows + 1), hipMemcpyDeviceToDevice));
        HIP_TRY(sc.alloc((void **)&pcol, sizeof(int32_t) * (nnz + 1)));
        HIP_TRY(sc.alloc((void **)&pval, sizeof(float) * (nnz + 1)));
        if (nnz) {
            HIP_TRY(hipMemcpy(pcol, d_colidx, sizeof(int32_t) * nnz, hipMemcpyDeviceToDevice));
            HIP_TRY(hipMemcpy(pval, d_vals, sizeof(float) * nnz, hipMemcpyDeviceToDevice));
        }
    } else {
        if (nnz + 1 > 0x7fffffffLL) return PCSR_E_TOO_LARGE; // the scan below counts in int32
        int32_t *cnt = nullptr, *shared = nullptr, *shared_scan = nullptr;
        HIP_TRY(sc.alloc((void **)&cnt, sizeof(int32_t) * (P + 1)));
        HIP_TRY(sc.alloc((void **)&shared, sizeof(int32_t) * (nnz + 1)));
        HIP_TRY(sc.alloc((void **)&shared_scan, sizeof(int32_t) * (nnz + 1)));
        hipLaunchKernelGGL(union_shared_kernel, dim3(blocks_for(nnz + 1)), dim3(kThreads), 0, 0, n_rows, nnz,
                           d_rowptr, d_colidx, shared);
        HIP_TRY(hipGetLastError());
        HIP_TRY(exclusive_scan(shared, shared_scan, nnz + 1, sc));
        hipLaunchKernelGGL(union_count_kernel, dim3(blocks_for(P + 1)), dim3(kThreads), 0, 0, P, n_rows,
                           d_rowptr, shared_scan, cnt);
        HIP_TRY(hipGetLastError());
        HIP_TRY(exclusive_scan(cnt, prow, P + 1, sc));
        int32_t total = 0;
        HIP_TRY(hipMemcpy(&total, prow + P, sizeof(int32_t), hipMemcpyDeviceToHost));
        nnz_v = total;
        HIP_TRY(sc.alloc((void **)&pcol, sizeof(int32_t) * (nnz_v + 1)));
        HIP_TRY(sc.alloc((void **)&pval, sizeof(float) * (2 * nnz_v + 1)));
        if (nnz > 0) {
            hipLaunchKernelGGL(union_fill_kernel, dim3(blocks_for(nnz)), dim3(kThreads), 0, 0, n_rows, nnz,
                               d_rowptr, d_colidx, d_vals, shared_scan, prow, pcol, pval);
            HIP_TRY(hipGetLastError());
        }
    }

    // ---- Eq. (3) from the panel lengths
    if (P > 0) {
        hipLaunchKernelGGL(panel_stats_kernel, dim3(blocks_for(P)), dim3(kThreads), 0, 0, P, prow,
                           reinterpret_cast<unsigned long long *>(d_flags + 4), d_flags + 1);
        HIP_TRY(hipGetLastError());
    }
    int h_flags[8];
    HIP_TRY(hipMemcpy(h_flags, d_flags, sizeof(h_flags), hipMemcpyDeviceToHost));
    unsigned long long nonempty = 0;
    memcpy(&nonempty, &h_flags[4], sizeof(nonempty));
    const int64_t longest = h_flags[1];
    int64_t sg = SG;
    if (sg <= 0) {
        sg = (nnz_v == 0 || nonempty == 0)
                 ? omega
                 : ((nnz_v + (int64_t)nonempty * omega - 1) / ((int64_t)nonempty * omega)) * omega;
    }
    if (sg >= (int64_t(1) << 31)) return PCSR_E_TOO_LARGE;

    out->P = P;
    out->nnz_v = nnz_v;
    out->SG = (int32_t)sg;
    out->n_split = 0;
    out->n_split_items = 0;
    out->trow = nullptr;
    out->split = nullptr;
    out->item_slot = nullptr;
    out->split_slot = nullptr;

    int32_t *final_rowptr = prow;
    int64_t M = P;
    if (!S) {
        out->max_item_len = longest;
    } else {
        if (P + nnz_v / sg >= (int64_t(1) << 31) - 2) return PCSR_E_TOO_LARGE;
        int32_t *items = nullptr, *first = nullptr;
        HIP_TRY(sc.alloc((void **)&items, sizeof(int32_t) * (P + 1)));
        HIP_TRY(sc.alloc((void **)&first, sizeof(int32_t) * (P + 1)));
        hipLaunchKernelGGL(items_kernel, dim3(blocks_for(P + 1)), dim3(kThreads), 0, 0, P, prow, (int32_t)sg,
                           items);
        HIP_TRY(hipGetLastError());
        HIP_TRY(exclusive_scan(items, first, P + 1, sc));
        int32_t m32 = 0;
        HIP_TRY(hipMemcpy(&m32, first + P, sizeof(int32_t), hipMemcpyDeviceToHost));
        M = m32;
        // panels that were split: ascending list, first workspace slot of each
        int32_t *mark = nullptr, *cnt = nullptr, *qpos = nullptr, *slotbase = nullptr;
        HIP_TRY(sc.alloc((void **)&mark, sizeof(int32_t) * (P + 1)));
        HIP_TRY(sc.alloc((void **)&cnt, sizeof(int32_t) * (P + 1)));
        HIP_TRY(sc.alloc((void **)&qpos, sizeof(int32_t) * (P + 1)));
        HIP_TRY(sc.alloc((void **)&slotbase, sizeof(int32_t) * (P + 1)));
        hipLaunchKernelGGL(split_marks_kernel, dim3(blocks_for(P + 1)), dim3(kThreads), 0, 0, P, items, mark,
                           cnt);
        HIP_TRY(hipGetLastError());
        HIP_TRY(exclusive_scan(mark, qpos, P + 1, sc));
        HIP_TRY(exclusive_scan(cnt, slotbase, P + 1, sc));
        int32_t n_split = 0, n_split_items = 0;
        HIP_TRY(hipMemcpy(&n_split, qpos + P, sizeof(int32_t), hipMemcpyDeviceToHost));
        HIP_TRY(hipMemcpy(&n_split_items, slotbase + P, sizeof(int32_t), hipMemcpyDeviceToHost));

        int32_t *srow = nullptr, *trow = nullptr, *item_slot = nullptr;
        HIP_TRY(sc.alloc((void **)&srow, sizeof(int32_t) * (M + 1)));
        HIP_TRY(sc.alloc((void **)&trow, sizeof(int32_t) * (M + 1)));
        HIP_TRY(sc.alloc((void **)&item_slot, sizeof(int32_t) * (M + 1)));
        if (P > 0) {
            hipLaunchKernelGGL(split_fill_kernel, dim3(blocks_for(P)), dim3(kThreads), 0, 0, P, prow, first,
                               slotbase, (int32_t)sg, srow, trow, item_slot);
            HIP_TRY(hipGetLastError());
        } else {
            HIP_TRY(hipMemset(srow, 0, sizeof(int32_t)));
        }
        int32_t *split = nullptr, *split_slot = nullptr;
        HIP_TRY(sc.alloc((void **)&split, sizeof(int32_t) * (n_split + 1)));
        HIP_TRY(sc.alloc((void **)&split_slot, sizeof(int32_t) * (n_split + 1)));
        hipLaunchKernelGGL(split_tables_kernel, dim3(blocks_for(P + 1)), dim3(kThreads), 0, 0, P, items, qpos,
                           slotbase, split, split_slot);
        HIP_TRY(hipGetLastError());
        out->n_split = n_split;
        out->n_split_items = n_split_items;
        out->max_item_len = sg < nnz_v ? sg : nnz_v;
        out->trow = trow;
        out->split = split;
        out->item_slot = item_slot;
        out->split_slot = split_slot;
        sc.release(trow);
        sc.release(split);
        sc.release(item_slot);
        sc.release(split_slot);
        final_rowptr = srow;
    }
    out->M = M;

    int32_t *d_xb = nullptr;
    HIP_TRY(sc.alloc((void **)&d_xb, 9 * sizeof(int32_t)));
    hipLaunchKernelGGL(xcd_bounds_kernel, dim3(1), dim3(64), 0, 0, (int32_t)M, final_rowptr, d_xb);
    HIP_TRY(hipGetLastError());
    HIP_TRY(hipMemcpy(out->xcd_bounds, d_xb, 9 * sizeof(int32_t), hipMemcpyDeviceToHost));
    HIP_TRY(hipDeviceSynchronize());
    out->sched = nullptr;
    if (S && column_order) {
        const int rc = schedule_by_column_device(M, out->n_split_items, final_rowptr, pcol, out->trow,
                                                 out->item_slot, &out->sched, out->xcd_bounds, hip_err);
        if (rc != PCSR_OK) {
            // the arrays already handed to *out go back to the caller's clean-up
            (void)hipFree(out->trow);
            (void)hipFree(out->split);
            (void)hipFree(out->item_slot);
            (void)hipFree(out->split_slot);
            out->trow = out->split = out->item_slot = out->split_slot = nullptr;
            return rc;
        }
    }

    out->rowptr = final_rowptr;
    out->colidx = pcol;
    out->val = pval;
    sc.release(final_rowptr);
    sc.release(pcol);
    sc.release(pval);
    return PCSR_OK;
}

int features_device(int64_t n_rows, int64_t n_cols, int64_t nnz, const int32_t *d_rowptr,
                    const int32_t *d_colidx, int32_t omega, double *out, int *hip_err)
{
    if (omega == 0) omega = 64;
    Scratch sc;
    FeatAcc *d_acc = nullptr;
    int32_t *len2 = nullptr;
    const int64_t P2 = (n_rows + 1) / 2;
    HIP_TRY(sc.alloc((void **)&d_acc, sizeof(FeatAcc)));
    HIP_TRY(sc.alloc((void **)&len2, sizeof(int32_t) * (P2 + 1)));
    HIP_TRY(hipMemset(d_acc, 0, sizeof(FeatAcc)));
    FeatAcc h;
    memset(&h, 0, sizeof(h));
    if (n_rows > 0) {
        hipLaunchKernelGGL(features_pass1_kernel, dim3(blocks_for(n_rows)), dim3(kThreads), 0, 0, n_rows,
                           d_rowptr, d_colidx, len2, d_acc);
        HIP_TRY(hipGetLastError());
        HIP_TRY(hipMemcpy(&h, d_acc, sizeof(h), hipMemcpyDeviceToHost));
    }
    const double d = n_rows ? double(nnz) / double(n_rows) : 0.0;
    const double d_hat = h.n_hat ? double(nnz) / double(h.n_hat) : 0.0;
    auto eq3 = [&](int64_t v, int64_t ne) -> int64_t {
        return (v == 0 || ne == 0) ? omega : ((v + ne * omega - 1) / (ne * omega)) * omega;
    };
    const int64_t sg1 = eq3(nnz, (int64_t)h.n_hat), sg2 = eq3((int64_t)h.nnz2, (int64_t)h.nonempty2);
    if (n_rows > 0) {
        hipLaunchKernelGGL(features_pass2_kernel, dim3(blocks_for(n_rows)), dim3(kThreads), 0, 0, n_rows,
                           d_rowptr, len2, d, d_hat, (long)sg1, (long)sg2, d_acc);
        HIP_TRY(hipGetLastError());
        HIP_TRY(hipMemcpy(&h, d_acc, sizeof(h), hipMemcpyDeviceToHost));
    }
    out[0] = double(n_rows);
    out[1] = double(h.n_hat);
    out[2] = double(nnz);
    out[3] = n_rows ? double(h.n_hat) / double(n_rows) : 0.0;
    out[4] = d;
    out[5] = d_hat;
    out[6] = double(h.d_max);
    out[7] = d > 0 ? sqrt(h.ss / double(n_rows)) / d : 0.0;
    out[8] = h.n_hat ? sqrt(h.ss_hat / double(h.n_hat)) / d_hat : 0.0;
    out[9] = n_rows ? double(h.M1) / double(n_rows) : 1.0;
    out[10] = P2 ? double(h.M2) / double(P2) : 1.0;
    out[11] = (n_rows && n_cols) ? double(nnz) / (double(n_rows) * double(n_cols)) : 0.0;
    out[12] = n_rows ? h.bw_sum / double(n_rows) : 0.0;
    out[13] = h.bw_max;
    out[14] = 0.0;
    out[15] = h.nnz2 ? 1.0 - double(nnz) / (double(h.nnz2) * 2.0) : 0.0;
    out[16] = nnz ? double(h.near) / double(nnz) : 0.0;
    return PCSR_OK;
}

} // namespace pcsr
