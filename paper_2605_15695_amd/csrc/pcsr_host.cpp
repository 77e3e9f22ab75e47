// Host-side PCSR generation (Section 4.2, "PCSR Generation") and the matrix features
// of Table 3.  Plain C++ with std::thread; no GPU calls here.
#include "pcsr_host.h"

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstring>
#include <new>
#include <thread>

#include "../../include/pcsr.h"

namespace pcsr {
namespace {

template <class F> void parallel_for(int64_t n, int64_t grain, F &&fn)
{
    if (n <= 0) return;
    unsigned hw = std::thread::hardware_concurrency();
    int64_t nt = std::max<int64_t>(1, std::min<int64_t>(hw ? hw : 4, 16));
    nt = std::min<int64_t>(nt, (n + grain - 1) / grain);
    if (nt <= 1) {
        fn(int64_t(0), n);
        return;
    }
    std::vector<std::thread> th;
    th.reserve(nt);
    int64_t per = (n + nt - 1) / nt;
    for (int64_t t = 0; t < nt; ++t) {
        int64_t lo = t * per, hi = std::min(n, lo + per);
        if (lo >= hi) break;
        th.emplace_back([=, &fn] { fn(lo, hi); });
    }
    for (auto &t : th) t.join();
}

inline int64_t ceildiv(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Number of distinct columns in the union of rows r0 and r0+1 (the second may be absent).
inline int64_t union_count(const int32_t *rowptr, const int32_t *colidx, int64_t r0, int64_t n_rows)
{
    int64_t a = rowptr[r0], ae = rowptr[r0 + 1];
    if (r0 + 1 >= n_rows) return ae - a;
    int64_t b = ae, be = rowptr[r0 + 2], cnt = 0;
    while (a < ae && b < be) {
        int32_t ca = colidx[a], cb = colidx[b];
        a += (ca <= cb);
        b += (cb <= ca);
        ++cnt;
    }
    return cnt + (ae - a) + (be - b);
}

// Eq. (3): SG = ceil(avg vectors per non-empty panel / omega) * omega, in exact integers.
inline int64_t eq3_sg(int64_t nnz_v, int64_t nonempty, int64_t omega)
{
    if (nnz_v == 0 || nonempty == 0) return omega;
    return ceildiv(nnz_v, nonempty * omega) * omega;
}

} // namespace

void balance_xcd_ranges(HostPcsr *hp);

int validate_csr(int64_t n_rows, int64_t n_cols, int64_t nnz, const int32_t *rowptr,
                 const int32_t *colidx)
{
    if (n_rows < 0 || n_cols < 0 || nnz < 0) return PCSR_E_INVALID_ARG;
    if (nnz >= (int64_t(1) << 31) || n_rows >= (int64_t(1) << 31) - 1 || n_cols >= (int64_t(1) << 31))
        return PCSR_E_TOO_LARGE;
    if (!rowptr || (nnz > 0 && !colidx)) return PCSR_E_INVALID_ARG;
    if (rowptr[0] != 0 || rowptr[n_rows] != nnz) return PCSR_E_BAD_CSR;
    std::atomic<int> bad{0};
    parallel_for(n_rows, 1 << 14, [&](int64_t lo, int64_t hi) {
        for (int64_t i = lo; i < hi; ++i) {
            int64_t s = rowptr[i], e = rowptr[i + 1];
            if (s > e || s < 0 || e > nnz) {
                bad = 1;
                return;
            }
            int64_t prev = -1;
            for (int64_t p = s; p < e; ++p) {
                int64_t c = colidx[p];
                if (c <= prev || c >= n_cols) {
                    bad = 1;
                    return;
                }
                prev = c;
            }
        }
    });
    return bad ? PCSR_E_BAD_CSR : PCSR_OK;
}

int build_host(int64_t n_rows, int64_t n_cols, int64_t nnz, const int32_t *rowptr,
               const int32_t *colidx, const float *vals, int32_t V, int32_t S, int32_t SG,
               int32_t omega, HostPcsr *out)
{
    if (V != 1 && V != 2) return PCSR_E_UNSUPPORTED;
    if (SG < 0 || omega < 0) return PCSR_E_INVALID_ARG;
    if (omega == 0) omega = 64;
    try {
        HostPcsr &h = *out;
        h.n_rows = n_rows;
        h.n_cols = n_cols;
        h.nnz = nnz;
        h.V = V;
        h.S = S ? 1 : 0;
        const int64_t P = ceildiv(n_rows, V);
        h.P = P;

        // ---- vectorised blocking: panel row pointer, then column / value fill
        std::vector<int32_t> prow(P + 1);
        prow[0] = 0;
        if (V == 1) {
            std::memcpy(prow.data(), rowptr, sizeof(int32_t) * (n_rows + 1));
            h.nnz_v = nnz;
            h.colidx.assign(colidx, colidx + nnz);
            h.val.assign(vals, vals + nnz);
        } else {
            std::vector<int32_t> cnt(P);
            parallel_for(P, 1 << 13, [&](int64_t lo, int64_t hi) {
                for (int64_t p = lo; p < hi; ++p)
                    cnt[p] = (int32_t)union_count(rowptr, colidx, 2 * p, n_rows);
            });
            int64_t run = 0;
            for (int64_t p = 0; p < P; ++p) {
                run += cnt[p];
                prow[p + 1] = (int32_t)run;
            }
            h.nnz_v = run;
            h.colidx.resize(run);
            h.val.resize(run * 2);
            parallel_for(P, 1 << 13, [&](int64_t lo, int64_t hi) {
                for (int64_t p = lo; p < hi; ++p) {
                    int64_t r0 = 2 * p;
                    int64_t a = rowptr[r0], ae = rowptr[r0 + 1];
                    int64_t b = ae, be = (r0 + 1 < n_rows) ? rowptr[r0 + 2] : ae;
                    int64_t o = prow[p];
                    while (a < ae || b < be) {
                        int32_t ca = a < ae ? colidx[a] : INT32_MAX;
                        int32_t cb = b < be ? colidx[b] : INT32_MAX;
                        int32_t c = std::min(ca, cb);
                        h.colidx[o] = c;
                        h.val[2 * o] = (ca == c) ? vals[a] : 0.0f;
                        h.val[2 * o + 1] = (cb == c) ? vals[b] : 0.0f;
                        a += (ca == c);
                        b += (cb == c);
                        ++o;
                    }
                }
            });
        }

        // ---- split granularity (Eq. 3) is reported even when S is off
        int64_t nonempty = 0;
        for (int64_t p = 0; p < P; ++p) nonempty += (prow[p + 1] > prow[p]);
        const int64_t sg = SG > 0 ? SG : eq3_sg(h.nnz_v, nonempty, omega);
        if (sg >= (int64_t(1) << 31)) return PCSR_E_TOO_LARGE;
        h.SG = (int32_t)sg;

        if (!h.S) {
            h.M = P;
            h.rowptr.swap(prow);
            h.trow.clear();
            int64_t mx = 0;
            for (int64_t p = 0; p < P; ++p) mx = std::max<int64_t>(mx, h.rowptr[p + 1] - h.rowptr[p]);
            h.max_item_len = mx;
            balance_xcd_ranges(&h);
            return PCSR_OK;
        }

        // ---- workload split: panel with l vectors -> max(1, ceil(l/SG)) items
        std::vector<int64_t> first(P + 1);
        first[0] = 0;
        int64_t slots = 0; // items of split panels seen so far (<= M)
        for (int64_t p = 0; p < P; ++p) {
            int64_t l = prow[p + 1] - prow[p];
            int64_t items = std::max<int64_t>(1, ceildiv(l, sg));
            first[p + 1] = first[p] + items;
            if (items > 1) {
                if (slots + items >= (int64_t(1) << 31) - 1) return PCSR_E_TOO_LARGE;
                h.split_panels.push_back((int32_t)p);
                h.split_slot.push_back((int32_t)slots);
                slots += items;
            }
        }
        h.split_slot.push_back((int32_t)slots);
        const int64_t M = first[P];
        if (M >= (int64_t(1) << 31) - 1) return PCSR_E_TOO_LARGE;
        h.M = M;
        h.rowptr.resize(M + 1);
        h.trow.resize(M);
        h.item_slot.assign(M, -1);
        parallel_for(P, 1 << 14, [&](int64_t lo, int64_t hi) {
            for (int64_t p = lo; p < hi; ++p) {
                int64_t start = prow[p];
                for (int64_t it = first[p]; it < first[p + 1]; ++it) {
                    h.rowptr[it] = (int32_t)start;
                    h.trow[it] = (int32_t)p;
                    start += sg;
                }
            }
        });
        for (size_t q = 0; q < h.split_panels.size(); ++q) {
            const int64_t p = h.split_panels[q];
            for (int64_t it = first[p], s = h.split_slot[q]; it < first[p + 1]; ++it, ++s)
                h.item_slot[it] = (int32_t)s;
        }
        h.rowptr[M] = (int32_t)h.nnz_v;
        h.max_item_len = std::min<int64_t>(sg, h.nnz_v);
        balance_xcd_ranges(&h);
        return PCSR_OK;
    } catch (const std::bad_alloc &) {
        return PCSR_E_OOM;
    }
}

void balance_xcd_ranges(HostPcsr *hp)
{
    HostPcsr &h = *hp;
    constexpr int64_t kItemCost = 8; // launch + write-back of one item, in units of one vector
    const int64_t M = h.M;
    const int64_t total = (M ? (int64_t)h.rowptr[M] : 0) + kItemCost * M;
    h.xcd_bounds[0] = 0;
    for (int x = 1; x < 8; ++x) {
        const int64_t target = total * x / 8;
        // smallest i with rowptr[i] + kItemCost*i >= target (monotone in i)
        int64_t lo = 0, hi = M;
        while (lo < hi) {
            const int64_t mid = (lo + hi) / 2;
            if ((int64_t)h.rowptr[mid] + kItemCost * mid >= target)
                hi = mid;
            else
                lo = mid + 1;
        }
        h.xcd_bounds[x] = (int32_t)lo;
    }
    h.xcd_bounds[8] = (int32_t)M;
}

int schedule_by_column(HostPcsr *hp)
{
    HostPcsr &h = *hp;
    constexpr int64_t kItemCost = 8; // as in balance_xcd_ranges
    try {
        const int64_t M = h.M;
        // (first column, item) packed in one key: ascending column, ties in item order.  Items
        // of split panels are never empty, so their first column exists.
        std::vector<uint64_t> keyed;
        std::vector<int32_t> longs, shorts;
        keyed.reserve(h.split_slot.empty() ? 0 : h.split_slot.back());
        shorts.reserve(M - (int64_t)keyed.capacity());
        for (int64_t it = 0; it < M; ++it) {
            if (h.item_slot[it] >= 0)
                keyed.push_back(((uint64_t)(uint32_t)h.colidx[h.rowptr[it]] << 32) | (uint32_t)it);
            else
                shorts.push_back((int32_t)it);
        }
        std::sort(keyed.begin(), keyed.end());
        longs.resize(keyed.size());
        for (size_t i = 0; i < keyed.size(); ++i) longs[i] = (int32_t)(keyed[i] & 0xffffffffu);
        std::vector<uint64_t>().swap(keyed);
        // 8 contiguous slices of equal work (vectors + a per-item cost) of a list
        auto slices = [&](const std::vector<int32_t> &v, int64_t (&b)[9]) {
            std::vector<int64_t> cum(v.size() + 1, 0);
            for (size_t i = 0; i < v.size(); ++i)
                cum[i + 1] = cum[i] + (h.rowptr[v[i] + 1] - h.rowptr[v[i]]) + kItemCost;
            b[0] = 0;
            for (int x = 1; x < 8; ++x)
                b[x] = std::lower_bound(cum.begin(), cum.end(), cum.back() * x / 8) - cum.begin();
            b[8] = (int64_t)v.size();
        };
        int64_t lb[9], sb[9];
        slices(longs, lb);
        slices(shorts, sb);
        h.sched.clear();
        h.sched.reserve(4 * M);
        auto emit = [&](int32_t it) {
            h.sched.push_back(h.rowptr[it]);
            h.sched.push_back(h.rowptr[it + 1] - h.rowptr[it]);
            h.sched.push_back(h.trow[it]);
            h.sched.push_back(h.item_slot[it]);
        };
        h.xcd_bounds[0] = 0;
        for (int x = 0; x < 8; ++x) {
            // the column-ordered part first: its B rows are shared between the waves of the XCD
            for (int64_t i = lb[x]; i < lb[x + 1]; ++i) emit(longs[i]);
            for (int64_t i = sb[x]; i < sb[x + 1]; ++i) emit(shorts[i]);
            h.xcd_bounds[x + 1] = (int32_t)(h.sched.size() / 4);
        }
        return PCSR_OK;
    } catch (const std::bad_alloc &) {
        return PCSR_E_OOM;
    }
}

int choose_windows(HostPcsr *hp, int32_t win_cols)
{
    HostPcsr &h = *hp;
    h.win_cols = win_cols;
    h.win_ptr.clear();
    h.win_start.clear();
    h.win_lo.clear();
    h.win_hi.clear();
    h.win_hit = 0.0;
    if (win_cols <= 0) return PCSR_OK;
    try {
        const int64_t M = h.M;
        constexpr int64_t kProbe = 32;     // items whose columns propose a block's window
        constexpr int64_t kSegment = 8192; // blocks never cross a multiple of this many items, so
                                           // segments can be cut in parallel with the same result
        struct Cut {
            std::vector<int32_t> ptr_end, start; // per block: one past its last item, window start
            int64_t hits = 0;
        };
        const int64_t n_seg = ceildiv(M, kSegment);
        std::vector<Cut> cuts(n_seg);
        parallel_for(n_seg, 1, [&](int64_t s0, int64_t s1) {
            std::vector<int32_t> cols;
            // first column of the densest window of win_cols columns over items [i0, i1), and
            // the vectors that fall inside it
            auto densest = [&](int64_t i0, int64_t i1, int64_t *hits) -> int64_t {
                const int64_t s = h.rowptr[i0], e = h.rowptr[i1];
                *hits = 0;
                if (e <= s) return -1;
                cols.assign(h.colidx.begin() + s, h.colidx.begin() + e);
                std::sort(cols.begin(), cols.end());
                int64_t best = 0, best_lo = 0, l = 0;
                for (int64_t r = 0; r < (int64_t)cols.size(); ++r) {
                    while (cols[r] - cols[l] >= win_cols) ++l;
                    if (r - l + 1 > best) {
                        best = r - l + 1;
                        best_lo = l;
                    }
                }
                int64_t c0 = cols[best_lo];
                c0 = std::min<int64_t>(c0, std::max<int64_t>(0, h.n_cols - win_cols));
                int64_t cnt = 0;
                for (int32_t c : cols) cnt += (c >= c0 && c < c0 + win_cols);
                *hits = cnt;
                return c0;
            };
            for (int64_t sg = s0; sg < s1; ++sg) {
                Cut &cut = cuts[sg];
                const int64_t seg_end = std::min<int64_t>(M, (sg + 1) * kSegment);
                // A block grows item by item while the items keep gathering from the window its
                // first kProbe items proposed (at least half of an item's vectors inside), up
                // to win_cols items; where the matrix has no such structure blocks are kProbe
                // items long.
                for (int64_t i = sg * kSegment; i < seg_end;) {
                    const int64_t probe_end = std::min<int64_t>(seg_end, i + kProbe);
                    int64_t hits = 0;
                    const int64_t c_probe = densest(i, probe_end, &hits);
                    int64_t j = probe_end;
                    if (c_probe >= 0) {
                        for (; j < seg_end && j - i < win_cols; ++j) {
                            const int64_t s = h.rowptr[j], e = h.rowptr[j + 1];
                            if (e == s) continue;
                            const int64_t in =
                                std::lower_bound(h.colidx.begin() + s, h.colidx.begin() + e,
                                                 (int32_t)std::min<int64_t>(c_probe + win_cols, INT32_MAX)) -
                                std::lower_bound(h.colidx.begin() + s, h.colidx.begin() + e, (int32_t)c_probe);
                            if (2 * in < e - s) break;
                        }
                    }
                    // the block's own window; staging costs win_cols row reads, worth it from
                    // two uses per staged row
                    const int64_t c0 = densest(i, j, &hits);
                    if (c0 >= 0 && hits >= 2 * (int64_t)win_cols) {
                        cut.start.push_back((int32_t)c0);
                        cut.hits += hits;
                    } else {
                        cut.start.push_back(-1);
                    }
                    cut.ptr_end.push_back((int32_t)j);
                    i = j;
                }
            }
        });
        int64_t total_hits = 0;
        h.win_ptr.push_back(0);
        for (const Cut &cut : cuts) {
            h.win_ptr.insert(h.win_ptr.end(), cut.ptr_end.begin(), cut.ptr_end.end());
            h.win_start.insert(h.win_start.end(), cut.start.begin(), cut.start.end());
            total_hits += cut.hits;
        }
        h.win_hit = h.nnz_v ? double(total_hits) / double(h.nnz_v) : 0.0;
        // the run of every item that lies inside its block's window
        h.win_lo.resize(M);
        h.win_hi.resize(M);
        const int64_t nb = (int64_t)h.win_start.size();
        parallel_for(nb, 64, [&](int64_t b0, int64_t b1) {
            for (int64_t b = b0; b < b1; ++b) {
                const int64_t c0 = h.win_start[b];
                for (int64_t it = h.win_ptr[b]; it < h.win_ptr[b + 1]; ++it) {
                    const int64_t s = h.rowptr[it], e = h.rowptr[it + 1];
                    if (c0 < 0) {
                        h.win_lo[it] = h.win_hi[it] = (int32_t)s;
                        continue;
                    }
                    const auto first = h.colidx.begin() + s, last = h.colidx.begin() + e;
                    h.win_lo[it] = (int32_t)(std::lower_bound(first, last, (int32_t)c0) - h.colidx.begin());
                    h.win_hi[it] = (int32_t)(std::lower_bound(first, last, (int32_t)std::min<int64_t>(
                                                                               c0 + win_cols, INT32_MAX)) -
                                             h.colidx.begin());
                }
            }
        });
        return PCSR_OK;
    } catch (const std::bad_alloc &) {
        return PCSR_E_OOM;
    }
}

int features_host(int64_t n_rows, int64_t n_cols, int64_t nnz, const int32_t *rowptr,
                  const int32_t *colidx, int32_t omega, double *out)
{
    if (omega == 0) omega = 64;
    if (omega < 0) return PCSR_E_INVALID_ARG;
    int64_t n_hat = 0, d_max = 0, nnz2 = 0, nonempty2 = 0;
    double bw_sum = 0.0, bw_max = 0.0;
    for (int64_t i = 0; i < n_rows; ++i) {
        int64_t s = rowptr[i], e = rowptr[i + 1], l = e - s;
        if (l > 0) {
            ++n_hat;
            d_max = std::max(d_max, l);
            double bw = double(colidx[e - 1]) - double(colidx[s]);
            bw_sum += bw;
            bw_max = std::max(bw_max, bw);
        }
    }
    const double d = n_rows ? double(nnz) / double(n_rows) : 0.0;
    const double d_hat = n_hat ? double(nnz) / double(n_hat) : 0.0;
    double ss = 0.0, ss_hat = 0.0;
    for (int64_t i = 0; i < n_rows; ++i) {
        double l = double(rowptr[i + 1] - rowptr[i]);
        ss += (l - d) * (l - d);
        if (l > 0) ss_hat += (l - d_hat) * (l - d_hat);
    }
    const double cv = d > 0 ? std::sqrt(ss / double(n_rows)) / d : 0.0;
    const double cv_hat = n_hat ? std::sqrt(ss_hat / double(n_hat)) / d_hat : 0.0;

    // V = 2 panel lengths
    const int64_t P2 = ceildiv(n_rows, 2);
    std::vector<int32_t> len2(P2);
    parallel_for(P2, 1 << 13, [&](int64_t lo, int64_t hi) { // the only O(nnz) pass
        for (int64_t p = lo; p < hi; ++p) len2[p] = (int32_t)union_count(rowptr, colidx, 2 * p, n_rows);
    });
    for (int64_t p = 0; p < P2; ++p) {
        nnz2 += len2[p];
        nonempty2 += (len2[p] > 0);
    }
    const int64_t sg1 = eq3_sg(nnz, n_hat, omega), sg2 = eq3_sg(nnz2, nonempty2, omega);
    int64_t M1 = 0, M2 = 0;
    for (int64_t i = 0; i < n_rows; ++i)
        M1 += std::max<int64_t>(1, ceildiv(rowptr[i + 1] - rowptr[i], sg1));
    for (int64_t p = 0; p < P2; ++p) M2 += std::max<int64_t>(1, ceildiv(len2[p], sg2));

    out[0] = double(n_rows);
    out[1] = double(n_hat);
    out[2] = double(nnz);
    out[3] = n_rows ? double(n_hat) / double(n_rows) : 0.0;
    out[4] = d;
    out[5] = d_hat;
    out[6] = double(d_max);
    out[7] = cv;
    out[8] = cv_hat;
    out[9] = n_rows ? double(M1) / double(n_rows) : 1.0;
    out[10] = P2 ? double(M2) / double(P2) : 1.0;
    out[11] = (n_rows && n_cols) ? double(nnz) / (double(n_rows) * double(n_cols)) : 0.0;
    out[12] = n_rows ? bw_sum / double(n_rows) : 0.0;
    out[13] = bw_max;
    out[14] = 0.0;
    out[15] = nnz2 ? 1.0 - double(nnz) / (double(nnz2) * 2.0) : 0.0;
    // Own addition to Table 3: the share of nonzeros within 512 columns of the diagonal
    // (columns ascend inside a row, so two binary searches per row count them).  High for
    // matrices whose rows gather from a neighbourhood of their own index, the case the
    // column-window kernel is for.
    std::atomic<int64_t> near{0};
    parallel_for(n_rows, 1 << 14, [&](int64_t lo, int64_t hi) {
        int64_t cnt = 0;
        for (int64_t i = lo; i < hi; ++i) {
            const int32_t *first = colidx + rowptr[i], *last = colidx + rowptr[i + 1];
            const int64_t c_lo = std::max<int64_t>(i - 511, 0), c_hi = std::min<int64_t>(i + 512, INT32_MAX);
            cnt += std::lower_bound(first, last, (int32_t)c_hi) - std::lower_bound(first, last, (int32_t)c_lo);
        }
        near += cnt;
    });
    out[16] = nnz ? double(near.load()) / double(nnz) : 0.0;
    return PCSR_OK;
}

} // namespace pcsr
