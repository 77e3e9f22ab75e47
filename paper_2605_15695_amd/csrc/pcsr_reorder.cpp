// Locality reordering pre-step (Section 4.4 makes a community-based relabelling the
// default first step of the pipeline).  This is our own light-weight scheme, not the
// third-party algorithm the paper uses: synchronous label propagation groups nodes that
// share neighbours, then nodes are renumbered cluster by cluster, so rows of one cluster
// sit next to each other and gather from a compact set of B rows.
#include <algorithm>
#include <atomic>
#include <cstdint>
#include <cstring>
#include <new>
#include <numeric>
#include <thread>
#include <vector>

#include "../../include/pcsr.h"

namespace {

template <class F> void par_for(int64_t n, F &&fn)
{
    unsigned hw = std::thread::hardware_concurrency();
    int64_t nt = std::max<int64_t>(1, std::min<int64_t>(hw ? hw : 4, 16));
    if (n < 4096) nt = 1;
    if (nt == 1) {
        fn(int64_t(0), n);
        return;
    }
    std::vector<std::thread> th;
    int64_t per = (n + nt - 1) / nt;
    for (int64_t t = 0; t < nt; ++t) {
        int64_t lo = t * per, hi = std::min(n, lo + per);
        if (lo >= hi) break;
        th.emplace_back([=, &fn] { fn(lo, hi); });
    }
    for (auto &t : th) t.join();
}

// deterministic tie-break priority of a label in a given round
inline uint32_t mix(uint32_t x, uint32_t round)
{
    x ^= round * 0x9E3779B9u;
    x ^= x >> 16;
    x *= 0x7feb352du;
    x ^= x >> 15;
    x *= 0x846ca68bu;
    x ^= x >> 16;
    return x;
}

} // namespace

extern "C" {

int pcsr_reorder(int64_t n, const int32_t *rowptr, const int32_t *colidx, int32_t max_rounds,
                 int32_t *perm, int64_t *n_clusters)
{
    if (n < 0 || !rowptr || !perm) return PCSR_E_INVALID_ARG;
    if (n >= (int64_t(1) << 31) - 1) return PCSR_E_TOO_LARGE;
    if (max_rounds <= 0) max_rounds = 8;
    const int64_t nnz = rowptr[n];
    if (nnz > 0 && !colidx) return PCSR_E_INVALID_ARG;
    for (int64_t p = 0; p < nnz; ++p)
        if (colidx[p] < 0 || colidx[p] >= n) return PCSR_E_BAD_CSR; // square pattern required
    try {
        std::vector<int32_t> lab(n), nxt(n);
        std::iota(lab.begin(), lab.end(), 0);
        for (int32_t round = 0; round < max_rounds; ++round) {
            std::vector<int64_t> changed_per(64, 0);
            par_for(n, [&](int64_t lo, int64_t hi) {
                std::vector<int32_t> tmp;
                int64_t changed = 0;
                for (int64_t i = lo; i < hi; ++i) {
                    const int64_t s = rowptr[i], e = rowptr[i + 1];
                    if (e == s) {
                        nxt[i] = lab[i];
                        continue;
                    }
                    tmp.resize(e - s);
                    for (int64_t p = s; p < e; ++p) tmp[p - s] = lab[colidx[p]];
                    std::sort(tmp.begin(), tmp.end());
                    // most frequent neighbour label; ties: keep the current label if it is
                    // among the winners, else the one with the smallest round-salted hash
                    int32_t best = tmp[0];
                    int64_t best_cnt = 0;
                    for (size_t a = 0; a < tmp.size();) {
                        size_t b = a;
                        while (b < tmp.size() && tmp[b] == tmp[a]) ++b;
                        const int64_t cnt = (int64_t)(b - a);
                        const int32_t l = tmp[a];
                        bool take = cnt > best_cnt;
                        if (cnt == best_cnt && best != lab[i])
                            take = (l == lab[i]) || mix((uint32_t)l, round) < mix((uint32_t)best, round);
                        if (take) {
                            best = l;
                            best_cnt = cnt;
                        }
                        a = b;
                    }
                    nxt[i] = best;
                    changed += (best != lab[i]);
                }
                changed_per[(lo * 64) / std::max<int64_t>(n, 1) % 64] += changed;
            });
            lab.swap(nxt);
            int64_t changed = 0;
            for (int64_t c : changed_per) changed += c;
            if (changed * 200 < n) break; // fewer than 0.5 % of the nodes moved
        }
        // renumber: clusters in order of their label, members in original order
        std::vector<int32_t> order(n);
        std::iota(order.begin(), order.end(), 0);
        std::stable_sort(order.begin(), order.end(),
                         [&](int32_t a, int32_t b) { return lab[a] < lab[b]; });
        int64_t clusters = 0;
        for (int64_t k = 0; k < n; ++k) {
            perm[order[k]] = (int32_t)k;
            clusters += (k == 0 || lab[order[k]] != lab[order[k - 1]]);
        }
        if (n_clusters) *n_clusters = clusters;
        return PCSR_OK;
    } catch (const std::bad_alloc &) {
        return PCSR_E_OOM;
    }
}

int pcsr_reorder_by_degree(int64_t n, const int32_t *rowptr, const int32_t *colidx, int32_t *perm)
{
    if (n < 0 || !rowptr || !perm) return PCSR_E_INVALID_ARG;
    if (n >= (int64_t(1) << 31) - 1) return PCSR_E_TOO_LARGE;
    const int64_t nnz = rowptr[n];
    if (nnz < 0 || (nnz > 0 && !colidx)) return PCSR_E_INVALID_ARG;
    try {
        // how often each node is gathered: its in-degree
        std::vector<int64_t> refs(n, 0);
        for (int64_t p = 0; p < nnz; ++p) {
            if (colidx[p] < 0 || colidx[p] >= n) return PCSR_E_BAD_CSR;
            ++refs[colidx[p]];
        }
        std::vector<int32_t> order(n);
        std::iota(order.begin(), order.end(), 0);
        std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return refs[a] > refs[b]; });
        for (int64_t k = 0; k < n; ++k) perm[order[k]] = (int32_t)k;
        return PCSR_OK;
    } catch (const std::bad_alloc &) {
        return PCSR_E_OOM;
    }
}

int pcsr_permute_csr(int64_t n, const int32_t *rowptr, const int32_t *colidx, const float *vals,
                     const int32_t *perm, int32_t *out_rowptr, int32_t *out_colidx, float *out_vals)
{
    if (n < 0 || !rowptr || !perm || !out_rowptr) return PCSR_E_INVALID_ARG;
    const int64_t nnz = rowptr[n];
    if (nnz > 0 && (!colidx || !vals || !out_colidx || !out_vals)) return PCSR_E_INVALID_ARG;
    try {
        // perm must be a permutation of [0, n)
        std::vector<int32_t> inv(n, -1);
        for (int64_t i = 0; i < n; ++i) {
            if (perm[i] < 0 || perm[i] >= n || inv[perm[i]] != -1) return PCSR_E_INVALID_ARG;
            inv[perm[i]] = (int32_t)i;
        }
        out_rowptr[0] = 0;
        for (int64_t k = 0; k < n; ++k) {
            const int64_t i = inv[k];
            out_rowptr[k + 1] = out_rowptr[k] + (rowptr[i + 1] - rowptr[i]);
        }
        std::atomic<int> bad{0};
        par_for(n, [&](int64_t lo, int64_t hi) {
            std::vector<std::pair<int32_t, float>> row;
            for (int64_t k = lo; k < hi; ++k) {
                const int64_t i = inv[k];
                const int64_t s = rowptr[i], e = rowptr[i + 1];
                row.resize(e - s);
                for (int64_t p = s; p < e; ++p) {
                    if (colidx[p] < 0 || colidx[p] >= n) { // not a square pattern: nothing to relabel it to
                        bad = 1;
                        return;
                    }
                    row[p - s] = {perm[colidx[p]], vals[p]};
                }
                std::sort(row.begin(), row.end(),
                          [](const std::pair<int32_t, float> &a, const std::pair<int32_t, float> &b) {
                              return a.first < b.first;
                          });
                int64_t o = out_rowptr[k];
                for (auto &cv : row) {
                    out_colidx[o] = cv.first;
                    out_vals[o] = cv.second;
                    ++o;
                }
            }
        });
        return bad ? PCSR_E_BAD_CSR : PCSR_OK;
    } catch (const std::bad_alloc &) {
        return PCSR_E_OOM;
    }
}

int pcsr_transpose_csr(int64_t n_rows, int64_t n_cols, const int32_t *rowptr, const int32_t *colidx,
                       const float *vals, int32_t *out_rowptr, int32_t *out_colidx, float *out_vals)
{
    if (n_rows < 0 || n_cols < 0 || !rowptr || !out_rowptr) return PCSR_E_INVALID_ARG;
    const int64_t nnz = rowptr[n_rows];
    if (nnz > 0 && (!colidx || !vals || !out_colidx || !out_vals)) return PCSR_E_INVALID_ARG;
    try {
        std::vector<int64_t> cnt(n_cols + 1, 0);
        for (int64_t p = 0; p < nnz; ++p) {
            if (colidx[p] < 0 || colidx[p] >= n_cols) return PCSR_E_BAD_CSR;
            ++cnt[colidx[p] + 1];
        }
        for (int64_t c = 0; c < n_cols; ++c) cnt[c + 1] += cnt[c];
        for (int64_t c = 0; c <= n_cols; ++c) out_rowptr[c] = (int32_t)cnt[c];
        // rows are visited in ascending order, so every output row ends up sorted
        for (int64_t i = 0; i < n_rows; ++i)
            for (int64_t p = rowptr[i]; p < rowptr[i + 1]; ++p) {
                const int64_t o = cnt[colidx[p]]++;
                out_colidx[o] = (int32_t)i;
                out_vals[o] = vals[p];
            }
        return PCSR_OK;
    } catch (const std::bad_alloc &) {
        return PCSR_E_OOM;
    }
}

} // extern "C"
