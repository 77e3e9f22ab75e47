// SpMM computing engine for gfx950 (wave64): the kernel of Algorithm 2 (Section 4.3),
// laid out for 64-lane wavefronts.
//
// Mapping.  A wavefront is cut into G = 64/LPR groups of LPR lanes; each group owns
// one work item (a row panel, or a slice of one when balancing is on).  Lane l of a
// group covers, for r in [0, REP), the VEC consecutive columns starting at
//   kbase + (r*LPR + l)*VEC,      kbase = blockIdx.y * LPR*VEC*REP,
// so every B load of a group is one contiguous LPR*VEC*4-byte segment.  REP plays the
// role of the coarsening factor F, blockDim/64 the role of W, and the V value slots of
// a nonzero vector reuse each fetched B segment V times.
//
// Traversal.  The group reads its colIdx/val range LPR vectors at a time with one
// coalesced load per lane, then broadcasts vector j to all lanes (v_readlane for a
// full-wave group, ds_bpermute otherwise) and gathers B.  Partial sums of one chunk
// are folded into the running sum once per chunk, which keeps fp32 error growth
// logarithmic-ish on rows with 1e5 nonzeros.
#include "pcsr_kernels.h"

#include <mutex>
#include <type_traits>
#include <set>
#include <utility>

// registers of B data a lane keeps in flight per gather step
#define PCSR_INFLIGHT 16
// balanced (power-law) inputs gather scattered lines: twice as deep (see spmm_kernel)
#define PCSR_INFLIGHT_SPLIT 32
// gathers per step at most
#define PCSR_MAXSTEP 8

// Workspace of the entry point that allocates nothing (pcsr_spmm_static).  In host code
// this name is only a handle for hipGetSymbolAddress; kernels get the looked-up address.
static __device__ __align__(256) unsigned char scratch[pcsr::kStaticScratchBytes];

// Read in place of a row of B by the column-window kernel's memory gathers where an entry
// slot past the end of a chunk, or a column past K, has nothing to load (an address select
// instead of a branch around the load).  Indexed by column within the grid.y slice (at most
// 64 lanes * 4 * 4 columns).
static __device__ __align__(16) float g_zero_row[1024];

namespace pcsr {
namespace {

template <int N> struct Vec;
template <> struct Vec<1> { using type = float; };
template <> struct Vec<2> { using type = float2; };
template <> struct Vec<4> { using type = float4; };

template <int VEC> __device__ __forceinline__ void load_vec(const float *p, float (&d)[VEC])
{
    using T = typename Vec<VEC>::type;
    T t = *reinterpret_cast<const T *>(p);
    if constexpr (VEC == 1) {
        d[0] = t;
    } else if constexpr (VEC == 2) {
        d[0] = t.x;
        d[1] = t.y;
    } else {
        d[0] = t.x;
        d[1] = t.y;
        d[2] = t.z;
        d[3] = t.w;
    }
}

// nontemporal store: C is never read again
template <int VEC> __device__ __forceinline__ void store_vec(float *p, const float (&s)[VEC])
{
    if constexpr (VEC == 1) {
        __builtin_nontemporal_store(s[0], p);
    } else {
        typedef float ext_t __attribute__((ext_vector_type(VEC)));
        ext_t x;
#pragma unroll
        for (int e = 0; e < VEC; ++e) x[e] = s[e];
        __builtin_nontemporal_store(x, reinterpret_cast<ext_t *>(p));
    }
}

// cacheable store: workspace partials are read back by the next kernel
template <int VEC> __device__ __forceinline__ void store_vec_cached(float *p, const float (&s)[VEC])
{
    using T = typename Vec<VEC>::type;
    T t;
    if constexpr (VEC == 1) {
        t = s[0];
    } else if constexpr (VEC == 2) {
        t.x = s[0];
        t.y = s[1];
    } else {
        t.x = s[0];
        t.y = s[1];
        t.z = s[2];
        t.w = s[3];
    }
    *reinterpret_cast<T *>(p) = t;
}

// colIdx / val are read exactly once per SpMM.  (A nontemporal load, meant to keep them
// from displacing B rows in L2, measured no different.)
template <class T> __device__ __forceinline__ T stream_load(const T *p)
{
    return *p;
}

template <int LPR> __device__ __forceinline__ int bcast(int x, int j)
{
    if constexpr (LPR == 64)
        return __builtin_amdgcn_readlane(x, j);
    else
        return __shfl(x, j, LPR);
}
template <int LPR> __device__ __forceinline__ float bcast(float x, int j)
{
    return __int_as_float(bcast<LPR>(__float_as_int(x), j));
}

// Broadcast inside a 16-lane group when the source lane is known at compile time (the
// unrolled step loop): a DPP move, "lane j of every row of 16 to the whole row", which runs
// in the vector ALU instead of going through the LDS crossbar like ds_bpermute.
__device__ __forceinline__ int bcast16_const(int x, int j)
{
#define PCSR_DPP_CASE(J) \
    case J: return __builtin_amdgcn_update_dpp(0, x, 0x150 + J, 0xf, 0xf, false)
    switch (j & 15) {
        PCSR_DPP_CASE(0);
        PCSR_DPP_CASE(1);
        PCSR_DPP_CASE(2);
        PCSR_DPP_CASE(3);
        PCSR_DPP_CASE(4);
        PCSR_DPP_CASE(5);
        PCSR_DPP_CASE(6);
        PCSR_DPP_CASE(7);
        PCSR_DPP_CASE(8);
        PCSR_DPP_CASE(9);
        PCSR_DPP_CASE(10);
        PCSR_DPP_CASE(11);
        PCSR_DPP_CASE(12);
        PCSR_DPP_CASE(13);
        PCSR_DPP_CASE(14);
    default: return __builtin_amdgcn_update_dpp(0, x, 0x150 + 15, 0xf, 0xf, false);
    }
#undef PCSR_DPP_CASE
}
// acc += (lane j of the 16-lane group's a) * b in one instruction: the DPP operand of a
// VOP2 multiply-add does the broadcast, so no separate move is spent on it.
__device__ __forceinline__ void fmac_bcast16_const(float &acc, float a, float b, int j)
{
#define PCSR_FMAC_CASE(J)                                                                             \
    case J:                                                                                           \
        asm("v_fmac_f32_dpp %0, %1, %2 row_newbcast:" #J " row_mask:0xf bank_mask:0xf"                 \
            : "+v"(acc)                                                                               \
            : "v"(a), "v"(b));                                                                        \
        break
    switch (j & 15) {
        PCSR_FMAC_CASE(0);
        PCSR_FMAC_CASE(1);
        PCSR_FMAC_CASE(2);
        PCSR_FMAC_CASE(3);
        PCSR_FMAC_CASE(4);
        PCSR_FMAC_CASE(5);
        PCSR_FMAC_CASE(6);
        PCSR_FMAC_CASE(7);
        PCSR_FMAC_CASE(8);
        PCSR_FMAC_CASE(9);
        PCSR_FMAC_CASE(10);
        PCSR_FMAC_CASE(11);
        PCSR_FMAC_CASE(12);
        PCSR_FMAC_CASE(13);
        PCSR_FMAC_CASE(14);
        PCSR_FMAC_CASE(15);
    }
#undef PCSR_FMAC_CASE
}

template <int LPR, bool CONST_LANE> __device__ __forceinline__ int bcast_any(int x, int j)
{
    if constexpr (LPR == 16 && CONST_LANE)
        return bcast16_const(x, j);
    else
        return bcast<LPR>(x, j);
}
template <int LPR, bool CONST_LANE> __device__ __forceinline__ float bcast_any(float x, int j)
{
    return __int_as_float(bcast_any<LPR, CONST_LANE>(__float_as_int(x), j));
}

template <int V, bool S, int LPR, int VEC, int REP>
__global__ void __launch_bounds__(512) spmm_kernel(SpmmArgs a)
{
    constexpr int G = 64 / LPR;
    // vectors gathered per inner step: 16 registers of B data in flight, 32 for balanced
    // handles and for V = 1 with groups of up to 8 lanes (K <= 32: 4-8 % faster on rows of 40
    // and more nonzeros, no different on short rows; with V = 2 it costs road-like inputs
    // 2-7 %, and with wider groups it changes nothing)
    constexpr bool DEEP = S || (V == 1 && LPR <= 8);
    constexpr int U0 = (DEEP ? PCSR_INFLIGHT_SPLIT : PCSR_INFLIGHT) / (REP * VEC);
    constexpr int Uc = U0 < 1 ? 1 : (U0 > PCSR_MAXSTEP ? PCSR_MAXSTEP : U0);
    constexpr int U = Uc > LPR ? LPR : Uc; // a step never reaches past the group's chunk
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int waves = blockDim.x >> 6;
    // Consecutive workgroup ids go round-robin over the 8 XCDs.  With xcd_remap each XCD
    // walks its own contiguous range of work items (ranges hold equal work, not equal
    // item counts), so neighbouring rows share one L2.
    long item_l = ((long)blockIdx.x * waves + wave) * G + (lane / LPR);
    int limit = a.M;
    if (a.xcd_remap) {
        const int x = blockIdx.x & 7;
        item_l = a.xb[x] + ((long)(blockIdx.x >> 3) * waves + wave) * G + (lane / LPR);
        limit = a.xb[x + 1];
    }
    const int lg = lane & (LPR - 1);
    if (item_l >= limit) return;

    // Everything the item needs to know about itself, fetched in one round trip: its
    // vector range, the panel it writes to (TRow) and its workspace slot (-1: the only
    // item of its panel).  A column-ordered schedule keeps these as one 16-byte record
    // per launch position.
    int head, tail, panel = (int)item_l, slot = -1;
    if constexpr (S) {
        if (a.sched) {
            const int4 rec = a.sched[item_l];
            head = rec.x;
            tail = rec.x + rec.y;
            panel = rec.z;
            slot = rec.w;
        } else {
            head = a.rowptr[item_l];
            tail = a.rowptr[item_l + 1];
            panel = a.trow[item_l];
            slot = a.item_slot[item_l];
        }
    } else {
        head = a.rowptr[item_l];
        tail = a.rowptr[item_l + 1];
    }
    if constexpr (LPR == 64) {
        head = __builtin_amdgcn_readfirstlane(head);
        tail = __builtin_amdgcn_readfirstlane(tail);
    }

    const int kbase = blockIdx.y * (LPR * VEC * REP);
    int kc[REP];
    bool kv[REP];
#pragma unroll
    for (int r = 0; r < REP; ++r) {
        kc[r] = kbase + (r * LPR + lg) * VEC;
        kv[r] = kc[r] < a.K;
    }

    float acc[V][REP][VEC];
#pragma unroll
    for (int v = 0; v < V; ++v)
#pragma unroll
        for (int r = 0; r < REP; ++r)
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc[v][r][e] = 0.0f;

    const float *__restrict__ B = a.B;
    const long K = a.K;

    // one lane's entry of the chunk that starts at `base` (zeros past the end of the range)
    auto load_entry = [&](int base, int &c, float (&av)[V]) {
        const int idx = base + lg;
        c = 0;
#pragma unroll
        for (int v = 0; v < V; ++v) av[v] = 0.0f;
        if (idx < tail) {
            c = stream_load(a.colidx + idx);
            if constexpr (V == 1) {
                av[0] = stream_load(a.val + idx);
            } else {
                typedef float f2 __attribute__((ext_vector_type(2)));
                const f2 t = stream_load(reinterpret_cast<const f2 *>(a.val) + idx);
                av[0] = t[0];
                av[1] = t[1];
            }
        }
    };

    // The next chunk's colIdx/val are requested before the current chunk's gathers, so
    // that a chunk costs one memory round trip, not two.
    int c_next;
    float av_next[V];
    load_entry(head, c_next, av_next);
    for (int base = head; base < tail; base += LPR) {
        const int c = c_next;
        float av[V];
#pragma unroll
        for (int v = 0; v < V; ++v) av[v] = av_next[v];
        load_entry(base + LPR, c_next, av_next);
        const int cnt = min(LPR, tail - base);

        float part[V][REP][VEC];
#pragma unroll
        for (int v = 0; v < V; ++v)
#pragma unroll
            for (int r = 0; r < REP; ++r)
#pragma unroll
                for (int e = 0; e < VEC; ++e) part[v][r][e] = 0.0f;

        // U vectors per step: all broadcasts first, then all gathers, then the FMAs,
        // so U*REP loads are in flight together.  Slots past the end of the range
        // carry val = 0 (set above) and load nothing.  (Branching around those loads
        // measured 1-3 % faster here than reading a row of zeros through an address select,
        // although it costs more instructions: these kernels wait on memory.)
        auto step = [&](int j, auto const_lane) {
            constexpr bool CL = decltype(const_lane)::value;
            int cj[U];
            float aj[U][V];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                cj[u] = bcast_any<LPR, CL>(c, j + u);
#pragma unroll
                for (int v = 0; v < V; ++v) aj[u][v] = bcast_any<LPR, CL>(av[v], j + u);
            }
            float b[U][REP][VEC];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const float *brow = B + (long)cj[u] * K;
                const bool ok = j + u < cnt;
#pragma unroll
                for (int r = 0; r < REP; ++r) {
                    if (ok && kv[r]) {
                        load_vec<VEC>(brow + kc[r], b[u][r]);
                    } else {
#pragma unroll
                        for (int e = 0; e < VEC; ++e) b[u][r][e] = 0.0f;
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int r = 0; r < REP; ++r)
#pragma unroll
                    for (int v = 0; v < V; ++v)
#pragma unroll
                        for (int e = 0; e < VEC; ++e)
                            part[v][r][e] = fmaf(aj[u][v], b[u][r][e], part[v][r][e]);
        };
        if constexpr (LPR == 16) {
            // the 16 / U steps written out, so every broadcast lane is a constant
#pragma unroll
            for (int j = 0; j < LPR; j += U)
                if (j < cnt) step(j, std::true_type{});
        } else {
            for (int j = 0; j < cnt; j += U) step(j, std::false_type{});
        }
#pragma unroll
        for (int v = 0; v < V; ++v)
#pragma unroll
            for (int r = 0; r < REP; ++r)
#pragma unroll
                for (int e = 0; e < VEC; ++e) acc[v][r][e] += part[v][r][e];
    }

    // write-back (Algorithm 2, last block): plain store for an item that is the only one
    // of its panel.  An item of a panel that was split (TRow names the panel) either
    // leaves its partial rows in the workspace slot that belongs to it, for the second
    // pass to add in item order, or, without a workspace, accumulates with atomics.
    const bool sole = slot < 0;
    float *wrow = nullptr;
    if constexpr (S) {
        if (!sole && a.ws) wrow = a.ws + (long)slot * V * K;
    }
#pragma unroll
    for (int v = 0; v < V; ++v) {
        const long row = (long)panel * V + v;
        if (row < a.n_rows) {
            float *crow = wrow ? wrow + v * K : a.C + row * K;
#pragma unroll
            for (int r = 0; r < REP; ++r) {
                if (kv[r]) {
                    if (sole) {
                        store_vec<VEC>(crow + kc[r], acc[v][r]);
                    } else if (wrow) {
                        store_vec_cached<VEC>(crow + kc[r], acc[v][r]);
                    } else {
#pragma unroll
                        for (int e = 0; e < VEC; ++e) atomicAdd(crow + kc[r] + e, acc[v][r][e]);
                    }
                }
            }
        }
    }
}


// Batched walk for matrices of short rows (no balancing): one lane group owns IPG
// consecutive work items and walks their joint colIdx/val range as one stream, so the
// gathers of several rows are in flight together.  Every entry carries the index of the
// item it belongs to and only that item's accumulator takes the multiply-add (a select,
// not a multiplication by zero: a non-finite B row must not leak into rows that do not
// reference it).  IPG-fold ALU work, irrelevant next to the memory time of short rows.
template <int V, int LPR, int VEC, int REP, int IPG>
__global__ void __launch_bounds__(512) spmm_batched_kernel(SpmmArgs a)
{
    static_assert(IPG < LPR, "item boundaries are broadcast from the group's own lanes");
    constexpr int G = 64 / LPR;
    constexpr int U0 = PCSR_INFLIGHT / (REP * VEC);
    constexpr int Uc = U0 < 1 ? 1 : (U0 > 8 ? 8 : U0);
    constexpr int U = Uc > LPR ? LPR : Uc; // a step never reaches past the group's chunk
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int waves = blockDim.x >> 6;
    long item0_l = (((long)blockIdx.x * waves + wave) * G + (lane / LPR)) * IPG;
    int limit = a.M;
    if (a.xcd_remap) { // work-balanced contiguous item range per XCD, as in spmm_kernel
        const int x = blockIdx.x & 7;
        item0_l = a.xb[x] + (((long)(blockIdx.x >> 3) * waves + wave) * G + (lane / LPR)) * IPG;
        limit = a.xb[x + 1];
    }
    const int lg = lane & (LPR - 1);
    if (item0_l >= limit) return;
    const int item0 = (int)item0_l;

    const int kbase = blockIdx.y * (LPR * VEC * REP);
    int kc[REP];
    bool kv[REP];
#pragma unroll
    for (int r = 0; r < REP; ++r) {
        kc[r] = kbase + (r * LPR + lg) * VEC;
        kv[r] = kc[r] < a.K;
    }

    // item boundaries: lane i of the group fetches rowPtr[item0 + i], i <= IPG
    const int bsel = item0 + (lg < IPG ? lg : IPG);
    const int my_rp = a.rowptr[bsel < limit ? bsel : limit];
    int rp[IPG + 1];
#pragma unroll
    for (int i = 0; i <= IPG; ++i) rp[i] = bcast<LPR>(my_rp, i);
    const int head = rp[0], tail = rp[IPG];

    float acc[IPG][V][REP][VEC];
#pragma unroll
    for (int i = 0; i < IPG; ++i)
#pragma unroll
        for (int v = 0; v < V; ++v)
#pragma unroll
            for (int r = 0; r < REP; ++r)
#pragma unroll
                for (int e = 0; e < VEC; ++e) acc[i][v][r][e] = 0.0f;

    const float *__restrict__ B = a.B;
    const long K = a.K;

    for (int base = head; base < tail; base += LPR) {
        const int idx = base + lg;
        int c = 0, tag = 0;
        float av[V];
#pragma unroll
        for (int v = 0; v < V; ++v) av[v] = 0.0f;
        if (idx < tail) {
            c = stream_load(a.colidx + idx);
            if constexpr (V == 1) {
                av[0] = stream_load(a.val + idx);
            } else {
                typedef float f2 __attribute__((ext_vector_type(2)));
                const f2 t = stream_load(reinterpret_cast<const f2 *>(a.val) + idx);
                av[0] = t[0];
                av[1] = t[1];
            }
#pragma unroll
            for (int i = 1; i < IPG; ++i) tag += (idx >= rp[i]);
        }
        const int cnt = min(LPR, tail - base);
        for (int j = 0; j < cnt; j += U) {
            int cj[U], tj[U];
            float aj[U][V];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                cj[u] = bcast<LPR>(c, j + u);
                tj[u] = bcast<LPR>(tag, j + u);
#pragma unroll
                for (int v = 0; v < V; ++v) aj[u][v] = bcast<LPR>(av[v], j + u);
            }
            float b[U][REP][VEC];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const float *brow = B + (long)cj[u] * K;
                const bool ok = j + u < cnt;
#pragma unroll
                for (int r = 0; r < REP; ++r) {
                    if (ok && kv[r]) {
                        load_vec<VEC>(brow + kc[r], b[u][r]);
                    } else {
#pragma unroll
                        for (int e = 0; e < VEC; ++e) b[u][r][e] = 0.0f;
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int i = 0; i < IPG; ++i)
#pragma unroll
                    for (int v = 0; v < V; ++v) {
                        const bool mine = tj[u] == i;
#pragma unroll
                        for (int r = 0; r < REP; ++r)
#pragma unroll
                            for (int e = 0; e < VEC; ++e) {
                                const float t = fmaf(aj[u][v], b[u][r][e], acc[i][v][r][e]);
                                acc[i][v][r][e] = mine ? t : acc[i][v][r][e];
                            }
                    }
        }
    }

#pragma unroll
    for (int i = 0; i < IPG; ++i) {
        const long item = (long)item0 + i;
        if (item < limit) {
#pragma unroll
            for (int v = 0; v < V; ++v) {
                const long row = item * V + v;
                if (row < a.n_rows) {
                    float *crow = a.C + row * K;
#pragma unroll
                    for (int r = 0; r < REP; ++r)
                        if (kv[r]) store_vec<VEC>(crow + kc[r], acc[i][v][r]);
                }
            }
        }
    }
}

// Column-window kernel (no balancing): one workgroup owns a block of consecutive work items
// (cut at build time where the rows move on to other columns) and one grid.y column slice.  It first copies rows [c0, c0 + win_cols) of
// that B slice into LDS (c0 chosen at build time as the densest window of the block's
// columns), then walks its items like spmm_kernel, taking each B segment from LDS when
// the column falls inside the window and from memory otherwise.  On clustered matrices
// most gathers then cost LDS bandwidth instead of L2 round trips: a compute unit can only
// keep a few hundred cache lines in flight, which caps L2-resident gathers near 23 TB/s
// on the whole chip, while its LDS delivers 128 bytes per clock.
// Everything that would put a memory round trip into the walk is requested one step ahead:
// the next item's vector range while the current item is processed, the next chunk of
// colIdx/val while the current chunk's rows are read.
template <int V, int LPR, int VEC, int REP>
__global__ void __launch_bounds__(1024) spmm_window_kernel(SpmmArgs a)
{
    extern __shared__ __align__(16) float lds[];
    constexpr int G = 64 / LPR;
    constexpr int TW = LPR * VEC * REP; // columns per slice
    constexpr int LW = TW + 4;          // floats per staged row, padded so rows start on different banks
    // Vectors per step.  The LDS window caps a compute unit at one or two workgroups, so a
    // wavefront may use many registers: memory gathers go 64 registers deep (the few
    // out-of-window vectors of an item then cost one round trip), LDS reads 32.
    constexpr int UG0 = 64 / (REP * VEC), UL0 = 32 / (REP * VEC);
    constexpr int UGc = UG0 < 1 ? 1 : (UG0 > 16 ? 16 : UG0), ULc = UL0 < 1 ? 1 : (UL0 > 16 ? 16 : UL0);
    constexpr int UG = UGc > LPR ? LPR : UGc; // a step never reaches past the group's chunk
    constexpr int UL = ULc > LPR ? LPR : ULc;
    // out-of-window vectors of an item whose gathers are issued before its LDS walk and used
    // after it (32 registers held across the walk)
    constexpr int UP = UL;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int waves = blockDim.x >> 6;
    int bid = blockIdx.x;
    if (a.xcd_remap) {
        const int x = bid & 7, idx = bid >> 3;
        const int q = a.nblk >> 3, r = a.nblk & 7;
        bid = x * q + (x < r ? x : r) + idx;
    }
    const int lg = lane & (LPR - 1);
    const int kbase = blockIdx.y * TW;
    const float *__restrict__ B = a.B;
    const long K = a.K;

    const int item_begin = a.win_ptr[bid];
    const int item_end = a.win_ptr[bid + 1];
    const int stride = waves * G;
    int item = item_begin + wave * G + lane / LPR;
    // the first item's ranges are requested before the window is staged
    int head = 0, tail = 0, lo = 0, hi = 0;
    if (item < item_end) {
        head = a.rowptr[item];
        tail = a.rowptr[item + 1];
        lo = a.win_lo[item];
        hi = a.win_hi[item];
    }

    const int c0 = a.win_start[bid];
    if (c0 >= 0) { // uniform over the workgroup
        constexpr int VPR = TW / VEC; // vector loads per staged row
        const int total = (a.win_cols + 1) * VPR; // the window, then one row of zeros
        for (int q = tid; q < total; q += blockDim.x) {
            const int r = q / VPR;
            const int e = (q - r * VPR) * VEC;
            const int col = c0 + r;
            float t[VEC];
            if (r < a.win_cols && col < a.n_cols && kbase + e < a.K) {
                load_vec<VEC>(B + (long)col * K + kbase + e, t);
            } else {
#pragma unroll
                for (int i = 0; i < VEC; ++i) t[i] = 0.0f;
            }
            store_vec_cached<VEC>(lds + r * LW + e, t);
        }
    }

    int kl[REP]; // column offset inside the slice
    bool kv[REP];
#pragma unroll
    for (int r = 0; r < REP; ++r) {
        kl[r] = (r * LPR + lg) * VEC;
        kv[r] = kbase + kl[r] < a.K;
    }

    // This lane's entry of the chunk that starts at member i0 of a walk: the walk's i-th
    // member is vector first + i (i < n1) or second + (i - n1); zeros past its n members.
    auto load_entry = [&](int first, int n1, int second, int n, int i0, int &c, float (&av)[V]) {
        const int i = i0 + lg;
        c = 0;
#pragma unroll
        for (int v = 0; v < V; ++v) av[v] = 0.0f;
        if (i < n) {
            const int idx = i < n1 ? first + i : second + (i - n1);
            c = stream_load(a.colidx + idx);
            if constexpr (V == 1) {
                av[0] = stream_load(a.val + idx);
            } else {
                typedef float f2 __attribute__((ext_vector_type(2)));
                const f2 t = stream_load(reinterpret_cast<const f2 *>(a.val) + idx);
                av[0] = t[0];
                av[1] = t[1];
            }
        }
    };
    // first chunk of both walks of the current item, requested while the previous item was
    // still being processed (here: before the window is complete)
    int cg0, cl0;
    float avg0[V], avl0[V];
    load_entry(head, lo - head, hi, (lo - head) + (tail - hi), 0, cg0, avg0);
    load_entry(lo, hi - lo, lo, hi - lo, 0, cl0, avl0);
    if (c0 >= 0) __syncthreads(); // the staged window is complete (uniform over the workgroup)

    while (item < item_end) {
        // ranges of the item this group takes next
        const int item_next = item + stride;
        int head_next = 0, tail_next = 0, lo_next = 0, hi_next = 0;
        if (item_next < item_end) {
            head_next = a.rowptr[item_next];
            tail_next = a.rowptr[item_next + 1];
            lo_next = a.win_lo[item_next];
            hi_next = a.win_hi[item_next];
        }

        float acc[V][REP][VEC];
#pragma unroll
        for (int v = 0; v < V; ++v)
#pragma unroll
            for (int r = 0; r < REP; ++r)
#pragma unroll
                for (int e = 0; e < VEC; ++e) acc[v][r][e] = 0.0f;

        // Walks the n vectors whose i-th member is vector first + i (i < n1) or
        // second + (i - n1): one contiguous run, or two runs taken as one.  The columns of an
        // item ascend, so the vectors inside the window are one run [lo, hi) and the others
        // the two runs around it; each kind is walked on its own, the memory gathers with
        // several loads in flight and no LDS access in between, the LDS reads with no memory
        // round trip in between.
        auto walk = [&](int first, int n1, int second, int n, int i_start, int c_first,
                        const float (&av_first)[V], auto from_lds) {
            constexpr bool LDS = decltype(from_lds)::value;
            constexpr int U = LDS ? UL : UG;
            int c_next = c_first;
            float av_next[V];
#pragma unroll
            for (int v = 0; v < V; ++v) av_next[v] = av_first[v];
            for (int base = i_start; base < n; base += LPR) {
                const int c = c_next;
                float av[V];
#pragma unroll
                for (int v = 0; v < V; ++v) av[v] = av_next[v];
                load_entry(first, n1, second, n, base + LPR, c_next, av_next);
                const int cnt = min(LPR, n - base);
                // where this lane's entry sits in the staged window (floats from lds); a slot
                // past the end of the run reads the row of zeros staged after the window
                const int loff = LDS ? (base + lg < n ? c - c0 : a.win_cols) * LW : 0;
                float part[V][REP][VEC];
#pragma unroll
                for (int v = 0; v < V; ++v)
#pragma unroll
                    for (int r = 0; r < REP; ++r)
#pragma unroll
                        for (int e = 0; e < VEC; ++e) part[v][r][e] = 0.0f;

                auto step = [&](int j, auto const_lane) {
                    constexpr bool CL = decltype(const_lane)::value;
                    // LDS reads of a 16-lane group with constant source lanes: the broadcast of
                    // the value rides on the multiply-add, and the row's LDS offset was
                    // computed once by the lane that holds the entry
                    constexpr bool FUSED = LDS && CL && LPR == 16;
                    int cj[U];
                    float aj[U][V];
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        cj[u] = bcast_any<LPR, CL>(LDS ? loff : c, j + u);
                        if constexpr (!FUSED) {
#pragma unroll
                            for (int v = 0; v < V; ++v) aj[u][v] = bcast_any<LPR, CL>(av[v], j + u);
                        }
                    }
                    float b[U][REP][VEC];
#pragma unroll
                    for (int u = 0; u < U; ++u) {
#pragma unroll
                        for (int r = 0; r < REP; ++r) {
                            if constexpr (LDS) {
                                // one ds_read of VEC floats, never predicated: slots past the
                                // end point at the zero row, columns past K were staged as zeros
                                load_vec<VEC>(lds + cj[u] + kl[r], b[u][r]);
                            } else {
                                const bool ok = j + u < cnt;
                                const float *src = (ok && kv[r]) ? B + (long)cj[u] * K + kbase + kl[r]
                                                                 : g_zero_row + kl[r];
                                load_vec<VEC>(src, b[u][r]);
                            }
                        }
                    }
#pragma unroll
                    for (int u = 0; u < U; ++u)
#pragma unroll
                        for (int r = 0; r < REP; ++r)
#pragma unroll
                            for (int v = 0; v < V; ++v)
#pragma unroll
                                for (int e = 0; e < VEC; ++e) {
                                    if constexpr (FUSED)
                                        fmac_bcast16_const(part[v][r][e], av[v], b[u][r][e], j + u);
                                    else
                                        part[v][r][e] = fmaf(aj[u][v], b[u][r][e], part[v][r][e]);
                                }
                };
                if constexpr (LPR == 16) {
#pragma unroll
                    for (int j = 0; j < LPR; j += U)
                        if (j < cnt) step(j, std::true_type{});
                } else {
                    for (int j = 0; j < cnt; j += U) step(j, std::false_type{});
                }
#pragma unroll
                for (int v = 0; v < V; ++v)
#pragma unroll
                    for (int r = 0; r < REP; ++r)
#pragma unroll
                        for (int e = 0; e < VEC; ++e) acc[v][r][e] += part[v][r][e];
            }
        };
        // Outside the window: memory gathers.  Those of the first UP such vectors are only
        // issued here; the LDS walk below runs while they are in flight, then they are added.
        const int n_out = (lo - head) + (tail - hi);
        float gb[UP][REP][VEC];
#pragma unroll
        for (int u = 0; u < UP; ++u) {
            const int cu = bcast_any<LPR, true>(cg0, u);
#pragma unroll
            for (int r = 0; r < REP; ++r) {
                const float *src = (u < n_out && kv[r]) ? B + (long)cu * K + kbase + kl[r] : g_zero_row + kl[r];
                load_vec<VEC>(src, gb[u][r]);
            }
        }
        // the next item's first chunks: its ranges have arrived by now, and the LDS walk
        // below covers the latency of these loads
        int cg0_next, cl0_next;
        float avg0_next[V], avl0_next[V];
        load_entry(head_next, lo_next - head_next, hi_next, (lo_next - head_next) + (tail_next - hi_next), 0,
                   cg0_next, avg0_next);
        load_entry(lo_next, hi_next - lo_next, lo_next, hi_next - lo_next, 0, cl0_next, avl0_next);
        // inside the window: LDS reads
        walk(lo, hi - lo, lo, hi - lo, 0, cl0, avl0, std::true_type{});
        // the gathers issued above
#pragma unroll
        for (int u = 0; u < UP; ++u)
#pragma unroll
            for (int r = 0; r < REP; ++r)
#pragma unroll
                for (int v = 0; v < V; ++v)
#pragma unroll
                    for (int e = 0; e < VEC; ++e) {
                        if constexpr (LPR == 16)
                            fmac_bcast16_const(acc[v][r][e], avg0[v], gb[u][r][e], u);
                        else
                            acc[v][r][e] = fmaf(bcast<LPR>(avg0[v], u), gb[u][r][e], acc[v][r][e]);
                    }
        // the rare item with more out-of-window vectors than that: the rest, one step at a time
        if (n_out > UP) {
            int cg;
            float avg[V];
            load_entry(head, lo - head, hi, n_out, UP, cg, avg);
            walk(head, lo - head, hi, n_out, UP, cg, avg, std::false_type{});
        }

#pragma unroll
        for (int v = 0; v < V; ++v) {
            const long row = (long)item * V + v;
            if (row < a.n_rows) {
                float *crow = a.C + row * K + kbase;
#pragma unroll
                for (int r = 0; r < REP; ++r)
                    if (kv[r]) store_vec<VEC>(crow + kl[r], acc[v][r]);
            }
        }
        item = item_next;
        head = head_next;
        tail = tail_next;
        lo = lo_next;
        hi = hi_next;
        cg0 = cg0_next;
        cl0 = cl0_next;
#pragma unroll
        for (int v = 0; v < V; ++v) {
            avg0[v] = avg0_next[v];
            avl0[v] = avl0_next[v];
        }
    }
}

__global__ void __launch_bounds__(256) zero_panels_kernel(const int32_t *__restrict__ panels,
                                                          long n_panels, int V, float *C,
                                                          int n_rows, int K)
{
    // one thread per fp32 element of the listed rows
    const long total = n_panels * V * (long)K;
    for (long t = (long)blockIdx.x * blockDim.x + threadIdx.x; t < total;
         t += (long)gridDim.x * blockDim.x) {
        const long r = t / K;
        const int k = (int)(t - r * K);
        const long row = (long)panels[r / V] * V + (r % V);
        if (row < n_rows) C[row * K + k] = 0.0f;
    }
}

// One thread per VEC consecutive elements (q, v, k..k+VEC) of the rows of split panels.  The
// partial rows of panel q sit in consecutive workspace slots in item order and are added in
// that order, whatever the grid looks like, so the balanced result is the same bits on
// every run.  Panels with more than `skip_above` slots are left to reduce_long_kernel.
template <int VEC>
__global__ void __launch_bounds__(256) reduce_split_kernel(const int32_t *__restrict__ split_panels,
                                                           const int32_t *__restrict__ split_slot,
                                                           long n_split, int V, const float *__restrict__ ws,
                                                           float *C, int n_rows, int K, int skip_above)
{
    const int kv = K / VEC; // vectors per row
    const long total = n_split * V * (long)kv;
    const long t = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= total) return;
    const long r = t / kv;
    const int k = (int)(t - r * kv) * VEC;
    const long q = r / V;
    const int v = (int)(r - q * V);
    const long row = (long)split_panels[q] * V + v;
    if (row >= n_rows) return;
    const long s0 = split_slot[q], s1 = split_slot[q + 1];
    if (s1 - s0 > skip_above) return;
    const long stride = (long)V * K;
    const float *w = ws + (s0 * V + v) * (long)K + k;
    float sum[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) sum[e] = 0.0f;
    long j = s0;
    for (; j + 4 <= s1; j += 4, w += 4 * stride) { // four loads in flight, adds in item order
        float t4[4][VEC];
#pragma unroll
        for (int u = 0; u < 4; ++u) load_vec<VEC>(w + u * stride, t4[u]);
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int e = 0; e < VEC; ++e) sum[e] += t4[u][e];
    }
    for (; j < s1; ++j, w += stride) {
        float t1[VEC];
        load_vec<VEC>(w, t1);
#pragma unroll
        for (int e = 0; e < VEC; ++e) sum[e] += t1[e];
    }
    store_vec<VEC>(C + row * K + k, sum);
}

// Split panels with many partial rows (a hub row of a power-law graph is cut into thousands
// of items): one workgroup per (panel row, 16 vectors of C), 16 threads per vector.  Thread
// j of a vector adds slots j, j+16, j+32, ... in ascending order, then the 16 partial sums
// are added in ascending j.  The order depends on the slot numbers alone, so the result is
// again the same bits on every run and for every schedule.
template <int VEC>
__global__ void __launch_bounds__(256) reduce_long_kernel(const int32_t *__restrict__ long_panels,
                                                          const int32_t *__restrict__ split_panels,
                                                          const int32_t *__restrict__ split_slot, int V,
                                                          const float *__restrict__ ws, float *C, int n_rows,
                                                          int K)
{
    __shared__ float part[kLongReduceLanes][16][VEC];
    const int c = threadIdx.x % 16, j = threadIdx.x / 16;
    const long r = blockIdx.x;
    const long q = long_panels[r / V];
    const int v = (int)(r % V);
    const long row = (long)split_panels[q] * V + v;
    if (row >= n_rows) return; // the whole workgroup leaves: no barrier is skipped by a part of it
    const int k = ((int)blockIdx.y * 16 + c) * VEC;
    const bool live = k < K;
    const long s0 = split_slot[q], s1 = split_slot[q + 1];
    const long stride = (long)V * K, step = kLongReduceLanes * stride;
    float sum[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) sum[e] = 0.0f;
    if (live) {
        long jj = s0 + j;
        const float *w = ws + (jj * V + v) * (long)K + k;
        for (; jj + 3 * kLongReduceLanes < s1; jj += 4 * kLongReduceLanes, w += 4 * step) {
            float t4[4][VEC];
#pragma unroll
            for (int u = 0; u < 4; ++u) load_vec<VEC>(w + u * step, t4[u]);
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int e = 0; e < VEC; ++e) sum[e] += t4[u][e];
        }
        for (; jj < s1; jj += kLongReduceLanes, w += step) {
            float t1[VEC];
            load_vec<VEC>(w, t1);
#pragma unroll
            for (int e = 0; e < VEC; ++e) sum[e] += t1[e];
        }
    }
#pragma unroll
    for (int e = 0; e < VEC; ++e) part[j][c][e] = sum[e];
    __syncthreads();
    if (j == 0 && live) {
        for (int jj = 1; jj < kLongReduceLanes; ++jj)
#pragma unroll
            for (int e = 0; e < VEC; ++e) sum[e] += part[jj][c][e];
        store_vec<VEC>(C + row * K + k, sum);
    }
}

using KernelFn = void (*)(SpmmArgs);

template <int V, bool S, int LPR, int VEC> KernelFn pick_rep(int rep)
{
    switch (rep) {
    case 1: return &spmm_kernel<V, S, LPR, VEC, 1>;
    case 2: return &spmm_kernel<V, S, LPR, VEC, 2>;
    case 4: return &spmm_kernel<V, S, LPR, VEC, 4>;
    }
    return nullptr;
}
template <int V, bool S, int LPR> KernelFn pick_vec(int vec, int rep)
{
    switch (vec) {
    case 1: return pick_rep<V, S, LPR, 1>(rep);
    case 2: return pick_rep<V, S, LPR, 2>(rep);
    case 4: return pick_rep<V, S, LPR, 4>(rep);
    }
    return nullptr;
}
template <int V, bool S> KernelFn pick_lpr(int lpr, int vec, int rep)
{
    switch (lpr) {
    case 4: return pick_vec<V, S, 4>(vec, rep);
    case 8: return pick_vec<V, S, 8>(vec, rep);
    case 16: return pick_vec<V, S, 16>(vec, rep);
    case 32: return pick_vec<V, S, 32>(vec, rep);
    case 64: return pick_vec<V, S, 64>(vec, rep);
    }
    return nullptr;
}
KernelFn pick(int V, int S, int lpr, int vec, int rep)
{
    if (V == 1) return S ? pick_lpr<1, true>(lpr, vec, rep) : pick_lpr<1, false>(lpr, vec, rep);
    if (V == 2) return S ? pick_lpr<2, true>(lpr, vec, rep) : pick_lpr<2, false>(lpr, vec, rep);
    return nullptr;
}

// batched instances exist where the accumulators stay within 32 registers
template <int V, int LPR, int VEC, int REP> KernelFn pickb_ipg(int ipg)
{
    if constexpr (2 < LPR && V * VEC * REP * 2 <= 32)
        if (ipg == 2) return &spmm_batched_kernel<V, LPR, VEC, REP, 2>;
    if constexpr (4 < LPR && V * VEC * REP * 4 <= 32)
        if (ipg == 4) return &spmm_batched_kernel<V, LPR, VEC, REP, 4>;
    return nullptr;
}
template <int V, int LPR, int VEC> KernelFn pickb_rep(int rep, int ipg)
{
    switch (rep) {
    case 1: return pickb_ipg<V, LPR, VEC, 1>(ipg);
    case 2: return pickb_ipg<V, LPR, VEC, 2>(ipg);
    case 4: return pickb_ipg<V, LPR, VEC, 4>(ipg);
    }
    return nullptr;
}
template <int V, int LPR> KernelFn pickb_vec(int vec, int rep, int ipg)
{
    switch (vec) {
    case 1: return pickb_rep<V, LPR, 1>(rep, ipg);
    case 2: return pickb_rep<V, LPR, 2>(rep, ipg);
    case 4: return pickb_rep<V, LPR, 4>(rep, ipg);
    }
    return nullptr;
}
template <int V> KernelFn pickb_lpr(int lpr, int vec, int rep, int ipg)
{
    switch (lpr) {
    case 4: return pickb_vec<V, 4>(vec, rep, ipg);
    case 8: return pickb_vec<V, 8>(vec, rep, ipg);
    case 16: return pickb_vec<V, 16>(vec, rep, ipg);
    case 32: return pickb_vec<V, 32>(vec, rep, ipg);
    case 64: return pickb_vec<V, 64>(vec, rep, ipg);
    }
    return nullptr;
}
KernelFn pick_any(int V, int S, int lpr, int vec, int rep, int ipg)
{
    if (ipg <= 1) return pick(V, S, lpr, vec, rep);
    if (S) return nullptr;
    if (V == 1) return pickb_lpr<1>(lpr, vec, rep, ipg);
    if (V == 2) return pickb_lpr<2>(lpr, vec, rep, ipg);
    return nullptr;
}

template <int V, int LPR, int VEC> KernelFn pickw_rep(int rep)
{
    switch (rep) {
    case 1: return &spmm_window_kernel<V, LPR, VEC, 1>;
    case 2: return &spmm_window_kernel<V, LPR, VEC, 2>;
    case 4: return &spmm_window_kernel<V, LPR, VEC, 4>;
    }
    return nullptr;
}
template <int V, int LPR> KernelFn pickw_vec(int vec, int rep)
{
    switch (vec) {
    case 1: return pickw_rep<V, LPR, 1>(rep);
    case 2: return pickw_rep<V, LPR, 2>(rep);
    case 4: return pickw_rep<V, LPR, 4>(rep);
    }
    return nullptr;
}
template <int V> KernelFn pickw_lpr(int lpr, int vec, int rep)
{
    switch (lpr) {
    case 4: return pickw_vec<V, 4>(vec, rep);
    case 8: return pickw_vec<V, 8>(vec, rep);
    case 16: return pickw_vec<V, 16>(vec, rep);
    case 32: return pickw_vec<V, 32>(vec, rep);
    case 64: return pickw_vec<V, 64>(vec, rep);
    }
    return nullptr;
}
KernelFn pick_window(int V, int lpr, int vec, int rep)
{
    if (V == 1) return pickw_lpr<1>(lpr, vec, rep);
    if (V == 2) return pickw_lpr<2>(lpr, vec, rep);
    return nullptr;
}

} // namespace

bool window_kernel_exists(int V, int lpr, int vec, int rep)
{
    return pick_window(V, lpr, vec, rep) != nullptr;
}

bool kernel_exists(int V, int S, int lpr, int vec, int rep, int ipg)
{
    return pick_any(V, S, lpr, vec, rep, ipg) != nullptr;
}

hipError_t launch_spmm(int V, int S, const LaunchShape &ls, const SpmmArgs &args, hipStream_t stream)
{
    if (ls.grid_x <= 0 || ls.grid_y <= 0) return hipSuccess; // nothing to do
    if (ls.window) {
        KernelFn fn = S ? nullptr : pick_window(V, ls.lpr, ls.vec, ls.rep);
        if (!fn) return hipErrorInvalidValue;
        // More than 64 KiB of dynamic LDS has to be allowed per kernel function: raised to
        // the 160 KiB of the CU once per function and device, not on every launch (the
        // call is host work and is not capturable in a HIP graph).
        {
            static std::mutex mu;
            static std::set<std::pair<int, const void *>> raised;
            int dev = -1;
            hipError_t e = hipGetDevice(&dev);
            if (e != hipSuccess) return e;
            std::lock_guard<std::mutex> lock(mu);
            const auto key = std::make_pair(dev, reinterpret_cast<const void *>(fn));
            if (!raised.count(key)) {
                e = hipFuncSetAttribute(reinterpret_cast<const void *>(fn),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
                if (e != hipSuccess) return e;
                raised.insert(key);
            }
        }
        hipLaunchKernelGGL(fn, dim3(ls.grid_x, ls.grid_y), dim3(64 * ls.waves), ls.lds_bytes, stream, args);
        return hipGetLastError();
    }
    KernelFn fn = pick_any(V, S, ls.lpr, ls.vec, ls.rep, ls.ipg);
    if (!fn) return hipErrorInvalidValue;
    hipLaunchKernelGGL(fn, dim3(ls.grid_x, ls.grid_y), dim3(64 * ls.waves), 0, stream, args);
    return hipGetLastError();
}

hipError_t launch_zero_panels(const int32_t *panels, int64_t n_panels, int V, float *C,
                              int32_t n_rows, int32_t K, hipStream_t stream)
{
    if (n_panels <= 0) return hipSuccess;
    const long total = n_panels * V * (long)K;
    long blocks = (total + 255) / 256;
    if (blocks > 256 * 64) blocks = 256 * 64;
    hipLaunchKernelGGL(zero_panels_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, panels,
                       (long)n_panels, V, C, n_rows, K);
    return hipGetLastError();
}

hipError_t static_scratch(void **ptr)
{
    constexpr int kMaxDevices = 64;
    static std::mutex mu;
    static void *addr[kMaxDevices] = {};
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(mu);
    if (!addr[dev]) {
        // every GPU holds its own copy of the array at its own address
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        addr[dev] = p;
    }
    *ptr = addr[dev];
    return hipSuccess;
}

hipError_t launch_reduce_split(const int32_t *split_panels, const int32_t *split_slot, int64_t n_split,
                               const int32_t *long_panels, int64_t n_long, int V, const float *ws, float *C,
                               int32_t n_rows, int32_t K, hipStream_t stream)
{
    if (n_split <= 0) return hipSuccess;
    // 16-byte accesses need rows that start on 16-byte boundaries (the workspace always does)
    const bool aligned = K % 4 == 0 && reinterpret_cast<uintptr_t>(C) % 16 == 0 &&
                         reinterpret_cast<uintptr_t>(ws) % 16 == 0;
    const int vec = aligned ? 4 : 1;
    const long total = n_split * V * (long)(K / vec);
    const long blocks = (total + 255) / 256;
    if (blocks > 0x7fffffffL || n_long * V > 0x7fffffffL) return hipErrorInvalidValue;
    const int skip_above = n_long > 0 ? kLongPanelSlots : 0x7fffffff;
    if (vec == 4)
        hipLaunchKernelGGL(reduce_split_kernel<4>, dim3((unsigned)blocks), dim3(256), 0, stream, split_panels,
                           split_slot, (long)n_split, V, ws, C, n_rows, K, skip_above);
    else
        hipLaunchKernelGGL(reduce_split_kernel<1>, dim3((unsigned)blocks), dim3(256), 0, stream, split_panels,
                           split_slot, (long)n_split, V, ws, C, n_rows, K, skip_above);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || n_long <= 0) return e;
    const int chunks = (K / vec + 15) / 16; // 16 vectors of C per workgroup
    if (chunks > 65535) return hipErrorInvalidValue;
    const dim3 grid((unsigned)(n_long * V), (unsigned)chunks);
    if (vec == 4)
        hipLaunchKernelGGL(reduce_long_kernel<4>, grid, dim3(16 * kLongReduceLanes), 0, stream, long_panels,
                           split_panels, split_slot, V, ws, C, n_rows, K);
    else
        hipLaunchKernelGGL(reduce_long_kernel<1>, grid, dim3(16 * kLongReduceLanes), 0, stream, long_panels,
                           split_panels, split_slot, V, ws, C, n_rows, K);
    return hipGetLastError();
}

} // namespace pcsr
