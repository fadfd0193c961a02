// The __global__ kernels of the softmax library (gfx950).
//
// rows path   rows_*: one workgroup owns a whole row and runs every pass of the
//             algorithm in one launch; the re-read of the row comes from L2.
// chunk path  chunk_*: a row is cut into chunks, one workgroup each.  A reducing
//             pass leaves one partial result per chunk.  The next pass folds up to
//             128 partials per row itself (lane i takes partials i, i + 64, then a wave
//             reduction); beyond that merge_* folds them into one value per row first.
#pragma once
#include "tp_device.h"

namespace tp {

// Cache hints.  A load whose data the next pass reads again stays cacheable; the
// last read of x and the stores of y carry the non-temporal hint so that they do
// not displace it.  On the chunk path the first read is non-temporal as well when
// the input is far larger than the caches (template parameter NT_FIRST).
constexpr bool kLoadKeep = false, kLoadStream = true;
constexpr bool kStoreKeep = false, kStoreStream = true;
constexpr uint32_t kXcds = 8;  // workgroup i is dispatched to XCD i % 8, each with its own L2

// ---- rows path: grid = rows ------------------------------------------------

template <class IO, int BLOCK, int U>
__global__ __launch_bounds__(BLOCK) void rows_2p(const typename IO::elem *x,
                                                 typename IO::elem *y, int64_t n)
{
    __shared__ float lds[2 * kMaxWaves];
    const Seg<IO> s = make_seg<IO>(x, y, n, blockIdx.x, 0, INT64_MAX / 2);
    PairSumOf<IO> acc;
    stream<IO, BLOCK, U, kLoadKeep, kStoreStream>(s, acc);
    float m_sum, n_sum;
    acc.finish(m_sum, n_sum);
    block_pair<BLOCK>(m_sum, n_sum, lds);
    PairOutOf<IO> out(1.0f / m_sum, n_sum);
    stream<IO, BLOCK, U, kLoadStream, kStoreStream>(s, out);
}

template <class IO, int BLOCK, int U>
__global__ __launch_bounds__(BLOCK) void rows_3p_recompute(const typename IO::elem *x,
                                                           typename IO::elem *y, int64_t n)
{
    __shared__ float lds[2 * kMaxWaves];
    const Seg<IO> s = make_seg<IO>(x, y, n, blockIdx.x, 0, INT64_MAX / 2);
    MaxOf mx;
    stream<IO, BLOCK, U, kLoadKeep, kStoreStream>(s, mx);
    const float mu = block_max<BLOCK>(mx.mx, lds);
    SumExp<IO::kIntExp> se{mu};
    stream<IO, BLOCK, U, kLoadKeep, kStoreStream>(s, se);
    const float sigma = block_sum<BLOCK>(se.s, lds);
    ExpScale<IO::kIntExp> es(mu, 1.0f / sigma);
    stream<IO, BLOCK, U, kLoadStream, kStoreStream>(s, es);
}

template <class IO, int BLOCK, int U>
__global__ __launch_bounds__(BLOCK) void rows_3p_reload(const typename IO::elem *x,
                                                        typename IO::elem *y, int64_t n)
{
    __shared__ float lds[2 * kMaxWaves];
    const Seg<IO> s = make_seg<IO>(x, y, n, blockIdx.x, 0, INT64_MAX / 2);
    MaxOf mx;
    stream<IO, BLOCK, U, kLoadKeep, kStoreStream>(s, mx);
    const float mu = block_max<BLOCK>(mx.mx, lds);
    ExpStoreSum<IO::kIntExp> ess{mu};
    stream<IO, BLOCK, U, kLoadStream, kStoreKeep>(s, ess);  // y is read back by the next pass
    const float sigma = block_sum<BLOCK>(ess.s, lds);
    // each thread re-reads exactly the vectors it stored itself, so program order suffices
    const Seg<IO> sy = make_seg<IO>(y, y, n, blockIdx.x, 0, INT64_MAX / 2);
    Scale sc{1.0f / sigma};
    stream<IO, BLOCK, U, kLoadStream, kStoreStream>(sy, sc);
}

// ---- short rows: LANES lanes per row, several rows per workgroup -----------------------
//
// Rows of at most a few hundred vectors cannot keep a whole workgroup busy.  Here a group of
// LANES lanes owns a row of its own: no LDS, no barrier, the lane-group reduction is the row
// reduction.  LANES = 64: one wave per row, four rows per workgroup.  LANES = 16, for rows of
// at most 64 vectors: one 16-lane DPP row per softmax row, sixteen rows per workgroup, so the
// per-row cost of reductions and addressing is shared by four rows per wave instruction.
// LANES = 4, for rows of at most 16 vectors: a quad per row, sixty-four rows per workgroup.

constexpr int kShortBlock = 256;

// NT_Y of the lane-group kernels: whether the stores of y carry the non-temporal hint.  The
// hint pays where y streams out in whole cache lines; rows whose length in bytes is not a
// multiple of the line share their first and last line with their neighbours, and without
// the hint the L2 caches merge what the neighbours (and the vector and the element-wise
// stores of one row) write to such a line before it leaves for memory (rows of 100 bf16
// elements: 0.118 -> 0.070 ms for 2^26 elements).

#define TP_SHORT_ROW_PROLOGUE                                                                \
    const int64_t row = (int64_t)blockIdx.x * (kShortBlock / LANES) + threadIdx.x / LANES;   \
    if (row >= rows)                                                                         \
        return;                                                                              \
    const uint32_t lane = threadIdx.x & (LANES - 1);                                         \
    const Seg<IO> s = make_seg<IO>(x, y, n, row, 0, INT64_MAX / 2);

template <class IO, int LANES, int U, bool NT_Y>
__global__ __launch_bounds__(kShortBlock) void waves_2p(const typename IO::elem *x,
                                                        typename IO::elem *y, int64_t n,
                                                        int64_t rows)
{
    TP_SHORT_ROW_PROLOGUE
    PairSumOf<IO> acc;
    stream<IO, LANES, U, kLoadKeep, kStoreStream>(s, acc, lane);
    float m_sum, n_sum;
    acc.finish(m_sum, n_sum);
    lanes_pair<LANES>(m_sum, n_sum);
    PairOutOf<IO> out(1.0f / m_sum, n_sum);
    stream<IO, LANES, U, kLoadStream, NT_Y>(s, out, lane);
}

template <class IO, int LANES, int U, bool NT_Y>
__global__ __launch_bounds__(kShortBlock) void waves_3p_recompute(
    const typename IO::elem *x, typename IO::elem *y, int64_t n, int64_t rows)
{
    TP_SHORT_ROW_PROLOGUE
    MaxOf mx;
    stream<IO, LANES, U, kLoadKeep, kStoreStream>(s, mx, lane);
    const float mu = lanes_max<LANES>(mx.mx);
    SumExp<IO::kIntExp> se{mu};
    stream<IO, LANES, U, kLoadKeep, kStoreStream>(s, se, lane);
    ExpScale<IO::kIntExp> es(mu, 1.0f / lanes_sum<LANES>(se.s));
    stream<IO, LANES, U, kLoadStream, NT_Y>(s, es, lane);
}

template <class IO, int LANES, int U, bool NT_Y>
__global__ __launch_bounds__(kShortBlock) void waves_3p_reload(
    const typename IO::elem *x, typename IO::elem *y, int64_t n, int64_t rows)
{
    TP_SHORT_ROW_PROLOGUE
    MaxOf mx;
    stream<IO, LANES, U, kLoadKeep, kStoreStream>(s, mx, lane);
    const float mu = lanes_max<LANES>(mx.mx);
    ExpStoreSum<IO::kIntExp> ess{mu};
    stream<IO, LANES, U, kLoadStream, kStoreKeep>(s, ess, lane);
    const Seg<IO> sy = make_seg<IO>(y, y, n, row, 0, INT64_MAX / 2);
    Scale sc{1.0f / lanes_sum<LANES>(ess.s)};
    stream<IO, LANES, U, kLoadStream, NT_Y>(sy, sc, lane);
}

// ---- on-chip rows: the row stays in registers between the passes -------------------
//
// For rows of at most BLOCK * U vectors, one workgroup per row.  x is read from memory once
// and y written once (2 N s bytes): the second read of Algorithm 3 is served by the register
// file.  A workgroup issues all its loads at once, computes, and stores; memory and arithmetic
// overlap across the two or more workgroups that share a compute unit and drift out of phase
// (the kernels are kept within 64 registers so that two 1024-thread workgroups fit).  Measured
// against the alternative, one persistent workgroup per compute unit that prefetches its next
// row while it computes: equal on 256 MiB of traffic, 10 % faster at 2 GiB (6.1 against
// 5.6 TB/s), because every compute unit of the persistent arrangement moves in lockstep.
// Reported as a variant of its own.

template <class IO, int U>
struct RowRegs {
    typename IO::vec v[U];
    float edge;
};

template <class IO>
__device__ __forceinline__ int64_t edge_index(const Seg<IO> &s)
{
    return (int)threadIdx.x < s.head ? (int64_t)threadIdx.x
                                     : s.tail0 + ((int64_t)threadIdx.x - s.head);
}

template <class IO>
__device__ __forceinline__ bool has_edge(const Seg<IO> &s)
{
    return (int64_t)threadIdx.x < s.head + (s.n - s.tail0);
}

// MODE says how much of the tile every row is known to fill:
//   kTileFull    every thread owns U real vectors and rows have no edge elements,
//   kTileMostly  the first U - 1 vector slots are full, the last one and the edges are not,
//   kTileAny     nothing is known.
// Slots known to be full are loaded and stored without a condition.
enum { kTileAny = 0, kTileMostly = 1, kTileFull = 2 };

template <int U, int MODE>
constexpr int lead_slots()
{
    return MODE == kTileFull ? U : MODE == kTileMostly ? U - 1 : 0;
}

template <class IO, int BLOCK, int U, int MODE>
__device__ __forceinline__ void load_row(const Seg<IO> &s, RowRegs<IO, U> &r)
{
    constexpr int LEAD = lead_slots<U, MODE>();
    const typename IO::vec *xb = s.xv + s.vb;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint32_t k = threadIdx.x + (uint32_t)(u * BLOCK);
        if (u < LEAD)
            r.v[u] = ld<kLoadStream>(xb + k);
        else
            r.v[u] = k < s.cnt ? ld<kLoadStream>(xb + k) : IO::zero();
    }
    r.edge = 0.f;
    if (MODE != kTileFull && has_edge(s))
        r.edge = IO::load1(s.xrow + edge_index(s));
}

// Feeds vectors [U0, U0 + GV) of the row to the policy: all at once if this thread owns
// all of them, else one by one.
template <class IO, int BLOCK, int U, int MODE, int U0, int GV, class P>
__device__ __forceinline__ void feed_group(const RowRegs<IO, U> &r, uint32_t cnt, P &p)
{
    constexpr int V = IO::V;
    constexpr int LEAD = lead_slots<U, MODE>();
    if (U0 + GV <= LEAD || threadIdx.x + (uint32_t)((U0 + GV - 1) * BLOCK) < cnt) {
        float f[GV * V];
#pragma unroll
        for (int g = 0; g < GV; ++g)
            IO::unpack(r.v[U0 + g], f + g * V);
        p.template group<GV * V>(f, nullptr);
    } else {
#pragma unroll
        for (int g = 0; g < GV; ++g) {
            if (U0 + g < LEAD || threadIdx.x + (uint32_t)((U0 + g) * BLOCK) < cnt) {
                float f[V];
                IO::unpack(r.v[U0 + g], f);
                p.template group<V>(f, nullptr);
            }
        }
    }
}

template <class IO, int BLOCK, int U, int MODE, int U0, class P>
__device__ __forceinline__ void feed_row(const RowRegs<IO, U> &r, uint32_t cnt, P &p)
{
    // 16 elements per group; 8 when the row buffers alone take half of the register file
    constexpr int GVMAX = (U * IO::V >= 32 ? 8 : 16) / IO::V;
    if constexpr (U0 < U) {
        constexpr int GV = (U - U0) < GVMAX ? (U - U0) : GVMAX;
        feed_group<IO, BLOCK, U, MODE, U0, GV>(r, cnt, p);
        feed_row<IO, BLOCK, U, MODE, U0 + GV>(r, cnt, p);
    }
}

// Pass 1 over the row's registers that also keeps what it computes: e[] receives every
// element's mantissa scaled to its group's exponent, g[u] that exponent for vector slot u.
template <class IO, int BLOCK, int U, int MODE, int U0, class P>
__device__ __forceinline__ void feed_row_keep(const RowRegs<IO, U> &r, uint32_t cnt, P &p, float *e,
                                              typename P::token *g)
{
    constexpr int V = IO::V;
    constexpr int LEAD = lead_slots<U, MODE>();
    constexpr int GVMAX = (U * V >= 32 ? 8 : 16) / V;
    if constexpr (U0 < U) {
        constexpr int GV = (U - U0) < GVMAX ? (U - U0) : GVMAX;
        if (U0 + GV <= LEAD || threadIdx.x + (uint32_t)((U0 + GV - 1) * BLOCK) < cnt) {
            float f[GV * V];
#pragma unroll
            for (int k = 0; k < GV; ++k)
                IO::unpack(r.v[U0 + k], f + k * V);
            p.template group<GV * V>(f, e + U0 * V);
#pragma unroll
            for (int k = 0; k < GV; ++k)
                g[U0 + k] = p.exponent();
        } else {
#pragma unroll
            for (int k = 0; k < GV; ++k) {
                if (U0 + k < LEAD || threadIdx.x + (uint32_t)((U0 + k) * BLOCK) < cnt) {
                    float f[V];
                    IO::unpack(r.v[U0 + k], f);
                    p.template group<V>(f, e + (U0 + k) * V);
                }
                g[U0 + k] = p.exponent();
            }
        }
        feed_row_keep<IO, BLOCK, U, MODE, U0 + GV>(r, cnt, p, e, g);
    }
}

// Algorithm 3 on one row held in registers.  Pass 1 leaves every element as its mantissa scaled
// to the exponent of its group, m_i 2^(n_i - n_g): the (m, n) pairs of Section 4 with one
// exponent shared by a group, kept in the registers that held x.  Pass 2 then needs no second
// ExtExp: y_i = (m_i 2^(n_i - n_g)) * (lambda 2^(n_g - n_sum)), one factor per group and one
// multiplication per element.  n_g <= n_sum, so the factor is at most lambda and nothing
// overflows; an element more than 126 binades below its group's largest is flushed to zero,
// and its result, below 2^-125, would be (all but) subnormal anyway.
template <class IO, int BLOCK, int U, int MODE>
__device__ __forceinline__ void onchip_row_2p(const Seg<IO> &s, const RowRegs<IO, U> &cur,
                                              float *lds)
{
    constexpr int V = IO::V;
    constexpr int LEAD = lead_slots<U, MODE>();
    using Acc = PairSumOf<IO>;
    const bool edge = MODE != kTileFull && has_edge(s);
    Acc acc;
    float e[U * V];
    typename Acc::token g[U];
    feed_row_keep<IO, BLOCK, U, MODE, 0>(cur, s.cnt, acc, e, g);
    float e_edge = 0.f;
    if (edge)
        acc.template group<1>(&cur.edge, &e_edge);
    const typename Acc::token g_edge = acc.exponent();
    float m_sum, n_sum;
    acc.finish(m_sum, n_sum);
    block_pair<BLOCK>(m_sum, n_sum, lds);
    const float lambda = 1.0f / m_sum;
    typename IO::vec *yb = s.yv + s.vb;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint32_t k = threadIdx.x + (uint32_t)(u * BLOCK);
        if (u < LEAD || k < s.cnt) {
            const float sc = Acc::factor(lambda, g[u], n_sum);
            float o[V];
#pragma unroll
            for (int i = 0; i < V; ++i)
                o[i] = e[u * V + i] * sc;
            st<kStoreStream>(yb + k, IO::pack(o));
        }
    }
    if (edge)
        IO::store1(s.yrow + edge_index(s), e_edge * Acc::factor(lambda, g_edge, n_sum));
}

// Algorithm 2 on one row held in registers: max, then Exp(x - mu) kept in registers where
// the algorithm keeps it in Y, their sum, and the rescaled values stored.  One exponential
// per element: in this regime the reloading Three-Pass algorithm is the cheapest, as the
// paper finds for data that fits in cache (Section 6.4).
template <class IO, int BLOCK, int U, int MODE>
__device__ __forceinline__ void onchip_row_3p(const Seg<IO> &s, const RowRegs<IO, U> &cur,
                                              float *lds)
{
    constexpr int V = IO::V;
    constexpr int LEAD = lead_slots<U, MODE>();
    const bool edge = MODE != kTileFull && has_edge(s);
    MaxOf mx;
    feed_row<IO, BLOCK, U, MODE, 0>(cur, s.cnt, mx);
    if (edge)
        mx.template group<1>(&cur.edge, nullptr);
    const float mu = block_max<BLOCK>(mx.mx, lds);
    float e[U * V];
    float part = 0.f;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint32_t k = threadIdx.x + (uint32_t)(u * BLOCK);
        if (u < LEAD || k < s.cnt) {
            float f[V], t[V];
            IO::unpack(cur.v[u], f);
#pragma unroll
            for (int i = 0; i < V; ++i)
                t[i] = e[u * V + i] = exp_nonpos_as<IO::kIntExp>(f[i] - mu);
            part += tree_sum<V>(t);
        } else {
#pragma unroll
            for (int i = 0; i < V; ++i)
                e[u * V + i] = 0.f;
        }
    }
    float e_edge = 0.f;
    if (edge) {
        e_edge = exp_nonpos_as<IO::kIntExp>(cur.edge - mu);
        part += e_edge;
    }
    const float lambda = 1.0f / block_sum<BLOCK>(part, lds);
    typename IO::vec *yb = s.yv + s.vb;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint32_t k = threadIdx.x + (uint32_t)(u * BLOCK);
        if (u < LEAD || k < s.cnt) {
            float o[V];
#pragma unroll
            for (int i = 0; i < V; ++i)
                o[i] = lambda * e[u * V + i];
            st<kStoreStream>(yb + k, IO::pack(o));
        }
    }
    if (edge)
        IO::store1(s.yrow + edge_index(s), lambda * e_edge);
}

enum { kOnchipTwoPass = 0, kOnchipThreePass = 1 };

template <class IO, int BLOCK, int U, int MODE, int ALGO>
__device__ __forceinline__ void onchip_row(const Seg<IO> &s, const RowRegs<IO, U> &cur, float *lds)
{
    if constexpr (ALGO == kOnchipTwoPass)
        onchip_row_2p<IO, BLOCK, U, MODE>(s, cur, lds);
    else
        onchip_row_3p<IO, BLOCK, U, MODE>(s, cur, lds);
}

template <class IO, int BLOCK, int U, int MODE, int ALGO>
__global__ __launch_bounds__(BLOCK) void rows_onchip(const typename IO::elem *x,
                                                     typename IO::elem *y, int64_t n)
{
    __shared__ float lds[2 * kMaxWaves];
    const Seg<IO> s = make_seg<IO>(x, y, n, blockIdx.x, 0, INT64_MAX / 2);
    RowRegs<IO, U> cur;
    load_row<IO, BLOCK, U, MODE>(s, cur);
    onchip_row<IO, BLOCK, U, MODE, ALGO>(s, cur, lds);
}

// The on-chip arrangement for short rows: LANES lanes (a wave, a row of 16 lanes or a quad)
// hold a softmax row of at most LANES * U vectors in their registers; reductions as in
// waves_*.  The elements before the first and after the last whole vector of a row (at most
// 2 (V - 1)) are spread over the lanes, E of them per lane.
template <class IO, int LANES, int U, int ALGO, bool NT_Y>
__global__ __launch_bounds__(kShortBlock) void waves_onchip(const typename IO::elem *x,
                                                            typename IO::elem *y, int64_t n,
                                                            int64_t rows)
{
    TP_SHORT_ROW_PROLOGUE
    constexpr int V = IO::V;
    constexpr int E = V == 1 ? 1 : (2 * (V - 1) + LANES - 1) / LANES;
    const typename IO::vec *xb = s.xv + s.vb;
    typename IO::vec *yb = s.yv + s.vb;
    typename IO::vec v[U];
    bool own[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        own[u] = lane + (uint32_t)(u * LANES) < s.cnt;
        v[u] = own[u] ? ld<kLoadStream>(xb + lane + u * LANES) : IO::zero();
    }
    const int nedge = s.edges ? s.head + (int)(s.n - s.tail0) : 0;
    bool edge[E];
    int64_t iedge[E];
    float x_edge[E], e_edge[E];
#pragma unroll
    for (int k = 0; k < E; ++k) {
        const int j = (int)lane + k * LANES;
        edge[k] = j < nedge;
        iedge[k] = j < s.head ? (int64_t)j : s.tail0 + (j - s.head);
        x_edge[k] = edge[k] ? IO::load1(s.xrow + iedge[k]) : 0.f;
        e_edge[k] = 0.f;
    }
    float e[U * V];
    if constexpr (ALGO == kOnchipTwoPass) {
        using Acc = PairSumOf<IO>;
        Acc acc;
        typename Acc::token g[U], g_edge[E];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (own[u]) {
                float f[V];
                IO::unpack(v[u], f);
                acc.template group<V>(f, e + u * V);
            }
            g[u] = acc.exponent();
        }
#pragma unroll
        for (int k = 0; k < E; ++k) {
            if (edge[k])
                acc.template group<1>(&x_edge[k], &e_edge[k]);
            g_edge[k] = acc.exponent();
        }
        float m_sum, n_sum;
        acc.finish(m_sum, n_sum);
        lanes_pair<LANES>(m_sum, n_sum);
        const float lambda = 1.0f / m_sum;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (own[u]) {
                const float sc = Acc::factor(lambda, g[u], n_sum);
                float o[V];
#pragma unroll
                for (int i = 0; i < V; ++i)
                    o[i] = e[u * V + i] * sc;
                st<NT_Y>(yb + lane + u * LANES, IO::pack(o));
            }
        }
#pragma unroll
        for (int k = 0; k < E; ++k)
            if (edge[k])
                IO::store1(s.yrow + iedge[k], e_edge[k] * Acc::factor(lambda, g_edge[k], n_sum));
    } else {
        float mx = -__builtin_inff();
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (own[u]) {
                float f[V];
                IO::unpack(v[u], f);
#pragma unroll
                for (int i = 0; i < V; ++i)
                    mx = fmaxf(mx, f[i]);
            }
        }
#pragma unroll
        for (int k = 0; k < E; ++k)
            if (edge[k])
                mx = fmaxf(mx, x_edge[k]);
        const float mu = lanes_max<LANES>(mx);
        float part = 0.f;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (own[u]) {
                float f[V], t[V];
                IO::unpack(v[u], f);
#pragma unroll
                for (int i = 0; i < V; ++i)
                    t[i] = e[u * V + i] = exp_nonpos_as<IO::kIntExp>(f[i] - mu);
                part += tree_sum<V>(t);
            }
        }
#pragma unroll
        for (int k = 0; k < E; ++k) {
            if (edge[k]) {
                e_edge[k] = exp_nonpos_as<IO::kIntExp>(x_edge[k] - mu);
                part += e_edge[k];
            }
        }
        const float lambda = 1.0f / lanes_sum<LANES>(part);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (own[u]) {
                float o[V];
#pragma unroll
                for (int i = 0; i < V; ++i)
                    o[i] = lambda * e[u * V + i];
                st<NT_Y>(yb + lane + u * LANES, IO::pack(o));
            }
        }
#pragma unroll
        for (int k = 0; k < E; ++k)
            if (edge[k])
                IO::store1(s.yrow + iedge[k], lambda * e_edge[k]);
    }
}

// ---- chunk path: grid = rows * chunks, rounded up to a multiple of kXcds ---------

struct ChunkArgs {
    int64_t n;
    int64_t chunk_vecs;
    int32_t chunks;
    uint32_t total;   // rows * chunks
    int32_t reverse;  // walk the chunks from the last to the first
};

// Successive passes walk memory in opposite directions, so a pass starts on the
// data the previous one touched last (still in L2 / the memory-side cache).  The
// reversal permutes groups of kXcds workgroups and keeps the position inside the
// group, so a chunk is handled by the same XCD - the same L2 - in both directions.
#define TP_CHUNK_PROLOGUE                                                  \
    uint32_t wg = blockIdx.x;                                              \
    if (a.reverse)                                                         \
        wg = (gridDim.x / kXcds - 1 - wg / kXcds) * kXcds + wg % kXcds;    \
    if (wg >= a.total)                                                     \
        return;                                                            \
    const int64_t row = wg / (uint32_t)a.chunks;                           \
    const int64_t chunk = wg % (uint32_t)a.chunks;

// Two-Pass pass 1: one (m, n) pair per chunk.
template <class IO, int BLOCK, int U, bool NT_FIRST>
__global__ __launch_bounds__(BLOCK) void chunk_2p_pass1(const typename IO::elem *x, ChunkArgs a,
                                                        float2 *partial)
{
    __shared__ float lds[2 * kMaxWaves];
    TP_CHUNK_PROLOGUE
    const Seg<IO> s = make_seg<IO>(x, nullptr, a.n, row, chunk, a.chunk_vecs);
    PairSumOf<IO> acc;
    stream<IO, BLOCK, U, NT_FIRST, kStoreStream>(s, acc);
    float m, n;
    acc.finish(m, n);
    block_pair<BLOCK>(m, n, lds);
    if (threadIdx.x == 0)
        partial[wg] = make_float2(m, n);
}

// Two-Pass pass 2.  pairs holds `npairs` (a few) pairs per row: the chunk partials of
// pass 1, or the single merged pair.
template <class IO, int BLOCK, int U>
__global__ __launch_bounds__(BLOCK) void chunk_2p_pass2(const typename IO::elem *x,
                                                        typename IO::elem *y, ChunkArgs a,
                                                        const float2 *pairs, int npairs)
{
    TP_CHUNK_PROLOGUE
    float m_sum, n_sum;
    wave_fold_pairs(pairs + row * npairs, npairs, m_sum, n_sum);
    const Seg<IO> s = make_seg<IO>(x, y, a.n, row, chunk, a.chunk_vecs);
    PairOutOf<IO> out(1.0f / m_sum, n_sum);
    stream<IO, BLOCK, U, kLoadStream, kStoreStream>(s, out);
}

template <class IO, int BLOCK, int U, bool NT_FIRST>
__global__ __launch_bounds__(BLOCK) void chunk_max(const typename IO::elem *x, ChunkArgs a,
                                                   float *pmax)
{
    __shared__ float lds[2 * kMaxWaves];
    TP_CHUNK_PROLOGUE
    const Seg<IO> s = make_seg<IO>(x, nullptr, a.n, row, chunk, a.chunk_vecs);
    MaxOf mx;
    stream<IO, BLOCK, U, NT_FIRST, kStoreStream>(s, mx);
    const float v = block_max<BLOCK>(mx.mx, lds);
    if (threadIdx.x == 0)
        pmax[wg] = v;
}

template <class IO, int BLOCK, int U, bool NT_FIRST>
__global__ __launch_bounds__(BLOCK) void chunk_sumexp(const typename IO::elem *x, ChunkArgs a,
                                                      const float *maxes, int nmax, float *psum)
{
    __shared__ float lds[2 * kMaxWaves];
    TP_CHUNK_PROLOGUE
    const Seg<IO> s = make_seg<IO>(x, nullptr, a.n, row, chunk, a.chunk_vecs);
    SumExp<IO::kIntExp> se{wave_fold_max(maxes + row * nmax, nmax)};
    stream<IO, BLOCK, U, NT_FIRST, kStoreStream>(s, se);
    const float v = block_sum<BLOCK>(se.s, lds);
    if (threadIdx.x == 0)
        psum[wg] = v;
}

template <class IO, int BLOCK, int U>
__global__ __launch_bounds__(BLOCK) void chunk_expscale(const typename IO::elem *x,
                                                        typename IO::elem *y, ChunkArgs a,
                                                        const float *maxes, int nmax,
                                                        const float *sums, int nsum)
{
    TP_CHUNK_PROLOGUE
    const float mu = wave_fold_max(maxes + row * nmax, nmax);
    const float sigma = wave_fold_sum(sums + row * nsum, nsum);
    const Seg<IO> s = make_seg<IO>(x, y, a.n, row, chunk, a.chunk_vecs);
    ExpScale<IO::kIntExp> es(mu, 1.0f / sigma);
    stream<IO, BLOCK, U, kLoadStream, kStoreStream>(s, es);
}

template <class IO, int BLOCK, int U>
__global__ __launch_bounds__(BLOCK) void chunk_expstore(const typename IO::elem *x,
                                                        typename IO::elem *y, ChunkArgs a,
                                                        const float *maxes, int nmax, float *psum)
{
    __shared__ float lds[2 * kMaxWaves];
    TP_CHUNK_PROLOGUE
    const Seg<IO> s = make_seg<IO>(x, y, a.n, row, chunk, a.chunk_vecs);
    ExpStoreSum<IO::kIntExp> ess{wave_fold_max(maxes + row * nmax, nmax)};
    stream<IO, BLOCK, U, kLoadStream, kStoreKeep>(s, ess);
    const float v = block_sum<BLOCK>(ess.s, lds);
    if (threadIdx.x == 0)
        psum[wg] = v;
}

// y = x / sigma (reload pass 3, x == y; `nsum` partial sums per row, a few);
// with sums == nullptr: y = lambda * x.
template <class IO, int BLOCK, int U>
__global__ __launch_bounds__(BLOCK) void chunk_scale(const typename IO::elem *x,
                                                     typename IO::elem *y, ChunkArgs a,
                                                     const float *sums, int nsum, float lambda)
{
    TP_CHUNK_PROLOGUE
    if (sums)
        lambda = 1.0f / wave_fold_sum(sums + row * nsum, nsum);
    const Seg<IO> s = make_seg<IO>(x, y, a.n, row, chunk, a.chunk_vecs);
    Scale sc{lambda};
    stream<IO, BLOCK, U, kLoadStream, kStoreStream>(s, sc);
}

// Calibration streams built from the same parts.
template <class IO, int BLOCK, int U>
__global__ __launch_bounds__(BLOCK) void chunk_read(const typename IO::elem *x, ChunkArgs a,
                                                    float *psum)
{
    __shared__ float lds[2 * kMaxWaves];
    TP_CHUNK_PROLOGUE
    const Seg<IO> s = make_seg<IO>(x, nullptr, a.n, row, chunk, a.chunk_vecs);
    SumOf so;
    stream<IO, BLOCK, U, kLoadStream, kStoreStream>(s, so);
    const float v = block_sum<BLOCK>(so.s, lds);
    if (threadIdx.x == 0)
        psum[wg] = v;
}

template <class IO, int BLOCK, int U>
__global__ __launch_bounds__(BLOCK) void chunk_copy(const typename IO::elem *x,
                                                    typename IO::elem *y, ChunkArgs a)
{
    TP_CHUNK_PROLOGUE
    const Seg<IO> s = make_seg<IO>(x, y, a.n, row, chunk, a.chunk_vecs);
    Copy cp;
    stream<IO, BLOCK, U, kLoadStream, kStoreStream>(s, cp);
}

// Write-only stream: y = value.  Same chunking and the same stores as the read-write passes.
template <int BLOCK, int U>
__global__ __launch_bounds__(BLOCK) void chunk_fill(float *y, ChunkArgs a, float value)
{
    TP_CHUNK_PROLOGUE
    const Seg<F32x4> s = make_seg<F32x4>(y, y, a.n, row, chunk, a.chunk_vecs);
    const f32x4 v = {value, value, value, value};
    f32x4 *yb = s.yv + s.vb;
    for (uint32_t k = threadIdx.x; k < s.cnt; k += BLOCK)
        st<kStoreStream>(yb + k, v);
    if (s.edges) {
        const int64_t nedge = s.head + (s.n - s.tail0);
        if ((int64_t)threadIdx.x < nedge)
            s.yrow[(int)threadIdx.x < s.head ? (int64_t)threadIdx.x
                                              : s.tail0 + ((int64_t)threadIdx.x - s.head)] = value;
    }
}

// ---- merges: grid = rows, one workgroup folds the `chunks` partials of its row ----

constexpr int kMergeBlock = 256;

__global__ __launch_bounds__(kMergeBlock) void merge_pairs_kernel(const float2 *partial, int chunks,
                                                                  float2 *out)
{
    __shared__ float lds[2 * kMaxWaves];
    const float2 *p = partial + (int64_t)blockIdx.x * chunks;
    float m = 0.f, n = kNIdent;
    for (int i = threadIdx.x; i < chunks; i += kMergeBlock) {
        const float2 q = p[i];
        const float nmax = fmaxf(n, q.y);
        m = scale_pow2(m, n - nmax) + scale_pow2(q.x, q.y - nmax);
        n = nmax;
    }
    block_pair<kMergeBlock>(m, n, lds);
    if (threadIdx.x == 0)
        out[blockIdx.x] = make_float2(m, n);
}

__global__ __launch_bounds__(kMergeBlock) void merge_max_kernel(const float *partial, int chunks,
                                                                float *out)
{
    __shared__ float lds[2 * kMaxWaves];
    const float *p = partial + (int64_t)blockIdx.x * chunks;
    float v = -__builtin_inff();
    for (int i = threadIdx.x; i < chunks; i += kMergeBlock)
        v = fmaxf(v, p[i]);
    v = block_max<kMergeBlock>(v, lds);
    if (threadIdx.x == 0)
        out[blockIdx.x] = v;
}

__global__ __launch_bounds__(kMergeBlock) void merge_sum_kernel(const float *partial, int chunks,
                                                                float *out)
{
    __shared__ float lds[2 * kMaxWaves];
    const float *p = partial + (int64_t)blockIdx.x * chunks;
    float v0 = 0.f, v1 = 0.f, v2 = 0.f, v3 = 0.f;  // four loads in flight per thread
    int i = threadIdx.x;
    for (; i + 3 * kMergeBlock < chunks; i += 4 * kMergeBlock) {
        v0 += p[i];
        v1 += p[i + kMergeBlock];
        v2 += p[i + 2 * kMergeBlock];
        v3 += p[i + 3 * kMergeBlock];
    }
    for (; i < chunks; i += kMergeBlock)
        v0 += p[i];
    const float v = block_sum<kMergeBlock>((v0 + v1) + (v2 + v3), lds);
    if (threadIdx.x == 0)
        out[blockIdx.x] = v;
}

// ---- ExtExp alone ------------------------------------------------------------

template <bool HW>
__global__ __launch_bounds__(256) void extexp_kernel(const float *x, float *m, float *e,
                                                     int64_t count)
{
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t step = (int64_t)gridDim.x * 256;
    for (; i < count; i += step) {
        if constexpr (HW)
            tp_extexp_hw(x[i], &m[i], &e[i]);
        else
            tp_extexp(x[i], &m[i], &e[i]);
    }
}

}  // namespace tp
