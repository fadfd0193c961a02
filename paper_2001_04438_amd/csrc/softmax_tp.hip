// Host side of the softmax library: launch planning, workspace, C ABI.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstring>
#include <map>
#include <mutex>
#include <type_traits>
#include <utility>

#include "../../include/softmax_tp.h"
#include "tp_kernels.h"

namespace tp {

// ===========================================================================
// planning
// ===========================================================================

struct Tuning {
    int64_t path = 0;
    int64_t block_rows = 0, unroll_rows = 0;
    int64_t block_reduce = 0, unroll_reduce = 0, target_reduce = 0;
    int64_t block_map = 0, unroll_map = 0, tiles_map = 0;
    int64_t block_mapsum = 0, unroll_mapsum = 0, tiles_mapsum = 0;
    int64_t direction = 0;
    int64_t nt_first = 0;
    int64_t fold_max = 0;
    int64_t nt_store = 0;
    int64_t scalar_io = 0;
};
// Written by softmax_tp_tune only; every reader takes a copy under the lock, so a sweep thread
// that retunes while another thread plans or launches is not a data race (the call then sees
// either the old or the new value of each key).
static Tuning g_tune_shared;
static std::mutex g_tune_mutex;

static Tuning tuning()
{
    std::lock_guard<std::mutex> lock(g_tune_mutex);
    return g_tune_shared;
}

constexpr int64_t kRowsPathMaxBytes = 256 * 1024;  // longest row one workgroup takes
constexpr int64_t kRowsPathMinRows = 32;           // fewer rows than this cannot fill the chip
constexpr int64_t kSmallRowBytes = 128 * 1024;     // ... unless the rows are this short (one launch wins)
// Partials per row a consuming pass folds itself.  Every wave of the launch reads them, so
// the limit is low: 128 still beat a merge launch (1.3 %), 512 lost 10 % on the 1 GiB vector.
constexpr int kFoldMax = 128;
constexpr int64_t kLatencyBoundBytes = (int64_t)4 << 20;  // below this a launch costs more than its traffic
// up to these sizes [fp32, 16-bit] a single row is cut into at most kFoldMax chunks for the
// read-only passes, handled by 512 threads each up to the second size and by 1024 beyond
constexpr int64_t kFewChunksBytes[2] = {(int64_t)64 << 20, (int64_t)32 << 20};
constexpr int64_t kFewChunksMidBytes[2] = {(int64_t)16 << 20, (int64_t)4 << 20};
constexpr int64_t kTargetReduce = 512;             // workgroups of a read-only pass (2 per CU)
constexpr int64_t kNtFirstBytes = (int64_t)512 << 20;  // inputs beyond this outlive every cache
// A launch may hold at most 2^32 - 1 threads in all (and 2^31 - 1 workgroups); grids are
// rounded up to a multiple of kXcds, hence the margin.
constexpr int64_t kThreadsMax = 0xFFFFFFFFll - 16 * 1024;
constexpr int64_t kGridMax = 0x7FFFFFF0;
constexpr int64_t kChunkVecsMax = (int64_t)1 << 26;  // a chunk is indexed with 32-bit offsets

static bool valid_block(int64_t b) { return b == 128 || b == 256 || b == 512 || b == 1024; }
static bool valid_unroll(int64_t u, int elem_bytes)
{
    return u == 1 || u == 2 || u == 4 || (u == 8 && elem_bytes == 4);
}

// Rows path.  Short rows get a group of lanes each, several rows per workgroup: a wave up to
// kWaveRowMaxVecs vectors (beyond 256 in a second round: up to these lengths that still beats
// a workgroup of 256 threads with its barriers), a row of 16 lanes (shape.block 16) up to
// kQuadRowMaxVecs, a quad of 4 lanes (shape.block 4) up to kTinyRowMaxVecs [fp32, 16-bit]; the
// on-chip entry points, which must hold the row in LANES * 4 vectors, switch at their own
// lengths.  From sweeps of every group size over rows of 1 to 1536 vectors.
constexpr int64_t kWaveRowMaxVecs[2][3] = {{352, 352, 272}, {512, 512, 304}};  // [format][algorithm]
constexpr int64_t kOnchipWaveRowMaxVecs = 256;  // a wave holds four vectors per lane
constexpr int64_t kQuadRowMaxVecs[2] = {64, 128};
constexpr int64_t kTinyRowMaxVecs[2] = {12, 16};
constexpr int64_t kOnchipQuadRowMaxVecs = 64;
constexpr int64_t kOnchipTinyRowMaxVecs = 8;
constexpr int kQuad = 16;
constexpr int kTiny = 4;
constexpr int kSolo = 1;
// Rows of at most this many elements [fp32, 16-bit] get a single lane each (shape.block 1), 256
// rows per workgroup: nothing to reduce across lanes and no lane idle.  With whole vectors if
// every row starts on a 16-byte boundary (fp32 rows of 4 or 8 elements, 16-bit rows of 8 or 16),
// element by element otherwise.  2^26 elements: fp32 rows of 4 0.280 -> 0.098 ms, of 5 0.341 ->
// 0.128, of 8 0.155 -> 0.108; bf16 rows of 4 0.226 -> 0.075, of 8 0.181 -> 0.063, of 10 0.228 ->
// 0.096, of 16 0.097 -> 0.065.  Longer rows lose: every lane then walks its own cache lines.
constexpr int64_t kSoloRowMaxElems[2] = {9, 16};

// Workgroup size and loads in flight on the rows path, by row length in 16-byte vectors.  From
// round-robin sweeps of every shape over rows of 1.5 K to 128 K elements: a lane should see two
// to eight vectors (a single round leaves nothing to overlap the loads with, many rounds of a
// small workgroup leave the row-wide reductions to too few waves), the variant that stores and
// re-reads its exponentials wants the larger workgroup one step earlier, and the 16-bit formats,
// with twice the arithmetic per vector, keep fewer loads in flight.
struct RowStep {
    int64_t below;  // applies to rows shorter than this many vectors
    int block, unroll;
};
constexpr int64_t kAnyLength = INT64_MAX;
static const RowStep kRowSteps[2][3][5] = {
    {   // fp32
        {{1024, 256, 2}, {3072, 512, 2}, {8192, 1024, 4}, {kAnyLength, 1024, 8}, {kAnyLength, 1024, 8}},
        {{1024, 256, 2}, {3072, 512, 2}, {6144, 1024, 4}, {kAnyLength, 1024, 8}, {kAnyLength, 1024, 8}},
        {{768, 256, 2}, {1536, 512, 2}, {3072, 1024, 2}, {4096, 1024, 4}, {kAnyLength, 1024, 8}},
    },
    {   // bf16, fp16
        {{1536, 256, 2}, {4096, 512, 2}, {12288, 1024, 2}, {kAnyLength, 1024, 4}, {kAnyLength, 1024, 4}},
        {{1536, 256, 2}, {2560, 512, 2}, {8192, 512, 4}, {kAnyLength, 1024, 4}, {kAnyLength, 1024, 4}},
        {{768, 256, 2}, {1536, 512, 2}, {6144, 1024, 2}, {kAnyLength, 1024, 4}, {kAnyLength, 1024, 4}},
    },
};

// algo: 0 Two-Pass, 1 Three-Pass with recomputation, 2 Three-Pass with reloading
static void rows_shape(const Tuning &g_tune, int64_t rows, int64_t n, int V, int elem_bytes,
                       int algo, softmax_tp_shape_t *s)
{
    const int64_t nvec = (n + V - 1) / V;
    s->chunk_vecs = 0;
    s->chunks = 1;
    if (n <= kSoloRowMaxElems[elem_bytes == 4 ? 0 : 1] && !g_tune.block_rows && !g_tune.unroll_rows &&
        (V == 1 || n % V == 0) && rows <= kThreadsMax) {
        s->block = kSolo;  // with vectors: one or two; element-wise: two at a time up to 3, else four
        s->unroll = V > 1 ? (int32_t)(n / V) : n <= 3 ? 2 : 4;
        return;
    }
    const bool group_forced = g_tune.block_rows == kSolo || g_tune.block_rows == kTiny ||
                              g_tune.block_rows == kQuad || g_tune.block_rows == kWave;
    if (group_forced || (nvec <= kWaveRowMaxVecs[elem_bytes == 4 ? 0 : 1][algo] && !g_tune.block_rows)) {
        // short rows: a group of 4, 16 or 64 lanes per row, several rows per workgroup
        const int wide = elem_bytes == 4 ? 0 : 1;
        // (the reloading variant, with a pass that writes y and one that reads it back, does not
        // gain from rounds of a small group: it moves to the wave at 64 vectors in every format)
        const int64_t quad_max = algo == 2 ? kQuadRowMaxVecs[0] : kQuadRowMaxVecs[wide];
        int lanes = nvec <= kTinyRowMaxVecs[wide] ? kTiny : nvec <= quad_max ? kQuad : kWave;
        if (group_forced) lanes = (int)g_tune.block_rows;
        // a launch holds fewer than 2^32 threads: very many rows make do with fewer lanes each
        while (lanes > kSolo && rows > kThreadsMax / lanes)
            lanes = lanes == kWave ? kQuad : lanes == kQuad ? kTiny : kSolo;
        int64_t rounds = (nvec + lanes - 1) / lanes;
        s->block = lanes;
        s->unroll = g_tune.unroll_rows ? (int32_t)g_tune.unroll_rows : rounds >= 4 ? 4 : (int32_t)rounds;
        return;
    }
    for (const RowStep &step : kRowSteps[elem_bytes == 4 ? 0 : 1][algo]) {
        if (nvec < step.below) {
            s->block = step.block;
            s->unroll = step.unroll;
            break;
        }
    }
    if (g_tune.block_rows) s->block = (int32_t)g_tune.block_rows;
    if (g_tune.unroll_rows) s->unroll = (int32_t)g_tune.unroll_rows;
}

static int chunk_shape(int64_t rows, int64_t nvec, int block, int unroll, int64_t chunk_vecs,
                       softmax_tp_shape_t *s)
{
    const int64_t tile = (int64_t)block * unroll;
    // the launch limits bound the number of chunks per row; longer chunks make up for it
    int64_t chunks_max = kThreadsMax / block / rows;
    if (chunks_max > kGridMax / rows) chunks_max = kGridMax / rows;
    if (chunks_max < 1)
        return TP_ERR_TOO_LARGE;
    const int64_t cv_min = (nvec + chunks_max - 1) / chunks_max;
    const int64_t cv_max = kChunkVecsMax / tile * tile;
    if (chunk_vecs < cv_min) chunk_vecs = cv_min;
    int64_t cv = (chunk_vecs + tile - 1) / tile * tile;
    if (cv < tile) cv = tile;
    if (cv > cv_max) cv = cv_max;
    if (cv < cv_min)
        return TP_ERR_TOO_LARGE;
    int64_t chunks = (nvec + cv - 1) / cv;
    if (chunks < 1) chunks = 1;
    s->block = block;
    s->unroll = unroll;
    s->chunk_vecs = cv;
    s->chunks = chunks;
    return TP_OK;
}

// force_path: 0 = choose (or take the tuning override), 1 = rows path, 2 = chunk path
static int make_plan(int64_t rows, int64_t n, int elem_bytes, bool congruent16, int force_path,
                     softmax_tp_plan_t *p)
{
    if (!p)
        return TP_ERR_NULL;
    if (rows < 0 || n < 0)
        return TP_ERR_NEGATIVE;
    if (elem_bytes != 4 && elem_bytes != 2)
        return TP_ERR_TUNING;
    std::memset(p, 0, sizeof *p);
    if (rows == 0 || n == 0)
        return TP_OK;
    const Tuning g_tune = tuning();
    if (n > INT64_MAX / elem_bytes / rows)
        return TP_ERR_TOO_LARGE;
    const int64_t row_bytes = n * elem_bytes;
    // (rows short enough for a lane of their own are read in vectors only if each of them can
    // start on a 16-byte boundary; whether the first one does is the caller's to say)
    const bool solo_ragged = n <= kSoloRowMaxElems[elem_bytes == 4 ? 0 : 1] && row_bytes % 16 != 0 &&
                             force_path != 2 && g_tune.path != 2;  // (a rows-path matter)
    const int V = congruent16 && !solo_ragged ? 16 / elem_bytes : 1;
    const int64_t nvec = (n + V - 1) / V;  // upper bound on the full vectors of a row
    p->vector_elems = V;

    bool rows_path = row_bytes <= kRowsPathMaxBytes &&
                     (rows >= kRowsPathMinRows || row_bytes <= kSmallRowBytes);
    const int64_t forced = force_path ? force_path : g_tune.path;
    if (forced == 1) rows_path = true;
    if (forced == 2) rows_path = false;

    if (rows_path) {
        if (rows > kGridMax || nvec > kChunkVecsMax)
            return TP_ERR_TOO_LARGE;
        p->path = 1;
        rows_shape(g_tune, rows, n, V, elem_bytes, 0, &p->rows);
        rows_shape(g_tune, rows, n, V, elem_bytes, 1, &p->rows_recompute);
        rows_shape(g_tune, rows, n, V, elem_bytes, 2, &p->rows_reload);
        p->launches = 1;
        for (const softmax_tp_shape_t *sh : {&p->rows, &p->rows_recompute, &p->rows_reload}) {
            // block threads per row, whether that is a workgroup, a wave or a few lanes
            if (rows > kThreadsMax / sh->block)
                return TP_ERR_TOO_LARGE;
            const bool group = sh->block == kWave || sh->block == kQuad || sh->block == kTiny ||
                               sh->block == kSolo;
            if (!(group ? sh->unroll >= 1 && sh->unroll <= 4
                        : valid_block(sh->block) && valid_unroll(sh->unroll, elem_bytes)))
                return TP_ERR_TUNING;
        }
        return TP_OK;
    }

    p->path = 2;
    const int64_t fold_limit = g_tune.fold_max ? g_tune.fold_max : kFoldMax;
    // read-only passes: few, long chunks.  Two workgroups of four waves per CU, each lane with
    // four 16-byte loads in flight (8 MiB over the chip), stream fastest; more waves or deeper
    // queues only add contention at the memory channels.
    {
        // (16-bit elements: twice the waves, these passes being bound by arithmetic there)
        int block = elem_bytes == 2 ? 512 : 256;
        const int unroll = g_tune.unroll_reduce ? (int)g_tune.unroll_reduce : 4;
        const int64_t target = g_tune.target_reduce ? g_tune.target_reduce : kTargetReduce;
        int64_t per_row = (target + rows - 1) / rows;
        if (per_row < 1) per_row = 1;
        // Up to a few dozen MiB a launch costs a good part of what its traffic does: stay within
        // what the next pass folds by itself, which saves the merge launch, and make up for the
        // fewer workgroups with larger ones (one to three rows only: more rows have at most
        // fold_limit chunks each anyway).
        const int64_t bytes = rows * row_bytes;
        if (per_row > fold_limit && !g_tune.target_reduce && bytes <= kFewChunksBytes[elem_bytes == 2]) {
            per_row = fold_limit;
            if (bytes > kLatencyBoundBytes)
                block = bytes <= kFewChunksMidBytes[elem_bytes == 2] ? 512 : 1024;
        }
        if (g_tune.block_reduce) block = (int)g_tune.block_reduce;
        int rc = chunk_shape(rows, nvec, block, unroll, (nvec + per_row - 1) / per_row, &p->reduce);
        if (rc != TP_OK) return rc;
    }
    // read-write passes: many short-lived workgroups, so that hardly any load has to queue
    // behind the stores of an earlier round of the same wave.  Arrays beyond the caches stream
    // fastest with one 16-byte access per lane at a time (two rounds of a 128-thread
    // workgroup); shorter ones, where the ramp and the tail of the launch weigh more, with one
    // round of 256 threads x 2.
    {
        const bool big = rows * row_bytes >= kNtFirstBytes;
        const int block = g_tune.block_map ? (int)g_tune.block_map : (big ? 128 : 256);
        const int unroll = g_tune.unroll_map ? (int)g_tune.unroll_map : (big ? 1 : 2);
        const int64_t tiles = g_tune.tiles_map ? g_tune.tiles_map : (big ? 2 : 1);
        int rc = chunk_shape(rows, nvec, block, unroll, tiles * block * unroll, &p->map);
        if (rc != TP_OK) return rc;
    }
    // the read-write pass that also leaves a partial sum per workgroup: fewer, larger ones
    {
        const int block = g_tune.block_mapsum ? (int)g_tune.block_mapsum : 1024;
        const int unroll = g_tune.unroll_mapsum ? (int)g_tune.unroll_mapsum : 4;
        const int64_t tiles = g_tune.tiles_mapsum ? g_tune.tiles_mapsum : 2;
        int rc = chunk_shape(rows, nvec, block, unroll, tiles * block * unroll, &p->mapsum);
        if (rc != TP_OK) return rc;
    }
    for (const softmax_tp_shape_t *s : {&p->reduce, &p->map, &p->mapsum})
        if (!valid_block(s->block) || !valid_unroll(s->unroll, elem_bytes))
            return TP_ERR_TUNING;
    p->nt_first_load = g_tune.nt_first ? (g_tune.nt_first == 2)
                                       : (rows * row_bytes >= kNtFirstBytes);
    // up to kFoldMax partials per row are folded by the consuming pass itself
    p->merge_kernel = p->reduce.chunks > fold_limit ? 1 : 0;
    p->launches = 2 + p->merge_kernel;
    const int64_t most = p->reduce.chunks > p->mapsum.chunks ? p->reduce.chunks : p->mapsum.chunks;
    p->workspace_bytes = (2 * rows * most + 2 * rows) * (int64_t)sizeof(float);
    return TP_OK;
}

// ===========================================================================
// workspace: one buffer per (device, stream)
// ===========================================================================

struct Workspace {
    void *ptr = nullptr;
    size_t bytes = 0;
};
static std::mutex g_ws_mutex;
static std::map<std::pair<int, void *>, Workspace> g_ws;

static int workspace(hipStream_t st, size_t bytes, float **out)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess)
        return (int)e;
    std::lock_guard<std::mutex> lock(g_ws_mutex);
    Workspace &w = g_ws[std::make_pair(dev, (void *)st)];
    if (w.bytes < bytes) {
        if (w.ptr) {
            e = hipFree(w.ptr);  // waits for work that may still use the old buffer
            w.ptr = nullptr;
            w.bytes = 0;
            if (e != hipSuccess)
                return (int)e;
        }
        const size_t want = bytes < (size_t)65536 ? (size_t)65536 : bytes;
        e = hipMalloc(&w.ptr, want);
        if (e != hipSuccess) {
            w.ptr = nullptr;
            return (int)e;
        }
        w.bytes = want;
    }
    *out = (float *)w.ptr;
    return TP_OK;
}

// ===========================================================================
// launching
// ===========================================================================

// Launches through hipLaunchKernel and reports that call's own return value.  The thread's
// "last error" is neither consulted nor cleared: it may hold the result of an earlier call of
// the caller's (an event query that was not ready, a failed allocation), which says nothing
// about this launch and is the caller's to read.
template <class... KArgs>
static int launch(void (*kernel)(KArgs...), dim3 grid, dim3 block, hipStream_t st,
                  typename std::common_type<KArgs>::type... args)
{
    void *ptrs[] = {(void *)&args...};
    const hipError_t e = hipLaunchKernel((const void *)kernel, grid, block, ptrs, 0, st);
    return e == hipSuccess ? TP_OK : (int)e;
}

static ChunkArgs chunk_args(int64_t n, const softmax_tp_shape_t &s, int64_t rows, bool reverse)
{
    return ChunkArgs{n, s.chunk_vecs, (int32_t)s.chunks, (uint32_t)(rows * s.chunks),
                     reverse ? 1 : 0};
}

static dim3 chunk_grid(int64_t rows, const softmax_tp_shape_t &s)
{
    const int64_t total = rows * s.chunks;
    return dim3((uint32_t)((total + kXcds - 1) / kXcds * kXcds));
}

static int fold_max()
{
    const int64_t f = tuning().fold_max;
    return f ? (int)f : kFoldMax;
}

// Every pass walks memory forwards.  With the tuning key "direction" = 2, pass k of a call
// (0-based) runs backwards when k is odd, so that it starts on what the previous pass touched
// last; on this part that measured the same or slightly worse, the caches being small next to
// the arrays that take this path.
static bool pass_reversed(int k) { return tuning().direction == 2 && (k & 1) != 0; }

template <int N>
using ic = std::integral_constant<int, N>;

// Calls f(ic<BLOCK>, ic<U>) for the shape's block and unroll.  16-bit vectors unpack to 8
// floats each, so 8 of them in flight would not fit the registers of a 1024-thread
// workgroup: the 16-bit formats stop at 4.
template <class IO, class F>
static int with_shape(const softmax_tp_shape_t &s, F &&f)
{
#define TP_CASE(B, UU)                                                       \
    case B * 16 + UU:                                                        \
        if constexpr (sizeof(typename IO::elem) == 2 && UU == 8) {           \
            return TP_ERR_TUNING;                                            \
        } else {                                                             \
            return f(ic<B>{}, ic<UU>{});                                     \
        }
    switch (s.block * 16 + s.unroll) {
        TP_CASE(128, 1)
        TP_CASE(256, 2) TP_CASE(256, 4) TP_CASE(256, 8)
        TP_CASE(512, 2) TP_CASE(512, 4) TP_CASE(512, 8)
        TP_CASE(1024, 2) TP_CASE(1024, 4) TP_CASE(1024, 8)
    default:
        return TP_ERR_TUNING;
    }
#undef TP_CASE
}

#define TP_B decltype(B)::value
#define TP_U decltype(U)::value

enum Algo { kTwoPass, kRecompute, kReload };

// Whether a lane-group launch stores y with the non-temporal hint.  Rows that take a wave each
// always do.  Rows on 4 or 16 lanes do not if neighbouring rows share cache lines in an
// irregular way (the row is neither a multiple nor a divisor of the 128-byte line) and are
// short enough for those shared lines to weigh (under 1 KiB; for the on-chip kernels, which
// write each row in one go, under one line): plain stores let the L2 caches merge the pieces
// of a line before it leaves for memory.  Steady-state sweep, 2^26 elements: rows of 100 bf16
// elements 0.121 -> 0.070 ms, of 50 bf16 0.126 -> 0.090, of 25 fp32 0.258 -> 0.154; rows of
// whole lines, and rows of 1000 bf16 elements and more, are 3 to 19 % faster with the hint.
static bool group_store_hint(int lanes, int64_t n, int elem_bytes, bool onchip)
{
    const int64_t forced = tuning().nt_store;
    if (lanes == kWave || forced == 2)
        return true;
    if (forced == 1)
        return false;
    const int64_t bytes = n * elem_bytes;
    const bool regular = bytes % 128 == 0 || 128 % bytes == 0;
    return regular || bytes >= (onchip ? 128 : 1024);
}

template <class IO>
static int run_rows(Algo algo, const softmax_tp_plan_t &plan, const typename IO::elem *x,
                    typename IO::elem *y, int64_t rows, int64_t n, hipStream_t st)
{
    const softmax_tp_shape_t &shape = algo == kTwoPass     ? plan.rows
                                      : algo == kRecompute ? plan.rows_recompute
                                                           : plan.rows_reload;
    if (shape.block == kWave || shape.block == kQuad || shape.block == kTiny || shape.block == kSolo) {
        // short rows: a lane group per row
        const int64_t per_group = kShortBlock / shape.block;
        const dim3 wgrid((uint32_t)((rows + per_group - 1) / per_group));
        const dim3 wblock(kShortBlock);
        const bool y_nt = group_store_hint(shape.block, n, (int)sizeof(typename IO::elem), false);
        auto go_nt = [&](auto LANES, auto U, auto NT) {
            constexpr int L = decltype(LANES)::value;
            constexpr bool N = decltype(NT)::value != 0;
            if (algo == kTwoPass)
                return launch(waves_2p<IO, L, TP_U, N>, wgrid, wblock, st, x, y, n, rows);
            if (algo == kRecompute)
                return launch(waves_3p_recompute<IO, L, TP_U, N>, wgrid, wblock, st, x, y, n, rows);
            return launch(waves_3p_reload<IO, L, TP_U, N>, wgrid, wblock, st, x, y, n, rows);
        };
        auto go = [&](auto LANES, auto U) {
            if constexpr (decltype(LANES)::value == kWave)
                return go_nt(LANES, U, ic<1>{});
            else
                return y_nt ? go_nt(LANES, U, ic<1>{}) : go_nt(LANES, U, ic<0>{});
        };
        switch (shape.block * 8 + shape.unroll) {
#define TP_GROUP(L, UU) case L * 8 + UU: return go(ic<L>{}, ic<UU>{});
            TP_GROUP(kSolo, 1) TP_GROUP(kSolo, 2) TP_GROUP(kSolo, 3) TP_GROUP(kSolo, 4)
            TP_GROUP(kTiny, 1) TP_GROUP(kTiny, 2) TP_GROUP(kTiny, 3) TP_GROUP(kTiny, 4)
            TP_GROUP(kQuad, 1) TP_GROUP(kQuad, 2) TP_GROUP(kQuad, 3) TP_GROUP(kQuad, 4)
            TP_GROUP(kWave, 1) TP_GROUP(kWave, 2) TP_GROUP(kWave, 3) TP_GROUP(kWave, 4)
#undef TP_GROUP
        default:
            return TP_ERR_TUNING;
        }
    }
    const dim3 grid((uint32_t)rows);
    return with_shape<IO>(shape, [&](auto B, auto U) {
        if (algo == kTwoPass)
            return launch(rows_2p<IO, TP_B, TP_U>, grid, dim3(TP_B), st, x, y, n);
        if (algo == kRecompute)
            return launch(rows_3p_recompute<IO, TP_B, TP_U>, grid, dim3(TP_B), st, x, y, n);
        return launch(rows_3p_reload<IO, TP_B, TP_U>, grid, dim3(TP_B), st, x, y, n);
    });
}

// Two-Pass pass 1 on the chunk path: partial pairs; if `merged` is given, one merged pair
// per row as well.
template <class IO>
static int run_2p_pass1(const softmax_tp_plan_t &plan, const typename IO::elem *x, int64_t rows,
                        int64_t n, hipStream_t st, float2 *partial, float2 *merged)
{
    const ChunkArgs a = chunk_args(n, plan.reduce, rows, pass_reversed(0));
    const dim3 grid = chunk_grid(rows, plan.reduce);
    const bool nt = plan.nt_first_load != 0;
    int rc = with_shape<IO>(plan.reduce, [&](auto B, auto U) {
        if (nt)
            return launch(chunk_2p_pass1<IO, TP_B, TP_U, true>, grid, dim3(TP_B), st, x, a, partial);
        return launch(chunk_2p_pass1<IO, TP_B, TP_U, false>, grid, dim3(TP_B), st, x, a, partial);
    });
    if (rc != TP_OK || !merged)
        return rc;
    return launch(merge_pairs_kernel, dim3((uint32_t)rows), dim3(kMergeBlock), st, partial,
                  (int)plan.reduce.chunks, merged);
}

template <class IO>
static int run_2p_pass2(const softmax_tp_plan_t &plan, const typename IO::elem *x,
                        typename IO::elem *y, int64_t rows, int64_t n, hipStream_t st,
                        const float2 *pairs, int npairs)
{
    const ChunkArgs a = chunk_args(n, plan.map, rows, pass_reversed(1));
    const dim3 grid = chunk_grid(rows, plan.map);
    return with_shape<IO>(plan.map, [&](auto B, auto U) {
        return launch(chunk_2p_pass2<IO, TP_B, TP_U>, grid, dim3(TP_B), st, x, y, a, pairs, npairs);
    });
}

// Bytes of partial results the Two-Pass chunk path needs: one pair per chunk and, when a
// merge launch is planned, one more per row.
static int64_t two_pass_scratch_bytes(const softmax_tp_plan_t &plan, int64_t rows)
{
    return (rows * plan.reduce.chunks + (plan.merge_kernel ? rows : 0)) * (int64_t)sizeof(float2);
}

// The Two-Pass chunk path on a buffer for its partial results (two_pass_scratch_bytes of it).
template <class IO>
static int run_chunks_2p_on(float *ws, const softmax_tp_plan_t &plan, const typename IO::elem *x,
                            typename IO::elem *y, int64_t rows, int64_t n, hipStream_t st)
{
    float2 *partial = (float2 *)ws;
    float2 *merged = plan.merge_kernel ? partial + rows * plan.reduce.chunks : nullptr;
    const int rc = run_2p_pass1<IO>(plan, x, rows, n, st, partial, merged);
    if (rc != TP_OK)
        return rc;
    return merged ? run_2p_pass2<IO>(plan, x, y, rows, n, st, merged, 1)
                  : run_2p_pass2<IO>(plan, x, y, rows, n, st, partial, (int)plan.reduce.chunks);
}

template <class IO>
static int run_chunks_2p(const softmax_tp_plan_t &plan, const typename IO::elem *x,
                         typename IO::elem *y, int64_t rows, int64_t n, hipStream_t st)
{
    float *ws = nullptr;
    const int rc = workspace(st, (size_t)plan.workspace_bytes, &ws);
    if (rc != TP_OK)
        return rc;
    return run_chunks_2p_on<IO>(ws, plan, x, y, rows, n, st);
}

template <class IO>
static int run_chunks_3p(Algo algo, const softmax_tp_plan_t &plan, const typename IO::elem *x,
                         typename IO::elem *y, int64_t rows, int64_t n, hipStream_t st)
{
    float *ws = nullptr;
    int rc = workspace(st, (size_t)plan.workspace_bytes, &ws);
    if (rc != TP_OK)
        return rc;
    const int64_t most =
        plan.reduce.chunks > plan.mapsum.chunks ? plan.reduce.chunks : plan.mapsum.chunks;
    float *pmax = ws, *psum = ws + rows * most;
    float *rowmax = ws + 2 * rows * most, *rowsum = rowmax + rows;
    const bool nt = plan.nt_first_load != 0;
    const dim3 rgrid = chunk_grid(rows, plan.reduce);
    const dim3 merge_grid((uint32_t)rows), merge_block(kMergeBlock);

    // pass 1: mu
    const float *maxes = pmax;
    int nmax = (int)plan.reduce.chunks;
    {
        const ChunkArgs a = chunk_args(n, plan.reduce, rows, pass_reversed(0));
        rc = with_shape<IO>(plan.reduce, [&](auto B, auto U) {
            if (nt)
                return launch(chunk_max<IO, TP_B, TP_U, true>, rgrid, dim3(TP_B), st, x, a, pmax);
            return launch(chunk_max<IO, TP_B, TP_U, false>, rgrid, dim3(TP_B), st, x, a, pmax);
        });
        if (rc != TP_OK)
            return rc;
        if (nmax > fold_max()) {
            rc = launch(merge_max_kernel, merge_grid, merge_block, st, (const float *)pmax, nmax,
                        rowmax);
            if (rc != TP_OK)
                return rc;
            maxes = rowmax;
            nmax = 1;
        }
    }
    // pass 2: sigma (and, for the reload variant, y = Exp(x - mu))
    const float *sums = psum;
    int nsum = 0;
    if (algo == kRecompute) {
        const ChunkArgs a = chunk_args(n, plan.reduce, rows, pass_reversed(1));
        nsum = (int)plan.reduce.chunks;
        rc = with_shape<IO>(plan.reduce, [&](auto B, auto U) {
            if (nt)
                return launch(chunk_sumexp<IO, TP_B, TP_U, true>, rgrid, dim3(TP_B), st, x, a, maxes,
                              nmax, psum);
            return launch(chunk_sumexp<IO, TP_B, TP_U, false>, rgrid, dim3(TP_B), st, x, a, maxes,
                          nmax, psum);
        });
    } else {
        const ChunkArgs a = chunk_args(n, plan.mapsum, rows, pass_reversed(1));
        const dim3 grid = chunk_grid(rows, plan.mapsum);
        nsum = (int)plan.mapsum.chunks;
        rc = with_shape<IO>(plan.mapsum, [&](auto B, auto U) {
            return launch(chunk_expstore<IO, TP_B, TP_U>, grid, dim3(TP_B), st, x, y, a, maxes, nmax,
                          psum);
        });
    }
    if (rc != TP_OK)
        return rc;
    if (nsum > fold_max()) {
        rc = launch(merge_sum_kernel, merge_grid, merge_block, st, (const float *)psum, nsum, rowsum);
        if (rc != TP_OK)
            return rc;
        sums = rowsum;
        nsum = 1;
    }
    // pass 3: y
    const ChunkArgs a = chunk_args(n, plan.map, rows, pass_reversed(2));
    const dim3 grid = chunk_grid(rows, plan.map);
    if (algo == kRecompute)
        return with_shape<IO>(plan.map, [&](auto B, auto U) {
            return launch(chunk_expscale<IO, TP_B, TP_U>, grid, dim3(TP_B), st, x, y, a, maxes, nmax,
                          sums, nsum);
        });
    const typename IO::elem *yc = y;
    return with_shape<IO>(plan.map, [&](auto B, auto U) {
        return launch(chunk_scale<IO, TP_B, TP_U>, grid, dim3(TP_B), st, yc, y, a, sums, nsum, 0.f);
    });
}

// ---- argument checks ---------------------------------------------------------

static int check_args(const void *x, const void *y, int64_t rows, int64_t n, int elem_bytes)
{
    if (rows < 0 || n < 0)
        return TP_ERR_NEGATIVE;
    if (rows == 0 || n == 0)
        return TP_OK;
    if (!x || !y)
        return TP_ERR_NULL;
    if (n > INT64_MAX / elem_bytes / rows)
        return TP_ERR_TOO_LARGE;
    if (((uintptr_t)x % elem_bytes) || ((uintptr_t)y % elem_bytes))
        return TP_ERR_ALIGN;
    return TP_OK;
}

static bool congruent16(const void *x, const void *y)
{
    return (((uintptr_t)x ^ (uintptr_t)y) & 15u) == 0;
}

// ---- on-chip rows ------------------------------------------------------------------

struct OnchipShape {
    int block, unroll, mode;
};

// A row must fit block * unroll vectors.  lo / hi bound the number of whole vectors a row
// can have (it depends on where the row starts relative to a 16-byte boundary).  Candidates
// are tiles the rows fill exactly (kTileFull), tiles whose first unroll - 1 slots every row
// fills (kTileMostly) and tiles that check every slot (kTileAny); the one with the least
// padding wins (a row of 513 vectors takes 256 x 3, not 1024 x 1 with half the threads idle),
// then the unroll closest to 4, then the cheaper kind, then the smaller block.
static bool onchip_shape(int64_t lo, int64_t hi, bool exact, int unroll_max, OnchipShape *out)
{
    static const int blocks[] = {256, 512, 1024};
    bool found = false;
    int64_t best_key = 0;
    for (int b : blocks) {
        const int64_t u = hi <= b ? 1 : (hi + b - 1) / b;
        if (u > unroll_max)
            continue;
        int mode;
        if (exact && hi == b * u && (u == 1 || u == 2 || u == 4 || u == 8))
            mode = kTileFull;
        else if ((u - 1) * b <= lo)
            mode = kTileMostly;
        else
            mode = kTileAny;
        const int64_t pad = b * u - hi;
        const int64_t key = (pad << 8) + ((u > 4 ? u - 4 : 4 - u) << 2) +
                            (mode == kTileFull ? 0 : mode == kTileMostly ? 1 : 2);
        if (!found || key < best_key) {
            found = true;
            best_key = key;
            *out = OnchipShape{b, (int)u, mode};
        }
    }
    return found;
}

template <class IO, int B, int U, int MODE>
static int launch_onchip(int algo, const typename IO::elem *x, typename IO::elem *y, int64_t rows,
                         int64_t n, hipStream_t st)
{
    auto kernel = algo == kOnchipTwoPass ? rows_onchip<IO, B, U, MODE, kOnchipTwoPass>
                                         : rows_onchip<IO, B, U, MODE, kOnchipThreePass>;
    return launch(kernel, dim3((uint32_t)rows), dim3(B), st, x, y, n);
}

template <class IO, int B, int U>
static int launch_onchip_mode(int mode, int algo, const typename IO::elem *x,
                              typename IO::elem *y, int64_t rows, int64_t n, hipStream_t st)
{
    if (mode == kTileFull) {
        if constexpr (U == 1 || U == 2 || U == 4 || U == 8)
            return launch_onchip<IO, B, U, kTileFull>(algo, x, y, rows, n, st);
        else
            return TP_ERR_TUNING;
    }
    if (mode == kTileMostly)
        return launch_onchip<IO, B, U, kTileMostly>(algo, x, y, rows, n, st);
    return launch_onchip<IO, B, U, kTileAny>(algo, x, y, rows, n, st);
}

template <class IO>
static int run_onchip(int algo, const typename IO::elem *x, typename IO::elem *y, int64_t rows,
                      int64_t n, void *stream)
{
    constexpr int es = (int)sizeof(typename IO::elem);
    constexpr int V = IO::V;
    constexpr int umax = es == 4 ? 8 : 4;
    int rc = check_args(x, y, rows, n, es);
    if (rc != TP_OK || rows == 0 || n == 0)
        return rc;
    if (!congruent16(x, y))
        return TP_ERR_ALIGN;
    const bool exact = ((uintptr_t)x % 16) == 0 && n % V == 0;
    const int64_t hi = (n + V - 1) / V;
    hipStream_t st = (hipStream_t)stream;
    if (hi <= kOnchipWaveRowMaxVecs) {  // short rows: a lane group per row, as on the rows path
        const Tuning t = tuning();
        int lanes = hi <= kOnchipTinyRowMaxVecs ? kTiny : hi <= kOnchipQuadRowMaxVecs ? kQuad : kWave;
        if (t.block_rows == kTiny || t.block_rows == kQuad || t.block_rows == kWave)
            lanes = (int)t.block_rows;  // for sweeps; the row still has to fit LANES * 4 vectors
        const int64_t u = (hi + lanes - 1) / lanes;
        if (u > 4)
            return TP_ERR_TUNING;
        if (rows > kThreadsMax / lanes)
            return TP_ERR_TOO_LARGE;
        const int64_t per_group = kShortBlock / lanes;
        const dim3 wgrid((uint32_t)((rows + per_group - 1) / per_group)), wblock(kShortBlock);
        const bool y_nt = group_store_hint(lanes, n, es, true);
        auto go_nt = [&](auto LANES, auto U, auto NT) {
            constexpr int L = decltype(LANES)::value;
            constexpr bool N = decltype(NT)::value != 0;
            if (algo == kOnchipTwoPass)
                return launch(waves_onchip<IO, L, TP_U, kOnchipTwoPass, N>, wgrid, wblock, st, x, y, n, rows);
            return launch(waves_onchip<IO, L, TP_U, kOnchipThreePass, N>, wgrid, wblock, st, x, y, n, rows);
        };
        auto go = [&](auto LANES, auto U) {
            if constexpr (decltype(LANES)::value == kWave)
                return go_nt(LANES, U, ic<1>{});
            else
                return y_nt ? go_nt(LANES, U, ic<1>{}) : go_nt(LANES, U, ic<0>{});
        };
        switch (lanes * 8 + (int)u) {
#define TP_GROUP(L, UU) case L * 8 + UU: return go(ic<L>{}, ic<UU>{});
            TP_GROUP(kTiny, 1) TP_GROUP(kTiny, 2) TP_GROUP(kTiny, 3) TP_GROUP(kTiny, 4)
            TP_GROUP(kQuad, 1) TP_GROUP(kQuad, 2) TP_GROUP(kQuad, 3) TP_GROUP(kQuad, 4)
            TP_GROUP(kWave, 1) TP_GROUP(kWave, 2) TP_GROUP(kWave, 3) TP_GROUP(kWave, 4)
#undef TP_GROUP
        default:
            return TP_ERR_TUNING;
        }
    }
    const int64_t lo = exact ? n / V : (n / V > 0 ? n / V - 1 : 0);
    OnchipShape sh;
    if (!onchip_shape(lo, hi, exact, umax, &sh) || rows > kGridMax || rows > kThreadsMax / 1024)
        return TP_ERR_TOO_LARGE;
#define TP_OC(B, UU)                                                              \
    case B * 16 + UU:                                                             \
        if constexpr (UU <= umax)                                                 \
            return launch_onchip_mode<IO, B, UU>(sh.mode, algo, x, y, rows, n, st); \
        else                                                                      \
            return TP_ERR_TUNING;
#define TP_OC_BLOCK(B) \
    TP_OC(B, 1) TP_OC(B, 2) TP_OC(B, 3) TP_OC(B, 4) TP_OC(B, 5) TP_OC(B, 6) TP_OC(B, 7) TP_OC(B, 8)
    switch (sh.block * 16 + sh.unroll) {
        TP_OC_BLOCK(256)
        TP_OC_BLOCK(512)
        TP_OC_BLOCK(1024)
    default:
        return TP_ERR_TUNING;
    }
#undef TP_OC_BLOCK
#undef TP_OC
}

// Whether a call reads and writes 16-byte vectors: x and y congruent modulo 16 bytes, and,
// for rows short enough to get a lane of their own, every row starting on a 16-byte boundary.
static bool vector_access(const void *x, const void *y, int64_t n, int elem_bytes)
{
    const bool solo = n <= kSoloRowMaxElems[elem_bytes == 4 ? 0 : 1];
    const bool rows_aligned = (uintptr_t)x % 16 == 0 && (n * elem_bytes) % 16 == 0;
    return congruent16(x, y) && tuning().scalar_io != 1 && (!solo || rows_aligned);
}

template <class IOV, class IOS>
static int softmax_any(Algo algo, const typename IOV::elem *x, typename IOV::elem *y,
                       int64_t rows, int64_t n, void *stream)
{
    constexpr int es = (int)sizeof(typename IOV::elem);
    int rc = check_args(x, y, rows, n, es);
    if (rc != TP_OK || rows == 0 || n == 0)
        return rc;
    const bool vec = vector_access(x, y, n, es);
    softmax_tp_plan_t plan;
    rc = make_plan(rows, n, es, vec, 0, &plan);
    if (rc != TP_OK)
        return rc;
    hipStream_t st = (hipStream_t)stream;
    if (plan.path == 1)
        return vec ? run_rows<IOV>(algo, plan, x, y, rows, n, st)
                   : run_rows<IOS>(algo, plan, x, y, rows, n, st);
    if (algo == kTwoPass)
        return vec ? run_chunks_2p<IOV>(plan, x, y, rows, n, st)
                   : run_chunks_2p<IOS>(plan, x, y, rows, n, st);
    return vec ? run_chunks_3p<IOV>(algo, plan, x, y, rows, n, st)
               : run_chunks_3p<IOS>(algo, plan, x, y, rows, n, st);
}

// The on-chip entry points.  Rows short enough for a lane of their own go through the lane-per-row
// kernels of the entry points above (Two-Pass, or Three-Pass with recomputation): a lane holds
// its row in a few cache lines that it has just read itself, so x still comes from memory
// once, and no group of lanes would be busy holding so little.
template <class IOV, class IOS>
static int onchip_any(int algo, const typename IOV::elem *x, typename IOV::elem *y, int64_t rows,
                      int64_t n, void *stream)
{
    constexpr int es = (int)sizeof(typename IOV::elem);
    if (n > 0 && rows > 0 && n <= kSoloRowMaxElems[es == 4 ? 0 : 1]) {
        const int rc = check_args(x, y, rows, n, es);
        if (rc != TP_OK)
            return rc;
        if (!congruent16(x, y))
            return TP_ERR_ALIGN;
        return softmax_any<IOV, IOS>(algo == kOnchipTwoPass ? kTwoPass : kRecompute, x, y, rows, n,
                                     stream);
    }
    return run_onchip<IOV>(algo, x, y, rows, n, stream);
}

}  // namespace tp

// ===========================================================================
// C ABI
// ===========================================================================

using namespace tp;

extern "C" {

int softmax2p_f32(const float *x, float *y, int64_t rows, int64_t n, void *stream)
{
    return softmax_any<F32x4, F32x1>(kTwoPass, x, y, rows, n, stream);
}

int softmax3p_recompute_f32(const float *x, float *y, int64_t rows, int64_t n, void *stream)
{
    return softmax_any<F32x4, F32x1>(kRecompute, x, y, rows, n, stream);
}

int softmax3p_reload_f32(const float *x, float *y, int64_t rows, int64_t n, void *stream)
{
    return softmax_any<F32x4, F32x1>(kReload, x, y, rows, n, stream);
}

int softmax2p_bf16io(const uint16_t *x, uint16_t *y, int64_t rows, int64_t n, void *stream)
{
    return softmax_any<BF16x8, BF16x1>(kTwoPass, x, y, rows, n, stream);
}

int softmax3p_recompute_bf16io(const uint16_t *x, uint16_t *y, int64_t rows, int64_t n,
                               void *stream)
{
    return softmax_any<BF16x8, BF16x1>(kRecompute, x, y, rows, n, stream);
}

int softmax3p_reload_bf16io(const uint16_t *x, uint16_t *y, int64_t rows, int64_t n, void *stream)
{
    return softmax_any<BF16x8, BF16x1>(kReload, x, y, rows, n, stream);
}

int softmax2p_f16io(const uint16_t *x, uint16_t *y, int64_t rows, int64_t n, void *stream)
{
    return softmax_any<F16x8, F16x1>(kTwoPass, x, y, rows, n, stream);
}

int softmax3p_recompute_f16io(const uint16_t *x, uint16_t *y, int64_t rows, int64_t n,
                              void *stream)
{
    return softmax_any<F16x8, F16x1>(kRecompute, x, y, rows, n, stream);
}

int softmax3p_reload_f16io(const uint16_t *x, uint16_t *y, int64_t rows, int64_t n, void *stream)
{
    return softmax_any<F16x8, F16x1>(kReload, x, y, rows, n, stream);
}

int softmax2p_onchip_f32(const float *x, float *y, int64_t rows, int64_t n, void *stream)
{
    return onchip_any<F32x4, F32x1>(kOnchipTwoPass, x, y, rows, n, stream);
}

int softmax2p_onchip_bf16io(const uint16_t *x, uint16_t *y, int64_t rows, int64_t n, void *stream)
{
    return onchip_any<BF16x8, BF16x1>(kOnchipTwoPass, x, y, rows, n, stream);
}

int softmax2p_onchip_f16io(const uint16_t *x, uint16_t *y, int64_t rows, int64_t n, void *stream)
{
    return onchip_any<F16x8, F16x1>(kOnchipTwoPass, x, y, rows, n, stream);
}

int softmax3p_onchip_f16io(const uint16_t *x, uint16_t *y, int64_t rows, int64_t n, void *stream)
{
    return onchip_any<F16x8, F16x1>(kOnchipThreePass, x, y, rows, n, stream);
}

int softmax3p_onchip_f32(const float *x, float *y, int64_t rows, int64_t n, void *stream)
{
    return onchip_any<F32x4, F32x1>(kOnchipThreePass, x, y, rows, n, stream);
}

int softmax3p_onchip_bf16io(const uint16_t *x, uint16_t *y, int64_t rows, int64_t n, void *stream)
{
    return onchip_any<BF16x8, BF16x1>(kOnchipThreePass, x, y, rows, n, stream);
}

static int run_extexp(bool hw, const float *x, float *m, float *e, int64_t count, void *stream)
{
    if (count < 0)
        return TP_ERR_NEGATIVE;
    if (count == 0)
        return TP_OK;
    if (!x || !m || !e)
        return TP_ERR_NULL;
    if (((uintptr_t)x | (uintptr_t)m | (uintptr_t)e) % 4)
        return TP_ERR_ALIGN;
    int64_t blocks = (count + 255) / 256;
    if (blocks > 65536)
        blocks = 65536;
    return launch(hw ? extexp_kernel<true> : extexp_kernel<false>, dim3((uint32_t)blocks), dim3(256),
                  (hipStream_t)stream, x, m, e, count);
}

int softmax_tp_extexp_f32(const float *x, float *m, float *e, int64_t count, void *stream)
{
    return run_extexp(false, x, m, e, count, stream);
}

int softmax_tp_extexp_hw_f32(const float *x, float *m, float *e, int64_t count, void *stream)
{
    return run_extexp(true, x, m, e, count, stream);
}

// The pass-level entry points always use the chunk kernels, also for shapes the full
// call would give to the rows path.
int softmax2p_f32_pass1(const float *x, float *pairs, int64_t rows, int64_t n, void *stream)
{
    int rc = check_args(x, pairs, rows, n, 4);
    if (rc != TP_OK || rows == 0 || n == 0)
        return rc;
    if ((uintptr_t)pairs % 8)
        return TP_ERR_ALIGN;
    softmax_tp_plan_t plan;
    // a read-only pass can use 16-byte loads whatever the alignment of x
    if ((rc = make_plan(rows, n, 4, true, 2, &plan)) != TP_OK)
        return rc;
    hipStream_t st = (hipStream_t)stream;
    float *ws = nullptr;
    if ((rc = workspace(st, (size_t)plan.workspace_bytes, &ws)) != TP_OK)
        return rc;
    return run_2p_pass1<F32x4>(plan, x, rows, n, st, (float2 *)ws, (float2 *)pairs);
}

int softmax2p_f32_pass2(const float *x, const float *pairs, float *y, int64_t rows, int64_t n,
                        void *stream)
{
    int rc = check_args(x, y, rows, n, 4);
    if (rc != TP_OK || rows == 0 || n == 0)
        return rc;
    if (!pairs)
        return TP_ERR_NULL;
    if ((uintptr_t)pairs % 8)
        return TP_ERR_ALIGN;
    const bool vec = congruent16(x, y);
    softmax_tp_plan_t plan;
    if ((rc = make_plan(rows, n, 4, vec, 2, &plan)) != TP_OK)
        return rc;
    hipStream_t st = (hipStream_t)stream;
    return vec ? run_2p_pass2<F32x4>(plan, x, y, rows, n, st, (const float2 *)pairs, 1)
               : run_2p_pass2<F32x1>(plan, x, y, rows, n, st, (const float2 *)pairs, 1);
}

int softmax_tp_stream_read_f32(const float *x, float *sink, int64_t count, void *stream)
{
    int rc = check_args(x, sink, 1, count, 4);
    if (rc != TP_OK || count == 0)
        return rc;
    softmax_tp_plan_t plan;
    if ((rc = make_plan(1, count, 4, true, 2, &plan)) != TP_OK)
        return rc;
    hipStream_t st = (hipStream_t)stream;
    float *ws = nullptr;
    if ((rc = workspace(st, (size_t)plan.workspace_bytes, &ws)) != TP_OK)
        return rc;
    const ChunkArgs a = chunk_args(count, plan.reduce, 1, false);
    const dim3 grid = chunk_grid(1, plan.reduce);
    rc = with_shape<F32x4>(plan.reduce, [&](auto B, auto U) {
        return launch(chunk_read<F32x4, TP_B, TP_U>, grid, dim3(TP_B), st, x, a, ws);
    });
    if (rc != TP_OK)
        return rc;
    return launch(merge_sum_kernel, dim3(1), dim3(kMergeBlock), st, (const float *)ws,
                  (int)plan.reduce.chunks, sink);
}

int softmax_tp_stream_copy_f32(const float *x, float *y, int64_t count, void *stream)
{
    int rc = check_args(x, y, 1, count, 4);
    if (rc != TP_OK || count == 0)
        return rc;
    const bool vec = congruent16(x, y);
    softmax_tp_plan_t plan;
    if ((rc = make_plan(1, count, 4, vec, 2, &plan)) != TP_OK)
        return rc;
    hipStream_t st = (hipStream_t)stream;
    const ChunkArgs a = chunk_args(count, plan.map, 1, false);
    const dim3 grid = chunk_grid(1, plan.map);
    if (vec)
        return with_shape<F32x4>(plan.map, [&](auto B, auto U) {
            return launch(chunk_copy<F32x4, TP_B, TP_U>, grid, dim3(TP_B), st, x, y, a);
        });
    return with_shape<F32x1>(plan.map, [&](auto B, auto U) {
        return launch(chunk_copy<F32x1, TP_B, TP_U>, grid, dim3(TP_B), st, x, y, a);
    });
}

int softmax_tp_stream_fill_f32(float *y, float value, int64_t count, void *stream)
{
    int rc = check_args(y, y, 1, count, 4);
    if (rc != TP_OK || count == 0)
        return rc;
    softmax_tp_plan_t plan;
    if ((rc = make_plan(1, count, 4, true, 2, &plan)) != TP_OK)
        return rc;
    const ChunkArgs a = chunk_args(count, plan.map, 1, false);
    const dim3 grid = chunk_grid(1, plan.map);
    return with_shape<F32x4>(plan.map, [&](auto B, auto U) {
        return launch(chunk_fill<TP_B, TP_U>, grid, dim3(TP_B), (hipStream_t)stream, y, a, value);
    });
}

int softmax_tp_stream_scale_f32(const float *x, float *y, float scale, int64_t count, void *stream)
{
    int rc = check_args(x, y, 1, count, 4);
    if (rc != TP_OK || count == 0)
        return rc;
    const bool vec = congruent16(x, y);
    softmax_tp_plan_t plan;
    if ((rc = make_plan(1, count, 4, vec, 2, &plan)) != TP_OK)
        return rc;
    hipStream_t st = (hipStream_t)stream;
    const ChunkArgs a = chunk_args(count, plan.map, 1, false);
    const dim3 grid = chunk_grid(1, plan.map);
    const float *none = nullptr;
    if (vec)
        return with_shape<F32x4>(plan.map, [&](auto B, auto U) {
            return launch(chunk_scale<F32x4, TP_B, TP_U>, grid, dim3(TP_B), st, x, y, a, none, 0,
                          scale);
        });
    return with_shape<F32x1>(plan.map, [&](auto B, auto U) {
        return launch(chunk_scale<F32x1, TP_B, TP_U>, grid, dim3(TP_B), st, x, y, a, none, 0, scale);
    });
}

// ---- Two-Pass softmax that allocates nothing ------------------------------------------
//
// The partial results of the chunk path live in a device array that is part of the library's
// code object.  Each GPU holds its own copy at its own address; the address is looked up once
// per device with that device current and kept.  In host code the array's name is only a
// handle for that lookup, never a pointer to hand to a kernel.
static __device__ __align__(256) unsigned char scratch[TP_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static void *g_scratch_ptr[kMaxDevices];

static int static_scratch(float **out)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess)
        return (int)e;
    if (dev < 0 || dev >= kMaxDevices)
        return (int)hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess)
            return (int)e;
        if (!ptr)
            return (int)hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = ptr;
    }
    *out = (float *)g_scratch_ptr[dev];
    return TP_OK;
}

int softmax2p_f32_static(const float *x, float *y, int64_t rows, int64_t n, void *stream)
{
    int rc = check_args(x, y, rows, n, 4);
    if (rc != TP_OK || rows == 0 || n == 0)
        return rc;
    const bool vec = vector_access(x, y, n, 4);
    softmax_tp_plan_t plan;
    if ((rc = make_plan(rows, n, 4, vec, 0, &plan)) != TP_OK)
        return rc;
    hipStream_t st = (hipStream_t)stream;
    if (plan.path == 1)  // one workgroup per row: no partial results outside the workgroup
        return vec ? run_rows<F32x4>(kTwoPass, plan, x, y, rows, n, st)
                   : run_rows<F32x1>(kTwoPass, plan, x, y, rows, n, st);
    if (two_pass_scratch_bytes(plan, rows) > (int64_t)TP_STATIC_SCRATCH_BYTES)
        return TP_ERR_SCRATCH;
    // Every slot that pass 2 or the merge reads is written by pass 1 of the same call first, so
    // nothing has to be cleared, whatever an earlier call left behind.
    float *ws = nullptr;
    if ((rc = static_scratch(&ws)) != TP_OK)
        return rc;
    return vec ? run_chunks_2p_on<F32x4>(ws, plan, x, y, rows, n, st)
               : run_chunks_2p_on<F32x1>(ws, plan, x, y, rows, n, st);
}

int softmax_tp_plan(int64_t rows, int64_t n, int32_t elem_bytes, int32_t congruent,
                    softmax_tp_plan_t *plan)
{
    return make_plan(rows, n, elem_bytes, congruent != 0, 0, plan);
}

int softmax_tp_tune(const char *key, int64_t value)
{
    if (!key)
        return TP_ERR_NULL;
    if (value < 0)
        return TP_ERR_TUNING;
    enum { kAny, kBlock, kUnroll, kThree };
    struct {
        const char *name;
        int64_t *slot;
        int kind;
    } keys[] = {
        {"path", &g_tune_shared.path, kThree},
        {"block_rows", &g_tune_shared.block_rows, kBlock},
        {"unroll_rows", &g_tune_shared.unroll_rows, kUnroll},
        {"block_reduce", &g_tune_shared.block_reduce, kBlock},
        {"unroll_reduce", &g_tune_shared.unroll_reduce, kUnroll},
        {"target_reduce", &g_tune_shared.target_reduce, kAny},
        {"block_map", &g_tune_shared.block_map, kBlock},
        {"unroll_map", &g_tune_shared.unroll_map, kUnroll},
        {"tiles_map", &g_tune_shared.tiles_map, kAny},
        {"block_mapsum", &g_tune_shared.block_mapsum, kBlock},
        {"unroll_mapsum", &g_tune_shared.unroll_mapsum, kUnroll},
        {"tiles_mapsum", &g_tune_shared.tiles_mapsum, kAny},
        {"direction", &g_tune_shared.direction, kThree},
        {"nt_first", &g_tune_shared.nt_first, kThree},
        {"fold_max", &g_tune_shared.fold_max, kAny},
        {"nt_store", &g_tune_shared.nt_store, kThree},
        {"scalar_io", &g_tune_shared.scalar_io, kThree},
    };
    std::lock_guard<std::mutex> lock(g_tune_mutex);
    for (auto &k : keys) {
        if (std::strcmp(key, k.name) != 0)
            continue;
        if (value != 0) {
            const bool rows_key = k.slot == &g_tune_shared.block_rows || k.slot == &g_tune_shared.unroll_rows;
            if (k.kind == kBlock && !valid_block(value) &&
                !(rows_key && (value == kSolo || value == kTiny || value == kQuad || value == kWave)))
                return TP_ERR_TUNING;
            if (k.kind == kUnroll && !valid_unroll(value, 4) && !(rows_key && value == 3))
                return TP_ERR_TUNING;
            if (k.kind == kThree && value > 2) return TP_ERR_TUNING;
            if (k.slot == &g_tune_shared.fold_max && value > 4096) return TP_ERR_TUNING;
        }
        *k.slot = value;
        return TP_OK;
    }
    return TP_ERR_TUNING;
}

int softmax_tp_reserve(int64_t rows, int64_t n, int32_t elem_bytes, void *stream)
{
    // The largest workspace any entry point can ask for with this shape: x and y congruent
    // modulo 16 bytes or not (element-wise accesses make more, shorter chunks in the pass that
    // stores and sums), and the chunk path forced, as the pass-level entry points do for shapes
    // whose full call takes the rows path.
    int64_t bytes = 0;
    for (int congruent = 0; congruent < 2; ++congruent)
        for (int force_path = 0; force_path <= 2; force_path += 2) {
            softmax_tp_plan_t plan;
            const int rc = make_plan(rows, n, elem_bytes, congruent != 0, force_path, &plan);
            if (rc != TP_OK)
                return rc;
            if (plan.workspace_bytes > bytes)
                bytes = plan.workspace_bytes;
        }
    if (bytes == 0)
        return TP_OK;
    float *ws = nullptr;
    return workspace((hipStream_t)stream, (size_t)bytes, &ws);
}

int softmax_tp_release(void)
{
    std::lock_guard<std::mutex> lock(g_ws_mutex);
    int rc = TP_OK;
    for (auto &kv : g_ws) {
        if (!kv.second.ptr)
            continue;
        int prev = 0;
        (void)hipGetDevice(&prev);
        (void)hipSetDevice(kv.first.first);
        const hipError_t e = hipFree(kv.second.ptr);
        (void)hipSetDevice(prev);
        if (e != hipSuccess)
            rc = (int)e;
    }
    g_ws.clear();
    return rc;
}

const char *softmax_tp_strerror(int code)
{
    switch (code) {
    case TP_OK: return "success";
    case TP_ERR_NULL: return "null pointer";
    case TP_ERR_NEGATIVE: return "negative size";
    case TP_ERR_TOO_LARGE: return "problem too large";
    case TP_ERR_ALIGN: return "pointer not aligned to the element size";
    case TP_ERR_TUNING: return "bad tuning key, value or unsupported configuration";
    case TP_ERR_SCRATCH: return "partial results exceed the static scratch buffer";
    default: return code > 0 ? hipGetErrorString((hipError_t)code) : "unknown error";
    }
}

}  // extern "C"
