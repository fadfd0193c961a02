// Kernels and C ABI of the Two-Pass softmax and its Three-Pass baselines (gfx950).
//
// Two launch shapes (see softmax_tp_plan):
//   rows path   one workgroup owns a whole row and runs every pass of the
//               algorithm in one launch; the re-read of the row comes from L2.
//   chunk path  a row is cut into chunks, one workgroup each.  A reducing pass
//               leaves one partial result per chunk in the workspace; the
//               workgroups of the next pass merge the partials of their row
//               themselves, or a small merge kernel does when there are many.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstring>
#include <map>
#include <mutex>
#include <utility>

#include "../../include/softmax_tp.h"
#include "tp_device.h"

namespace tp {

// ===========================================================================
// kernels
// ===========================================================================

// Loads of a pass whose data is read again later stay cacheable; the last read
// of x and every store of y are streamed (nt) so they do not displace it.
constexpr bool kKeep = false, kStream = true;

template <int BLOCK>
__device__ __forceinline__ void merge_pairs(const float2 *p, int cnt, float &m, float &n,
                                            float *lds)
{
    m = 0.f;
    n = kNIdent;
    for (int i = threadIdx.x; i < cnt; i += BLOCK) {
        float2 q = p[i];
        float nmax = fmaxf(n, q.y);
        m = scale_pow2(m, n - nmax) + scale_pow2(q.x, q.y - nmax);
        n = nmax;
    }
    block_pair<BLOCK>(m, n, lds);
}

template <int BLOCK>
__device__ __forceinline__ float merge_max(const float *p, int cnt, float *lds)
{
    float v = -__builtin_inff();
    for (int i = threadIdx.x; i < cnt; i += BLOCK)
        v = fmaxf(v, p[i]);
    return block_max<BLOCK>(v, lds);
}

template <int BLOCK>
__device__ __forceinline__ float merge_sum(const float *p, int cnt, float *lds)
{
    float v = 0.f;
    for (int i = threadIdx.x; i < cnt; i += BLOCK)
        v += p[i];
    return block_sum<BLOCK>(v, lds);
}

// ---- rows path: grid = rows ------------------------------------------------

template <class IO, int BLOCK, int U>
__global__ __launch_bounds__(BLOCK) void rows_2p(const typename IO::elem *x,
                                                 typename IO::elem *y, int64_t n)
{
    __shared__ float lds[2 * kMaxWaves];
    const Seg<IO> s = make_seg<IO>(x, y, n, blockIdx.x, 0, INT64_MAX / 2);
    PairSum acc;
    stream<IO, BLOCK, U, kKeep, kStream>(s, acc);
    block_pair<BLOCK>(acc.m, acc.n, lds);
    PairOut out{1.0f / acc.m, acc.n};
    stream<IO, BLOCK, U, kStream, kStream>(s, out);
}

template <class IO, int BLOCK, int U>
__global__ __launch_bounds__(BLOCK) void rows_3p_recompute(const typename IO::elem *x,
                                                           typename IO::elem *y, int64_t n)
{
    __shared__ float lds[2 * kMaxWaves];
    const Seg<IO> s = make_seg<IO>(x, y, n, blockIdx.x, 0, INT64_MAX / 2);
    MaxOf mx;
    stream<IO, BLOCK, U, kKeep, kStream>(s, mx);
    const float mu = block_max<BLOCK>(mx.mx, lds);
    SumExp se{mu};
    stream<IO, BLOCK, U, kKeep, kStream>(s, se);
    const float sigma = block_sum<BLOCK>(se.s, lds);
    ExpScale es{mu, 1.0f / sigma};
    stream<IO, BLOCK, U, kStream, kStream>(s, es);
}

template <class IO, int BLOCK, int U>
__global__ __launch_bounds__(BLOCK) void rows_3p_reload(const typename IO::elem *x,
                                                        typename IO::elem *y, int64_t n)
{
    __shared__ float lds[2 * kMaxWaves];
    const Seg<IO> s = make_seg<IO>(x, y, n, blockIdx.x, 0, INT64_MAX / 2);
    MaxOf mx;
    stream<IO, BLOCK, U, kKeep, kStream>(s, mx);
    const float mu = block_max<BLOCK>(mx.mx, lds);
    ExpStoreSum ess{mu};
    stream<IO, BLOCK, U, kStream, kKeep>(s, ess);  // y is read back in the next pass
    const float sigma = block_sum<BLOCK>(ess.s, lds);
    __syncthreads();  // every store of this workgroup to y is issued before y is re-read
    const Seg<IO> sy = make_seg<IO>(y, y, n, blockIdx.x, 0, INT64_MAX / 2);
    Scale sc{1.0f / sigma};
    stream<IO, BLOCK, U, kStream, kStream>(sy, sc);
}

// ---- chunk path: grid = rows * chunks --------------------------------------

struct ChunkArgs {
    int64_t n;
    int64_t chunk_vecs;
    int32_t chunks;
};

#define TP_CHUNK_PROLOGUE                                                         \
    __shared__ float lds[2 * kMaxWaves];                                          \
    const int64_t row = blockIdx.x / (uint32_t)a.chunks;                          \
    const int64_t chunk = blockIdx.x % (uint32_t)a.chunks;

template <class IO, int BLOCK, int U>
__global__ __launch_bounds__(BLOCK) void chunk_2p_pass1(const typename IO::elem *x, ChunkArgs a,
                                                        float2 *partial)
{
    TP_CHUNK_PROLOGUE
    const Seg<IO> s = make_seg<IO>(x, nullptr, a.n, row, chunk, a.chunk_vecs);
    PairSum acc;
    stream<IO, BLOCK, U, kKeep, kStream>(s, acc);
    block_pair<BLOCK>(acc.m, acc.n, lds);
    if (threadIdx.x == 0)
        partial[blockIdx.x] = make_float2(acc.m, acc.n);
}

// pairs: `npairs` pairs per row (the chunk partials, or 1 after the merge kernel)
template <class IO, int BLOCK, int U>
__global__ __launch_bounds__(BLOCK) void chunk_2p_pass2(const typename IO::elem *x,
                                                        typename IO::elem *y, ChunkArgs a,
                                                        const float2 *pairs, int npairs)
{
    TP_CHUNK_PROLOGUE
    float m_sum, n_sum;
    merge_pairs<BLOCK>(pairs + row * npairs, npairs, m_sum, n_sum, lds);
    const Seg<IO> s = make_seg<IO>(x, y, a.n, row, chunk, a.chunk_vecs);
    PairOut out{1.0f / m_sum, n_sum};
    stream<IO, BLOCK, U, kStream, kStream>(s, out);
}

template <int BLOCK>
__global__ __launch_bounds__(BLOCK) void merge_pairs_kernel(const float2 *partial, int chunks,
                                                            float2 *out)
{
    __shared__ float lds[2 * kMaxWaves];
    float m, n;
    merge_pairs<BLOCK>(partial + (int64_t)blockIdx.x * chunks, chunks, m, n, lds);
    if (threadIdx.x == 0)
        out[blockIdx.x] = make_float2(m, n);
}

template <class IO, int BLOCK, int U>
__global__ __launch_bounds__(BLOCK) void chunk_max(const typename IO::elem *x, ChunkArgs a,
                                                   float *pmax)
{
    TP_CHUNK_PROLOGUE
    const Seg<IO> s = make_seg<IO>(x, nullptr, a.n, row, chunk, a.chunk_vecs);
    MaxOf mx;
    stream<IO, BLOCK, U, kKeep, kStream>(s, mx);
    const float v = block_max<BLOCK>(mx.mx, lds);
    if (threadIdx.x == 0)
        pmax[blockIdx.x] = v;
}

template <class IO, int BLOCK, int U>
__global__ __launch_bounds__(BLOCK) void chunk_sumexp(const typename IO::elem *x, ChunkArgs a,
                                                      const float *pmax, int nmax, float *psum)
{
    TP_CHUNK_PROLOGUE
    const float mu = merge_max<BLOCK>(pmax + row * nmax, nmax, lds);
    const Seg<IO> s = make_seg<IO>(x, nullptr, a.n, row, chunk, a.chunk_vecs);
    SumExp se{mu};
    stream<IO, BLOCK, U, kKeep, kStream>(s, se);
    const float v = block_sum<BLOCK>(se.s, lds);
    if (threadIdx.x == 0)
        psum[blockIdx.x] = v;
}

template <class IO, int BLOCK, int U>
__global__ __launch_bounds__(BLOCK) void chunk_expscale(const typename IO::elem *x,
                                                        typename IO::elem *y, ChunkArgs a,
                                                        const float *pmax, int nmax,
                                                        const float *psum, int nsum)
{
    TP_CHUNK_PROLOGUE
    const float mu = merge_max<BLOCK>(pmax + row * nmax, nmax, lds);
    const float sigma = merge_sum<BLOCK>(psum + row * nsum, nsum, lds);
    const Seg<IO> s = make_seg<IO>(x, y, a.n, row, chunk, a.chunk_vecs);
    ExpScale es{mu, 1.0f / sigma};
    stream<IO, BLOCK, U, kStream, kStream>(s, es);
}

template <class IO, int BLOCK, int U>
__global__ __launch_bounds__(BLOCK) void chunk_expstore(const typename IO::elem *x,
                                                        typename IO::elem *y, ChunkArgs a,
                                                        const float *pmax, int nmax, float *psum)
{
    TP_CHUNK_PROLOGUE
    const float mu = merge_max<BLOCK>(pmax + row * nmax, nmax, lds);
    const Seg<IO> s = make_seg<IO>(x, y, a.n, row, chunk, a.chunk_vecs);
    ExpStoreSum ess{mu};
    stream<IO, BLOCK, U, kStream, kKeep>(s, ess);
    const float v = block_sum<BLOCK>(ess.s, lds);
    if (threadIdx.x == 0)
        psum[blockIdx.x] = v;
}

// y = y / sigma in place (reload pass 3); with psum == nullptr: y = lambda * x (calibration).
template <class IO, int BLOCK, int U>
__global__ __launch_bounds__(BLOCK) void chunk_scale(const typename IO::elem *x,
                                                     typename IO::elem *y, ChunkArgs a,
                                                     const float *psum, int nsum, float lambda)
{
    TP_CHUNK_PROLOGUE
    if (psum)
        lambda = 1.0f / merge_sum<BLOCK>(psum + row * nsum, nsum, lds);
    const Seg<IO> s = make_seg<IO>(x, y, a.n, row, chunk, a.chunk_vecs);
    Scale sc{lambda};
    stream<IO, BLOCK, U, kStream, kStream>(s, sc);
}

template <int BLOCK>
__global__ __launch_bounds__(BLOCK) void merge_max_kernel(const float *p, int chunks, float *out)
{
    __shared__ float lds[2 * kMaxWaves];
    const float v = merge_max<BLOCK>(p + (int64_t)blockIdx.x * chunks, chunks, lds);
    if (threadIdx.x == 0)
        out[blockIdx.x] = v;
}

template <int BLOCK>
__global__ __launch_bounds__(BLOCK) void merge_sum_kernel(const float *p, int chunks, float *out)
{
    __shared__ float lds[2 * kMaxWaves];
    const float v = merge_sum<BLOCK>(p + (int64_t)blockIdx.x * chunks, chunks, lds);
    if (threadIdx.x == 0)
        out[blockIdx.x] = v;
}

// ---- calibration and debug -------------------------------------------------

template <class IO, int BLOCK, int U>
__global__ __launch_bounds__(BLOCK) void chunk_read(const typename IO::elem *x, ChunkArgs a,
                                                    float *psum)
{
    TP_CHUNK_PROLOGUE
    const Seg<IO> s = make_seg<IO>(x, nullptr, a.n, row, chunk, a.chunk_vecs);
    SumOf so;
    stream<IO, BLOCK, U, kStream, kStream>(s, so);
    const float v = block_sum<BLOCK>(so.s, lds);
    if (threadIdx.x == 0)
        psum[blockIdx.x] = v;
}

template <class IO, int BLOCK, int U>
__global__ __launch_bounds__(BLOCK) void chunk_copy(const typename IO::elem *x,
                                                    typename IO::elem *y, ChunkArgs a)
{
    TP_CHUNK_PROLOGUE
    (void)lds;
    const Seg<IO> s = make_seg<IO>(x, y, a.n, row, chunk, a.chunk_vecs);
    Copy cp;
    stream<IO, BLOCK, U, kStream, kStream>(s, cp);
}

__global__ __launch_bounds__(256) void extexp_kernel(const float *x, float *m, float *e,
                                                     int64_t count)
{
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t step = (int64_t)gridDim.x * 256;
    for (; i < count; i += step)
        tp_extexp(x[i], &m[i], &e[i]);
}

// ===========================================================================
// host side
// ===========================================================================

struct Tuning {
    int64_t path = 0;
    int64_t block_rows = 0, unroll_rows = 0;
    int64_t block_chunk = 0, unroll_chunk = 0;
    int64_t target_chunks = 0, min_chunk_vecs = 0, fold_max = 0;
};
static Tuning g_tune;

constexpr int64_t kRowsPathMaxBytes = 256 * 1024;  // longest row one workgroup takes
constexpr int64_t kRowsPathMinRows = 32;           // fewer rows than this cannot fill the chip
constexpr int64_t kSmallRowBytes = 32 * 1024;      // ... unless the rows are this short
constexpr int64_t kTargetChunks = 4096;            // workgroups aimed for on the chunk path
constexpr int64_t kFoldMax = 64;                   // partials merged inside the next pass
constexpr int64_t kGridMax = 0x7FFFFFFF;

static bool valid_block(int64_t b) { return b == 256 || b == 512 || b == 1024; }
static bool valid_unroll(int64_t u) { return u == 2 || u == 4 || u == 8; }

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
    if (n > INT64_MAX / elem_bytes / rows)
        return TP_ERR_TOO_LARGE;
    const int V = congruent16 ? 16 / elem_bytes : 1;
    const int64_t nvec = (n + V - 1) / V;  // upper bound on full vectors per row
    const int64_t row_bytes = n * elem_bytes;
    p->vector_elems = V;

    bool rows_path = row_bytes <= kRowsPathMaxBytes &&
                     (rows >= kRowsPathMinRows || row_bytes <= kSmallRowBytes);
    const int64_t forced = force_path ? force_path : g_tune.path;
    if (forced == 1)
        rows_path = true;
    if (forced == 2)
        rows_path = false;
    if (rows_path && rows > kGridMax)
        return TP_ERR_TOO_LARGE;

    if (rows_path) {
        p->path = 1;
        p->block = nvec >= 4096 ? 1024 : nvec >= 1536 ? 512 : 256;
        p->unroll = 4;
        if (g_tune.block_rows) p->block = (int32_t)g_tune.block_rows;
        if (g_tune.unroll_rows) p->unroll = (int32_t)g_tune.unroll_rows;
        p->launches = 1;
        return TP_OK;
    }

    p->path = 2;
    p->block = g_tune.block_chunk ? (int32_t)g_tune.block_chunk : 256;
    p->unroll = g_tune.unroll_chunk ? (int32_t)g_tune.unroll_chunk : 4;
    const int64_t tile = (int64_t)p->block * p->unroll;  // vectors per workgroup iteration
    const int64_t target = g_tune.target_chunks ? g_tune.target_chunks : kTargetChunks;
    const int64_t min_cv = g_tune.min_chunk_vecs ? g_tune.min_chunk_vecs : 2 * tile;
    int64_t per_row = (target + rows - 1) / rows;  // chunks per row aimed for
    if (per_row < 1) per_row = 1;
    int64_t cv = (nvec + per_row - 1) / per_row;
    if (cv < min_cv) cv = min_cv;
    cv = (cv + tile - 1) / tile * tile;
    if (cv > (int64_t)1 << 26)  // a chunk is indexed with 32-bit vector offsets
        cv = (int64_t)1 << 26;
    int64_t chunks = (nvec + cv - 1) / cv;
    if (chunks < 1) chunks = 1;
    if (chunks > kGridMax / rows || chunks > 0x7FFFFFF)
        return TP_ERR_TOO_LARGE;
    p->chunk_vecs = cv;
    p->chunks = chunks;
    const int64_t fold = g_tune.fold_max ? g_tune.fold_max : kFoldMax;
    p->merge_kernel = chunks > fold ? 1 : 0;
    p->launches = 2 + p->merge_kernel;
    p->workspace_bytes = (2 * rows * chunks + 2 * rows) * (int64_t)sizeof(float);
    return TP_OK;
}

// ---- workspace: one buffer per (device, stream) -----------------------------

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
        size_t want = bytes < (size_t)65536 ? (size_t)65536 : bytes;
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

static int launch_status()
{
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? TP_OK : (int)e;
}

// ---- dispatch over (BLOCK, U) ------------------------------------------------

// bf16 vectors unpack to 8 floats each, so 8 of them in flight would not fit the
// register budget of a 1024-thread workgroup: the bf16 formats stop at 4.
#define TP_BU_CASE(IO, B, UU, CALL)                                         \
    case B * 16 + UU:                                                       \
        if constexpr (sizeof(typename IO::elem) == 2 && UU == 8) {          \
            return TP_ERR_TUNING;                                           \
        } else {                                                            \
            CALL(IO, B, UU);                                                \
        }                                                                   \
        break;

#define TP_BU_CASES(IO, CALL)                 \
    switch (plan.block * 16 + plan.unroll) {  \
        TP_BU_CASE(IO, 256, 2, CALL)          \
        TP_BU_CASE(IO, 256, 4, CALL)          \
        TP_BU_CASE(IO, 256, 8, CALL)          \
        TP_BU_CASE(IO, 512, 2, CALL)          \
        TP_BU_CASE(IO, 512, 4, CALL)          \
        TP_BU_CASE(IO, 512, 8, CALL)          \
        TP_BU_CASE(IO, 1024, 2, CALL)         \
        TP_BU_CASE(IO, 1024, 4, CALL)         \
        TP_BU_CASE(IO, 1024, 8, CALL)         \
    default:                                  \
        return TP_ERR_TUNING;                 \
    }

enum Algo { kTwoPass, kRecompute, kReload };

template <class IO>
static int run_rows(Algo algo, const softmax_tp_plan_t &plan, const typename IO::elem *x,
                    typename IO::elem *y, int64_t rows, int64_t n, hipStream_t st)
{
    const dim3 grid((uint32_t)rows);
#define TP_CALL_ROWS(IOT, B, UU)                                                               \
    do {                                                                                       \
        if constexpr (sizeof(typename IOT::elem) == 2) { /* bf16: Two-Pass only */             \
            hipLaunchKernelGGL((rows_2p<IOT, B, UU>), grid, dim3(B), 0, st, x, y, n);          \
        } else {                                                                               \
            if (algo == kTwoPass)                                                              \
                hipLaunchKernelGGL((rows_2p<IOT, B, UU>), grid, dim3(B), 0, st, x, y, n);      \
            else if (algo == kRecompute)                                                       \
                hipLaunchKernelGGL((rows_3p_recompute<IOT, B, UU>), grid, dim3(B), 0, st, x, y, \
                                   n);                                                         \
            else                                                                               \
                hipLaunchKernelGGL((rows_3p_reload<IOT, B, UU>), grid, dim3(B), 0, st, x, y, n); \
        }                                                                                      \
    } while (0)
    TP_BU_CASES(IO, TP_CALL_ROWS)
#undef TP_CALL_ROWS
    return launch_status();
}

// Two-Pass on the chunk path.  Either half can be skipped (pass-level entry points):
// final_out != nullptr receives the merged pair of every row; final_in supplies it.
template <class IO>
static int run_chunks_2p(const softmax_tp_plan_t &plan, const typename IO::elem *x,
                         typename IO::elem *y, int64_t rows, int64_t n, hipStream_t st,
                         float2 *final_out, const float2 *final_in, bool do_pass2)
{
    const ChunkArgs a{n, plan.chunk_vecs, (int32_t)plan.chunks};
    const dim3 grid((uint32_t)(rows * plan.chunks));
    const float2 *pairs = final_in;
    int npairs = 1;
    if (!final_in) {
        float *ws = nullptr;
        int rc = workspace(st, (size_t)plan.workspace_bytes, &ws);
        if (rc != TP_OK)
            return rc;
        float2 *partial = (float2 *)ws;
        float2 *merged = final_out ? final_out : partial + rows * plan.chunks;
#define TP_CALL_P1(IOT, B, UU) \
    hipLaunchKernelGGL((chunk_2p_pass1<IOT, B, UU>), grid, dim3(B), 0, st, x, a, partial)
        TP_BU_CASES(IO, TP_CALL_P1)
#undef TP_CALL_P1
        rc = launch_status();
        if (rc != TP_OK)
            return rc;
        if (plan.merge_kernel || final_out) {
            hipLaunchKernelGGL((merge_pairs_kernel<256>), dim3((uint32_t)rows), dim3(256), 0, st,
                               partial, (int)plan.chunks, merged);
            rc = launch_status();
            if (rc != TP_OK)
                return rc;
            pairs = merged;
            npairs = 1;
        } else {
            pairs = partial;
            npairs = (int)plan.chunks;
        }
    }
    if (!do_pass2)
        return TP_OK;
#define TP_CALL_P2(IOT, B, UU)                                                               \
    hipLaunchKernelGGL((chunk_2p_pass2<IOT, B, UU>), grid, dim3(B), 0, st, x, y, a, pairs, npairs)
    TP_BU_CASES(IO, TP_CALL_P2)
#undef TP_CALL_P2
    return launch_status();
}

template <class IO>
static int run_chunks_3p(Algo algo, const softmax_tp_plan_t &plan, const typename IO::elem *x,
                         typename IO::elem *y, int64_t rows, int64_t n, hipStream_t st)
{
    const ChunkArgs a{n, plan.chunk_vecs, (int32_t)plan.chunks};
    const dim3 grid((uint32_t)(rows * plan.chunks));
    float *ws = nullptr;
    int rc = workspace(st, (size_t)plan.workspace_bytes, &ws);
    if (rc != TP_OK)
        return rc;
    const int64_t rc_count = rows * plan.chunks;
    float *pmax = ws, *psum = ws + rc_count;
    float *fmax = ws + 2 * rc_count, *fsum = fmax + rows;
    const float *maxes = pmax, *sums = psum;
    int nmax = (int)plan.chunks, nsum = (int)plan.chunks;

#define TP_CALL_MAX(IOT, B, UU) \
    hipLaunchKernelGGL((chunk_max<IOT, B, UU>), grid, dim3(B), 0, st, x, a, pmax)
    TP_BU_CASES(IO, TP_CALL_MAX)
#undef TP_CALL_MAX
    if ((rc = launch_status()) != TP_OK)
        return rc;
    if (plan.merge_kernel) {
        hipLaunchKernelGGL((merge_max_kernel<256>), dim3((uint32_t)rows), dim3(256), 0, st, pmax,
                           (int)plan.chunks, fmax);
        if ((rc = launch_status()) != TP_OK)
            return rc;
        maxes = fmax;
        nmax = 1;
    }
    if (algo == kRecompute) {
#define TP_CALL_SE(IOT, B, UU)                                                                  \
    hipLaunchKernelGGL((chunk_sumexp<IOT, B, UU>), grid, dim3(B), 0, st, x, a, maxes, nmax, psum)
        TP_BU_CASES(IO, TP_CALL_SE)
#undef TP_CALL_SE
    } else {
#define TP_CALL_ES(IOT, B, UU)                                                                 \
    hipLaunchKernelGGL((chunk_expstore<IOT, B, UU>), grid, dim3(B), 0, st, x, y, a, maxes, nmax, \
                       psum)
        TP_BU_CASES(IO, TP_CALL_ES)
#undef TP_CALL_ES
    }
    if ((rc = launch_status()) != TP_OK)
        return rc;
    if (plan.merge_kernel) {
        hipLaunchKernelGGL((merge_sum_kernel<256>), dim3((uint32_t)rows), dim3(256), 0, st, psum,
                           (int)plan.chunks, fsum);
        if ((rc = launch_status()) != TP_OK)
            return rc;
        sums = fsum;
        nsum = 1;
    }
    if (algo == kRecompute) {
#define TP_CALL_XS(IOT, B, UU)                                                                 \
    hipLaunchKernelGGL((chunk_expscale<IOT, B, UU>), grid, dim3(B), 0, st, x, y, a, maxes, nmax, \
                       sums, nsum)
        TP_BU_CASES(IO, TP_CALL_XS)
#undef TP_CALL_XS
    } else {
        const typename IO::elem *yc = y;
#define TP_CALL_SC(IOT, B, UU)                                                                \
    hipLaunchKernelGGL((chunk_scale<IOT, B, UU>), grid, dim3(B), 0, st, yc, y, a, sums, nsum, 0.f)
        TP_BU_CASES(IO, TP_CALL_SC)
#undef TP_CALL_SC
    }
    return launch_status();
}

// ---- argument checks ---------------------------------------------------------

static int check_args(const void *x, const void *y, int64_t rows, int64_t n, int elem_bytes,
                      bool need_y)
{
    if (rows < 0 || n < 0)
        return TP_ERR_NEGATIVE;
    if (rows == 0 || n == 0)
        return TP_OK;
    if (!x || (need_y && !y))
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

template <class IOV, class IOS>
static int softmax_any(Algo algo, const typename IOV::elem *x, typename IOV::elem *y,
                       int64_t rows, int64_t n, void *stream)
{
    constexpr int es = (int)sizeof(typename IOV::elem);
    int rc = check_args(x, y, rows, n, es, true);
    if (rc != TP_OK || rows == 0 || n == 0)
        return rc;
    const bool vec = congruent16(x, y);
    softmax_tp_plan_t plan;
    rc = make_plan(rows, n, es, vec, 0, &plan);
    if (rc != TP_OK)
        return rc;
    if (!valid_block(plan.block) || !valid_unroll(plan.unroll))
        return TP_ERR_TUNING;
    hipStream_t st = (hipStream_t)stream;
    if (plan.path == 1)
        return vec ? run_rows<IOV>(algo, plan, x, y, rows, n, st)
                   : run_rows<IOS>(algo, plan, x, y, rows, n, st);
    if (algo == kTwoPass)
        return vec ? run_chunks_2p<IOV>(plan, x, y, rows, n, st, nullptr, nullptr, true)
                   : run_chunks_2p<IOS>(plan, x, y, rows, n, st, nullptr, nullptr, true);
    if constexpr (es == 4)
        return vec ? run_chunks_3p<IOV>(algo, plan, x, y, rows, n, st)
                   : run_chunks_3p<IOS>(algo, plan, x, y, rows, n, st);
    return TP_ERR_TUNING;
}

// plan for the flat calibration streams: one "row" of `count` floats on the chunk path
static int flat_plan(int64_t count, bool vec, softmax_tp_plan_t *plan)
{
    int rc = make_plan(1, count, 4, vec, 2, plan);
    if (rc == TP_OK && (!valid_block(plan->block) || !valid_unroll(plan->unroll)))
        rc = TP_ERR_TUNING;
    return rc;
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

int softmax_tp_extexp_f32(const float *x, float *m, float *e, int64_t count, void *stream)
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
    hipLaunchKernelGGL(extexp_kernel, dim3((uint32_t)blocks), dim3(256), 0, (hipStream_t)stream, x,
                       m, e, count);
    return launch_status();
}

int softmax2p_f32_pass1(const float *x, float *pairs, int64_t rows, int64_t n, void *stream)
{
    int rc = check_args(x, pairs, rows, n, 4, true);
    if (rc != TP_OK || rows == 0 || n == 0)
        return rc;
    if ((uintptr_t)pairs % 8)
        return TP_ERR_ALIGN;
    softmax_tp_plan_t plan;
    // the pass-level entry points always use the chunk kernels; a read-only pass can
    // use 16-byte loads whatever the alignment of x
    rc = make_plan(rows, n, 4, true, 2, &plan);
    if (rc != TP_OK)
        return rc;
    if (!valid_block(plan.block) || !valid_unroll(plan.unroll))
        return TP_ERR_TUNING;
    return run_chunks_2p<F32x4>(plan, x, nullptr, rows, n, (hipStream_t)stream, (float2 *)pairs,
                                nullptr, false);
}

int softmax2p_f32_pass2(const float *x, const float *pairs, float *y, int64_t rows, int64_t n,
                        void *stream)
{
    int rc = check_args(x, y, rows, n, 4, true);
    if (rc != TP_OK || rows == 0 || n == 0)
        return rc;
    if (!pairs)
        return TP_ERR_NULL;
    if ((uintptr_t)pairs % 8)
        return TP_ERR_ALIGN;
    const bool vec = congruent16(x, y);
    softmax_tp_plan_t plan;
    rc = make_plan(rows, n, 4, vec, 2, &plan);
    if (rc != TP_OK)
        return rc;
    if (!valid_block(plan.block) || !valid_unroll(plan.unroll))
        return TP_ERR_TUNING;
    hipStream_t st = (hipStream_t)stream;
    return vec ? run_chunks_2p<F32x4>(plan, x, y, rows, n, st, nullptr, (const float2 *)pairs, true)
               : run_chunks_2p<F32x1>(plan, x, y, rows, n, st, nullptr, (const float2 *)pairs, true);
}

int softmax_tp_stream_read_f32(const float *x, float *sink, int64_t count, void *stream)
{
    int rc = check_args(x, sink, 1, count, 4, true);
    if (rc != TP_OK || count == 0)
        return rc;
    softmax_tp_plan_t plan;
    if ((rc = flat_plan(count, true, &plan)) != TP_OK)
        return rc;
    hipStream_t st = (hipStream_t)stream;
    float *ws = nullptr;
    if ((rc = workspace(st, (size_t)plan.workspace_bytes, &ws)) != TP_OK)
        return rc;
    const ChunkArgs a{count, plan.chunk_vecs, (int32_t)plan.chunks};
    const dim3 grid((uint32_t)plan.chunks);
#define TP_CALL_RD(IOT, B, UU) \
    hipLaunchKernelGGL((chunk_read<IOT, B, UU>), grid, dim3(B), 0, st, x, a, ws)
    TP_BU_CASES(F32x4, TP_CALL_RD)
#undef TP_CALL_RD
    if ((rc = launch_status()) != TP_OK)
        return rc;
    hipLaunchKernelGGL((merge_sum_kernel<256>), dim3(1), dim3(256), 0, st, ws, (int)plan.chunks,
                       sink);
    return launch_status();
}

int softmax_tp_stream_copy_f32(const float *x, float *y, int64_t count, void *stream)
{
    int rc = check_args(x, y, 1, count, 4, true);
    if (rc != TP_OK || count == 0)
        return rc;
    const bool vec = congruent16(x, y);
    softmax_tp_plan_t plan;
    if ((rc = flat_plan(count, vec, &plan)) != TP_OK)
        return rc;
    hipStream_t st = (hipStream_t)stream;
    const ChunkArgs a{count, plan.chunk_vecs, (int32_t)plan.chunks};
    const dim3 grid((uint32_t)plan.chunks);
#define TP_CALL_CP(IOT, B, UU) \
    hipLaunchKernelGGL((chunk_copy<IOT, B, UU>), grid, dim3(B), 0, st, x, y, a)
    if (vec) {
        TP_BU_CASES(F32x4, TP_CALL_CP)
    } else {
        TP_BU_CASES(F32x1, TP_CALL_CP)
    }
#undef TP_CALL_CP
    return launch_status();
}

int softmax_tp_stream_scale_f32(const float *x, float *y, float scale, int64_t count, void *stream)
{
    int rc = check_args(x, y, 1, count, 4, true);
    if (rc != TP_OK || count == 0)
        return rc;
    const bool vec = congruent16(x, y);
    softmax_tp_plan_t plan;
    if ((rc = flat_plan(count, vec, &plan)) != TP_OK)
        return rc;
    hipStream_t st = (hipStream_t)stream;
    const ChunkArgs a{count, plan.chunk_vecs, (int32_t)plan.chunks};
    const dim3 grid((uint32_t)plan.chunks);
    const float *nosum = nullptr;
#define TP_CALL_SC(IOT, B, UU) \
    hipLaunchKernelGGL((chunk_scale<IOT, B, UU>), grid, dim3(B), 0, st, x, y, a, nosum, 0, scale)
    if (vec) {
        TP_BU_CASES(F32x4, TP_CALL_SC)
    } else {
        TP_BU_CASES(F32x1, TP_CALL_SC)
    }
#undef TP_CALL_SC
    return launch_status();
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
    struct {
        const char *name;
        int64_t *slot;
        int kind;  // 0 any, 1 block, 2 unroll, 3 path
    } keys[] = {
        {"path", &g_tune.path, 3},
        {"block_rows", &g_tune.block_rows, 1},
        {"unroll_rows", &g_tune.unroll_rows, 2},
        {"block_chunk", &g_tune.block_chunk, 1},
        {"unroll_chunk", &g_tune.unroll_chunk, 2},
        {"target_chunks", &g_tune.target_chunks, 0},
        {"min_chunk_vecs", &g_tune.min_chunk_vecs, 0},
        {"fold_max", &g_tune.fold_max, 0},
    };
    for (auto &k : keys) {
        if (std::strcmp(key, k.name) != 0)
            continue;
        if (value != 0) {
            if (k.kind == 1 && !valid_block(value)) return TP_ERR_TUNING;
            if (k.kind == 2 && !valid_unroll(value)) return TP_ERR_TUNING;
            if (k.kind == 3 && value > 2) return TP_ERR_TUNING;
        }
        *k.slot = value;
        return TP_OK;
    }
    return TP_ERR_TUNING;
}

int softmax_tp_release(void)
{
    std::lock_guard<std::mutex> lock(g_ws_mutex);
    int rc = TP_OK;
    for (auto &kv : g_ws) {
        if (kv.second.ptr) {
            int prev = 0;
            (void)hipGetDevice(&prev);
            (void)hipSetDevice(kv.first.first);
            hipError_t e = hipFree(kv.second.ptr);
            (void)hipSetDevice(prev);
            if (e != hipSuccess)
                rc = (int)e;
        }
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
    default: return code > 0 ? hipGetErrorString((hipError_t)code) : "unknown error";
    }
}

}  // extern "C"
