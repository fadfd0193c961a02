/*
 * softmax_tp: Two-Pass softmax (arXiv 2001.04438) and its Three-Pass baselines for
 * AMD MI355X (gfx950), as a C ABI.
 *
 * Every entry point computes, for each of `rows` independent vectors of `n`
 * elements stored contiguously (row-major, row pitch = n elements),
 *
 *        y[r, i] = exp(x[r, i]) / sum_k exp(x[r, k])            (Section 1)
 *
 * Common conventions
 *   x, y     DEVICE pointers.  x is never written.  y == x (exact aliasing) is
 *            allowed; any other overlap is undefined.  Pointers need only be
 *            aligned to the element size; when x and y are congruent modulo 16
 *            bytes the kernels move 128 bits per lane, otherwise they fall back
 *            to element-wise accesses (same results, lower bandwidth).
 *   rows, n  rows == 0 or n == 0 is a successful no-op.
 *   stream   a hipStream_t passed as void* (NULL = the default stream).  Work is
 *            enqueued and the call returns; nothing is synchronised and nothing
 *            is copied to the host.  The caller keeps x and y alive until the
 *            stream has finished.
 *   inputs   finite values.  Full accuracy (max relative error 4e-6 for fp32
 *            I/O) holds for |x| <= 1e5; see the Two-Pass entry for larger
 *            magnitudes.  A NaN anywhere in a row makes that row's outputs NaN, and
 *            so does an infinity of either sign (the range reduction turns it into
 *            NaN); other rows are not affected.  To mask an element out, give it a
 *            large finite negative value, not -inf.  The 16-bit entry points take the
 *            exponent from the bit pattern of x log2(e) + 1.5 * 2^23, which is valid
 *            for |x| < 2.9e6: every binary16 value, and bfloat16 values up to there.
 *   return   0 on success; a negative TP_ERR_* code for an invalid argument,
 *            detected before any GPU call is made; a positive value is the
 *            hipError_t of a failed allocation or launch.
 *   memory   long rows are cut into chunks whose partial results live in a small
 *            workspace owned by the library (a few KB to a few hundred KB per
 *            stream), allocated on first use and kept; softmax_tp_release()
 *            frees it.  The library allocates nothing else.
 *   threads  several host threads may call at once provided no two of them use the
 *            same stream at the same time (two calls interleaved on one stream would
 *            share that stream's workspace).  softmax_tp_release must not run concurrently
 *            with any other call; for softmax_tp_tune see there.
 */
#ifndef SOFTMAX_TP_H
#define SOFTMAX_TP_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TP_API __attribute__((visibility("default")))

#define TP_OK 0
#define TP_ERR_NULL (-1)      /* x or y is NULL while rows * n > 0 (or an out-pointer is NULL) */
#define TP_ERR_NEGATIVE (-2)  /* rows < 0 or n < 0 */
#define TP_ERR_TOO_LARGE (-3) /* rows * n * element size overflows, or rows / chunks exceed the grid limit */
#define TP_ERR_ALIGN (-4)     /* a pointer is not aligned to the element size */
#define TP_ERR_TUNING (-5)    /* unknown tuning key or value out of range */
#define TP_ERR_SCRATCH (-6)   /* softmax2p_f32_static: the shape needs more than TP_STATIC_SCRATCH_BYTES */

/*
 * Algorithm 3 (Section 4), fp32 in and out.  Pass 1 evaluates every e^x as a pair
 * (m, n) with e^x = m * 2^n (ExtExp: Algorithm 4 of Section 6.3 without its
 * reconstruction step) and reduces the pairs of a row to one (m_sum, n_sum),
 * always rescaling to the larger exponent so nothing overflows; pass 2 recomputes
 * each pair and writes y = m * (1 / m_sum) * 2^(n - n_sum).  Reads x twice, writes
 * y once: 3 N elements of traffic (Table 2).
 * Beyond |x| = 1e5 the fp32 range reduction loses accuracy (the product
 * x * log2(e) is rounded to 24 bits); outputs stay finite up to |x| ~ 1e15.
 */
TP_API int softmax2p_f32(const float *x, float *y, int64_t rows, int64_t n, void *stream);

/*
 * Algorithm 1 (Section 3): mu = max x; sigma = sum Exp(x - mu); y = Exp(x - mu) / sigma,
 * with Exp recomputed in the last pass.  3 reads + 1 write per element (Table 2).
 */
TP_API int softmax3p_recompute_f32(const float *x, float *y, int64_t rows, int64_t n, void *stream);

/*
 * Algorithm 2 (Section 3): as Algorithm 1, but the second pass stores Exp(x - mu) in y
 * and the third rescales y in place.  3 reads + 2 writes per element (Table 2).
 */
TP_API int softmax3p_reload_f32(const float *x, float *y, int64_t rows, int64_t n, void *stream);

/*
 * Algorithm 3 with bfloat16 storage: x and y hold bf16 bit patterns; each element
 * is widened to fp32, the pair arithmetic is the fp32 one of softmax2p_f32, and
 * y is rounded to bf16 (nearest even).  Not in the paper, which is fp32 only
 * (Section 6.3); target accuracy 1e-2 relative against the unrounded result.
 */
TP_API int softmax2p_bf16io(const uint16_t *x, uint16_t *y, int64_t rows, int64_t n, void *stream);

/*
 * Algorithms 1 and 2 with bfloat16 storage, as baselines for softmax2p_bf16io: same
 * widening / rounding as there.  In the reloading variant y holds Exp(x - mu) rounded to
 * bf16 between the second and the third pass (sigma is accumulated from the unrounded
 * fp32 values), so its result carries two bf16 roundings.
 */
TP_API int softmax3p_recompute_bf16io(const uint16_t *x, uint16_t *y, int64_t rows, int64_t n,
                                      void *stream);
TP_API int softmax3p_reload_bf16io(const uint16_t *x, uint16_t *y, int64_t rows, int64_t n,
                                   void *stream);

/*
 * Algorithms 3, 1 and 2 with IEEE binary16 storage: x and y hold fp16 bit patterns, widened
 * to fp32 exactly (subnormal inputs included) and rounded to fp16 (nearest even) on the
 * way out; the arithmetic between is the fp32 one of the *_f32 entry points.  Not in the
 * paper, which is fp32 only (Section 6.3).  fp16 has 11 significand bits and a narrow
 * exponent range: results below 2^-14 come out as fp16 subnormals (absolute error at most
 * 2^-25) and results below 2^-25 as zero, which is where this format stops being useful
 * for rows of many millions of comparable elements.  Target accuracy against the unrounded
 * result: 5e-4 relative for results of at least 2^-14 (1.1e-3 for the reloading variant,
 * whose y holds Exp(x - mu) rounded to fp16 between its second and third pass).
 */
TP_API int softmax2p_f16io(const uint16_t *x, uint16_t *y, int64_t rows, int64_t n, void *stream);
TP_API int softmax3p_recompute_f16io(const uint16_t *x, uint16_t *y, int64_t rows, int64_t n,
                                     void *stream);
TP_API int softmax3p_reload_f16io(const uint16_t *x, uint16_t *y, int64_t rows, int64_t n,
                                  void *stream);

/*
 * On-chip variant of Algorithm 3 for short rows (n <= TP_ONCHIP_MAX_N): a workgroup
 * loads its row into registers, runs pass 1 on them, keeps every element as its mantissa
 * scaled to a group exponent (the (m, n) pairs of Section 4 with one n per group of 8 or 16
 * elements), and pass 2 multiplies by lambda * 2^(n_group - n_sum) and writes y.  Same
 * results as softmax2p_f32 / _bf16io / _f16io up to rounding order, but x is read from memory
 * only once (2 N elements of traffic instead of 3 N) and ExtExp is evaluated once per element:
 * the regime in which, as the paper notes
 * (Sections 6.4 and 7), the Two-Pass algorithm has no bandwidth advantage left to offer.
 * Kept as an entry point of its own so that its throughput is never mistaken for the
 * three-traversal algorithm's.  x and y must be congruent modulo 16 bytes
 * (TP_ERR_ALIGN otherwise); longer rows give TP_ERR_TOO_LARGE.  Rows of at most 9 fp32 or 16
 * 16-bit elements are handled by one lane each with the kernels of softmax2p_* (of
 * softmax3p_recompute_* for the softmax3p_onchip_* entry points): the lane re-reads, and
 * re-evaluates, the one or two cache lines it has just read, so memory traffic is the same.
 */
#define TP_ONCHIP_MAX_N 32768
TP_API int softmax2p_onchip_f32(const float *x, float *y, int64_t rows, int64_t n, void *stream);
TP_API int softmax2p_onchip_bf16io(const uint16_t *x, uint16_t *y, int64_t rows, int64_t n,
                                   void *stream);
TP_API int softmax2p_onchip_f16io(const uint16_t *x, uint16_t *y, int64_t rows, int64_t n,
                                  void *stream);

/*
 * The same on-chip arrangement for Algorithm 2 (Section 3): max, Exp(x - mu) held in
 * registers where the algorithm holds it in Y, sum, rescale, store.  One exponential per
 * element, so this is the cheapest of all variants when rows fit on chip: the paper's
 * finding for in-cache data (Section 6.4), kept here as the honest baseline of
 * softmax2p_onchip_*.  Same limits and error codes.
 */
TP_API int softmax3p_onchip_f32(const float *x, float *y, int64_t rows, int64_t n, void *stream);
TP_API int softmax3p_onchip_bf16io(const uint16_t *x, uint16_t *y, int64_t rows, int64_t n,
                                   void *stream);
TP_API int softmax3p_onchip_f16io(const uint16_t *x, uint16_t *y, int64_t rows, int64_t n,
                                  void *stream);

/*
 * softmax2p_f32 for callers that cannot allocate: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same kernels, launch plan and results (bit for bit)
 * as softmax2p_f32, but the chunk path's partial results (one 8-byte pair per chunk, plus one
 * per row when a merge launch is planned) go to a fixed array of TP_STATIC_SCRATCH_BYTES that
 * is part of the library's device code instead of the allocated workspace: the call makes no
 * hipMalloc / hipFree, no memset, no synchronisation, needs no softmax_tp_reserve, and its
 * first call on a device only looks the array's address up.  Each GPU the library runs on
 * holds that array until the process ends.
 * A shape whose partial results do not fit returns TP_ERR_SCRATCH before anything is
 * launched.  It fits when rows * (reduce.chunks + 1) <= 32768 (softmax_tp_plan reports
 * reduce.chunks): with the default tuning that is every chunk-path input of up to 32768 rows
 * of at most 1 GiB each; the one-workgroup-per-row path needs no scratch at any row count.
 * All calls on one GPU share the array, whatever their stream: two calls whose execution
 * overlaps on one GPU race on it and give wrong results.  Calls that follow one another
 * on one stream are safe, and nothing needs clearing between them: every slot a call reads it
 * has written itself first.
 */
#define TP_STATIC_SCRATCH_BYTES (256 * 1024)
TP_API int softmax2p_f32_static(const float *x, float *y, int64_t rows, int64_t n, void *stream);

/* ----- pieces of the path, exported for tests and for per-pass timing ----- */

/*
 * ExtExp alone (Section 4): m[i], e[i] = pair of x[i] for i < count, e an
 * integer-valued float.  x, m, e are device pointers to `count` floats.
 */
TP_API int softmax_tp_extexp_f32(const float *x, float *m, float *e, int64_t count, void *stream);

/*
 * The same pairs from the other evaluator Section 4 allows for the reduced argument: base-2
 * reduction with a two-term log2 e and the hardware's 2^f instruction instead of the
 * polynomial.  Same e[i] as softmax_tp_extexp_f32, m[i] within 1 ULP or so of it.  Not used
 * by the softmax entry points (it is not faster on this part); here for comparison.
 */
TP_API int softmax_tp_extexp_hw_f32(const float *x, float *m, float *e, int64_t count,
                                    void *stream);

/*
 * Pass 1 of Algorithm 3 including every merge level: pairs[2 r] = m_sum and
 * pairs[2 r + 1] = n_sum of row r.  pairs is a device pointer to 2 * rows floats.
 */
TP_API int softmax2p_f32_pass1(const float *x, float *pairs, int64_t rows, int64_t n, void *stream);

/*
 * Pass 2 of Algorithm 3 given the per-row pairs produced by softmax2p_f32_pass1.
 */
TP_API int softmax2p_f32_pass2(const float *x, const float *pairs, float *y, int64_t rows, int64_t n,
                        void *stream);

/*
 * Bandwidth calibration in the manner of the STREAM comparison of Section 6.4,
 * using the same streaming code as the softmax passes: read `count` floats
 * (their sum goes to sink[0], a device float), copy y = x, scale y = a * x, and a
 * write-only stream y = value (a pass that reads and writes takes as long as the read-only
 * and the write-only stream of its size together, so both ceilings are worth knowing).
 */
TP_API int softmax_tp_stream_read_f32(const float *x, float *sink, int64_t count, void *stream);
TP_API int softmax_tp_stream_fill_f32(float *y, float value, int64_t count, void *stream);
TP_API int softmax_tp_stream_copy_f32(const float *x, float *y, int64_t count, void *stream);
TP_API int softmax_tp_stream_scale_f32(const float *x, float *y, float a, int64_t count, void *stream);

/* ----- planning, workspace, tuning (host side) ----- */

typedef struct {
    int32_t block;      /* threads per workgroup; on the rows path 1, 4, 16 or 64 stand for that many
                           lanes per row, several rows sharing a workgroup of 256 threads */
    int32_t unroll;     /* 16-byte loads in flight per thread */
    int64_t chunk_vecs; /* 16-byte vectors per workgroup (0 on the rows path: the whole row) */
    int64_t chunks;     /* workgroups per row */
} softmax_tp_shape_t;

typedef struct {
    int32_t path;          /* 1: one workgroup per row, every pass in a single launch;
                              2: rows cut into chunks, one launch per pass + small merge launches */
    int32_t vector_elems;  /* elements per access: 4 (fp32) / 8 (16-bit), or 1 when x and y are not
                              congruent modulo 16 bytes, and for rows of at most 9 fp32 / 16 16-bit
                              elements (one lane per row) whose length is not a multiple of 16 bytes;
                              a call also uses 1 for such rows if x itself is not 16-byte aligned */
    int32_t launches;      /* kernel launches of the Two-Pass call */
    int32_t merge_kernel;  /* path 2: 1 if a row has more than 128 chunk partials, which a small
                              kernel of its own then merges; 0 if the next pass folds them itself */
    int32_t nt_first_load; /* path 2: 1 if even the first read of x carries the non-temporal hint
                              (input too large for any cache to help the second read) */
    softmax_tp_shape_t rows;    /* path 1, Two-Pass */
    softmax_tp_shape_t rows_recompute; /* path 1, Three-Pass with recomputation */
    softmax_tp_shape_t rows_reload;    /* path 1, Three-Pass with reloading */
    softmax_tp_shape_t reduce;  /* path 2, read-only passes (Two-Pass pass 1; max; sum-exp) */
    softmax_tp_shape_t map;     /* path 2, read-write passes (Two-Pass pass 2; exp-scale; scale) */
    softmax_tp_shape_t mapsum;  /* path 2, the read-write pass that also reduces (exp-store) */
    int64_t workspace_bytes;
} softmax_tp_plan_t;

/*
 * The launch plan the library would use.  elem_bytes is 4 or 2; congruent16 says
 * whether x and y are congruent modulo 16 bytes.  Pure host logic: no GPU needed.
 */
TP_API int softmax_tp_plan(int64_t rows, int64_t n, int32_t elem_bytes, int32_t congruent16,
                           softmax_tp_plan_t *plan);

/*
 * Overrides a planner parameter (for sweeps).  Keys:
 *   "path"            0 auto, 1 rows path, 2 chunk path
 *   "block_rows", "unroll_rows"          shape on the rows path
 *   "block_reduce", "unroll_reduce", "target_reduce"  read-only passes: shape and the
 *                     number of workgroups aimed for over the whole launch
 *   "block_map", "unroll_map", "tiles_map"  read-write passes: shape and tiles
 *                     (block * unroll vectors) per workgroup
 *   "block_mapsum", "unroll_mapsum", "tiles_mapsum"  the same for the exp-store pass
 *   "direction"       1 (default): every pass walks memory forwards; 2: successive
 *                     passes alternate direction
 *   "nt_first"        1: first read of x cacheable; 2: non-temporal; default: by size
 *   "fold_max"        most partial results per row that a consuming pass folds by itself;
 *                     more than that go through a merge kernel first (at most 4096)
 *   "nt_store"        rows on groups of 4 or 16 lanes: 1 stores y without the non-temporal
 *                     hint, 2 with it; default: without it for rows under 1 KiB (on-chip entry
 *                     points: under 128 bytes) whose length neither divides nor is a multiple
 *                     of 128 bytes, so that neighbouring rows share cache lines unevenly
 *   "scalar_io"       1: element-wise accesses even where x and y would allow 16-byte vectors
 * block is 256, 512 or 1024; unroll 2, 4 or 8 (16-bit formats: 2 or 4); in addition the
 * pair block 128, unroll 1.  "block_rows" also takes 1, 4, 16 or 64: a group of that many lanes
 * per row, several rows per workgroup (what rows of at most 256 vectors get by default), with
 * "unroll_rows" 1 to 4; the on-chip entry points follow such a "block_rows" for rows that fit
 * four vectors per lane.  value 0 restores the default.  May be called while other threads plan or launch (each call reads the settings
 * under a lock and sees every key either before or after the change), but a call that
 * overlaps a retune may mix old and new keys: retune between calls when that matters.
 */
TP_API int softmax_tp_tune(const char *key, int64_t value);

/*
 * Allocates (or grows) the workspace a later softmax call with this shape on this stream
 * would need, so that the call itself does not allocate: the largest any entry point asks for
 * with this shape, whether or not x and y are congruent modulo 16 bytes, the pass-level entry
 * points included.  Shapes on the rows path need none.  After it, a softmax call on that
 * stream consists of kernel launches only (no allocation, no memset, no host
 * synchronisation) and can be captured into a HIP graph and replayed.
 * A stream has one workspace.  A call (or reserve) that needs more than the stream holds
 * frees the old buffer, which waits for the device, and allocates a larger one: a graph
 * captured earlier on that stream still points at the freed buffer and must be captured
 * again.  Reserve the largest shape first, or capture after the last reserve.
 */
TP_API int softmax_tp_reserve(int64_t rows, int64_t n, int32_t elem_bytes, void *stream);

/* Frees every workspace the library holds (synchronises the device). */
TP_API int softmax_tp_release(void);

/* Text for a return code of this library (negative codes; positive ones are HIP's). */
TP_API const char *softmax_tp_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif
