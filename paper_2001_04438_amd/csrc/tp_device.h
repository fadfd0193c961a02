// Device-side building blocks of the softmax kernels (gfx950, wave64).
//
//  * pair arithmetic for the (m, n) representation of Section 4,
//  * wave / workgroup reductions (DPP inside a row of 16 lanes, v_readlane across
//    the four rows, LDS across waves),
//  * 128-bit coalesced streaming of a row segment with scalar handling of the few
//    elements before / after the 16-byte-aligned body of a row.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "extexp.h"

namespace tp {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));

constexpr int kWave = 64;
constexpr int kMaxWaves = 16;

// Exponent of the additive identity pair (0, -inf) of Algorithm 3.  A finite
// stand-in is used so that two identities can meet in a tree reduction without
// producing (-inf) - (-inf) = NaN; it is below every exponent the evaluator can
// return for a finite input, and its mantissa is 0 so it never contributes.
constexpr float kNIdent = -3.402823466e38f;

// float -> int32 with saturation (v_cvt_i32_f32 saturates and maps NaN to 0; a C
// cast would be undefined for the huge negative differences that occur when an
// identity pair is rescaled).
__device__ __forceinline__ int cvt_i32_sat(float f)
{
    int r;
    asm("v_cvt_i32_f32 %0, %1" : "=v"(r) : "v"(f));
    return r;
}

// m * 2^dn for an integer-valued float dn <= 0 (Algorithm 3: values are only
// ever scaled down).  v_ldexp_f32 returns 0 once the result underflows.
__device__ __forceinline__ float scale_pow2(float m, float dn)
{
    return __builtin_ldexpf(m, cvt_i32_sat(dn));
}

// Exp of Algorithm 4 for a non-positive argument: ExtExp followed by the
// reconstruction p * 2^n (the v_ldexp_f32 analogue of the VSCALEFPS step).
__device__ __forceinline__ float exp_nonpos(float d)
{
    float m, n;
    tp_extexp(d, &m, &n);
    return scale_pow2(m, n);
}

// ---- the same for the evaluator whose exponent is the bit pattern of z (extexp.h) ----

// Saturating 32-bit subtraction / addition (v_sub_i32 / v_add_i32 with clamp): differences of
// exponent bit patterns never wrap, whatever the input, so a scale factor is never positive
// by accident.
__device__ __forceinline__ int sub_sat(int a, int b) { return __builtin_elementwise_sub_sat(a, b); }
__device__ __forceinline__ int add_sat(int a, int b) { return __builtin_elementwise_add_sat(a, b); }

// Bit pattern standing for the exponent of the additive identity: below that of every z.
constexpr int kZIdent = -0x40000000;

__device__ __forceinline__ float exp_nonpos_bits(float d)
{
    float m, z;
    tp_extexp_bits(d, &m, &z);
    return __builtin_ldexpf(m, sub_sat(tp_float_bits(z), TP_MAGIC_BITS));
}

template <bool INT_EXP>
__device__ __forceinline__ float exp_nonpos_as(float d)
{
    if constexpr (INT_EXP)
        return exp_nonpos_bits(d);
    else
        return exp_nonpos(d);
}

// ---------------------------------------------------------------------------
// wave-level reductions
// ---------------------------------------------------------------------------

template <int CTRL>
__device__ __forceinline__ float dpp(float v)
{
    return __builtin_bit_cast(
        float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, false));
}

__device__ __forceinline__ float lane_value(float v, int lane)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), lane));
}

// DPP controls: quad_perm [1,0,3,2], quad_perm [2,3,0,1], row_half_mirror, row_mirror.
// After the four steps every lane of a 16-lane row holds the row's result.
#define TP_ROW_BUTTERFLY(v, OP)      \
    v = OP(v, dpp<0xB1>(v));         \
    v = OP(v, dpp<0x4E>(v));         \
    v = OP(v, dpp<0x141>(v));        \
    v = OP(v, dpp<0x140>(v));

__device__ __forceinline__ float op_max(float a, float b) { return fmaxf(a, b); }
__device__ __forceinline__ float op_add(float a, float b) { return a + b; }

__device__ __forceinline__ float wave_max(float v)
{
    TP_ROW_BUTTERFLY(v, op_max)
    return fmaxf(fmaxf(lane_value(v, 0), lane_value(v, 16)),
                 fmaxf(lane_value(v, 32), lane_value(v, 48)));
}

__device__ __forceinline__ float wave_sum(float v)
{
    TP_ROW_BUTTERFLY(v, op_add)
    return (lane_value(v, 0) + lane_value(v, 16)) + (lane_value(v, 32) + lane_value(v, 48));
}

// 64 pairs -> one: wave maximum of the exponents, each lane rescales its mantissa
// to it, wave sum of the mantissas: 63 pair additions of Algorithm 3 done as a tree.
__device__ __forceinline__ void wave_pair(float &m, float &n)
{
    float nw = wave_max(n);
    m = wave_sum(scale_pow2(m, n - nw));
    n = nw;
}

// The same reductions over a group of LANES lanes, every group of the wave on its own:
// LANES = 64 (the wave), 16 (a DPP row: the four butterfly steps, no cross-row step) or 4 (a
// quad: the first two steps).
template <int LANES>
__device__ __forceinline__ float lanes_max(float v)
{
    static_assert(LANES == 64 || LANES == 16 || LANES == 4 || LANES == 1, "a wave, a row of 16 lanes, a quad or a lane");
    if constexpr (LANES == 1) {
        return v;
    } else if constexpr (LANES == 64) {
        return wave_max(v);
    } else {
        v = fmaxf(v, dpp<0xB1>(v));
        v = fmaxf(v, dpp<0x4E>(v));
        if constexpr (LANES == 16) {
            v = fmaxf(v, dpp<0x141>(v));
            v = fmaxf(v, dpp<0x140>(v));
        }
        return v;
    }
}

template <int LANES>
__device__ __forceinline__ float lanes_sum(float v)
{
    static_assert(LANES == 64 || LANES == 16 || LANES == 4 || LANES == 1, "a wave, a row of 16 lanes, a quad or a lane");
    if constexpr (LANES == 1) {
        return v;
    } else if constexpr (LANES == 64) {
        return wave_sum(v);
    } else {
        v += dpp<0xB1>(v);
        v += dpp<0x4E>(v);
        if constexpr (LANES == 16) {
            v += dpp<0x141>(v);
            v += dpp<0x140>(v);
        }
        return v;
    }
}

template <int LANES>
__device__ __forceinline__ void lanes_pair(float &m, float &n)
{
    const float nw = lanes_max<LANES>(n);
    m = lanes_sum<LANES>(scale_pow2(m, n - nw));
    n = nw;
}

// A row's partial results folded by every wave on its own: lane i takes partials i,
// i + 64, ... in that order, then the wave reduction.  No LDS, no barrier, and every wave of
// every workgroup gets the bit-identical value.  The partials are read by all the waves of a
// launch, so the host sends more than a hundred or so through a merge kernel first.
__device__ __forceinline__ void wave_fold_pairs(const float2 *p, int cnt, float &m, float &n)
{
    const int lane = threadIdx.x & (kWave - 1);
    m = 0.f;
    n = kNIdent;
    for (int k = lane; k < cnt; k += kWave) {
        const float2 q = p[k];
        const float nn = fmaxf(n, q.y);
        m = scale_pow2(m, n - nn) + scale_pow2(q.x, q.y - nn);
        n = nn;
    }
    wave_pair(m, n);
}

__device__ __forceinline__ float wave_fold_max(const float *p, int cnt)
{
    const int lane = threadIdx.x & (kWave - 1);
    float v = -__builtin_inff();
    for (int k = lane; k < cnt; k += kWave)
        v = fmaxf(v, p[k]);
    return wave_max(v);
}

__device__ __forceinline__ float wave_fold_sum(const float *p, int cnt)
{
    const int lane = threadIdx.x & (kWave - 1);
    float v = 0.f;
    for (int k = lane; k < cnt; k += kWave)
        v += p[k];
    return wave_sum(v);
}

// ---------------------------------------------------------------------------
// workgroup-level reductions (result returned to every thread)
// ---------------------------------------------------------------------------

// Stage 1: wave reduction; stage 2: lane w of every wave picks up wave w's result from
// LDS and the wave reduces again, so all waves end up with the same bits and only a
// couple of registers are live across the barrier.

template <int BLOCK>
__device__ __forceinline__ float block_max(float v, float *lds)
{
    constexpr int W = BLOCK / kWave;
    v = wave_max(v);
    if constexpr (W == 1)
        return v;
    __syncthreads();  // lds may still be read by an earlier reduction
    if ((threadIdx.x & (kWave - 1)) == 0)
        lds[threadIdx.x / kWave] = v;
    __syncthreads();
    const int lane = threadIdx.x & (kWave - 1);
    return wave_max(lane < W ? lds[lane] : -__builtin_inff());
}

template <int BLOCK>
__device__ __forceinline__ float block_sum(float v, float *lds)
{
    constexpr int W = BLOCK / kWave;
    v = wave_sum(v);
    if constexpr (W == 1)
        return v;
    __syncthreads();
    if ((threadIdx.x & (kWave - 1)) == 0)
        lds[threadIdx.x / kWave] = v;
    __syncthreads();
    const int lane = threadIdx.x & (kWave - 1);
    return wave_sum(lane < W ? lds[lane] : 0.f);
}

template <int BLOCK>
__device__ __forceinline__ void block_pair(float &m, float &n, float *lds)
{
    constexpr int W = BLOCK / kWave;
    wave_pair(m, n);
    if constexpr (W == 1)
        return;
    __syncthreads();
    if ((threadIdx.x & (kWave - 1)) == 0) {
        lds[threadIdx.x / kWave] = m;
        lds[kMaxWaves + threadIdx.x / kWave] = n;
    }
    __syncthreads();
    const int lane = threadIdx.x & (kWave - 1);
    m = lane < W ? lds[lane] : 0.f;
    n = lane < W ? lds[kMaxWaves + lane] : kNIdent;
    wave_pair(m, n);
}

// ---------------------------------------------------------------------------
// element formats: how 16 bytes (or one element) become floats and back
// ---------------------------------------------------------------------------

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __builtin_bit_cast(float, w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w)
{
    return __builtin_bit_cast(float, w & 0xFFFF0000u);
}
__device__ __forceinline__ uint32_t bf16_pack(float lo, float hi)  // round to nearest even
{
    f32x2 p = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(p, bf16x2));
}

struct F32x4 {  // fp32, 16-byte vectors
    static constexpr bool kIntExp = false;  // which ExtExp evaluator: see extexp.h
    using elem = float;
    using vec = f32x4;
    static constexpr int V = 4;
    static __device__ __forceinline__ void unpack(vec v, float *o)
    {
        o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w;
    }
    static __device__ __forceinline__ vec pack(const float *o)
    {
        vec v = {o[0], o[1], o[2], o[3]};
        return v;
    }
    static __device__ __forceinline__ float load1(const elem *p) { return *p; }
    static __device__ __forceinline__ void store1(elem *p, float v) { *p = v; }
    static __device__ __forceinline__ vec zero() { vec v = {0.f, 0.f, 0.f, 0.f}; return v; }
};

struct F32x1 {  // fp32, element-wise (x and y not congruent modulo 16 bytes)
    static constexpr bool kIntExp = false;  // which ExtExp evaluator: see extexp.h
    using elem = float;
    using vec = float;
    static constexpr int V = 1;
    static __device__ __forceinline__ void unpack(vec v, float *o) { o[0] = v; }
    static __device__ __forceinline__ vec pack(const float *o) { return o[0]; }
    static __device__ __forceinline__ float load1(const elem *p) { return *p; }
    static __device__ __forceinline__ void store1(elem *p, float v) { *p = v; }
    static __device__ __forceinline__ vec zero() { return 0.f; }
};

struct BF16x8 {  // bf16 in and out, 16-byte vectors, fp32 arithmetic
    static constexpr bool kIntExp = true;  // which ExtExp evaluator: see extexp.h
    using elem = uint16_t;
    using vec = u32x4;
    static constexpr int V = 8;
    static __device__ __forceinline__ void unpack(vec v, float *o)
    {
        o[0] = bf16_lo(v.x); o[1] = bf16_hi(v.x); o[2] = bf16_lo(v.y); o[3] = bf16_hi(v.y);
        o[4] = bf16_lo(v.z); o[5] = bf16_hi(v.z); o[6] = bf16_lo(v.w); o[7] = bf16_hi(v.w);
    }
    static __device__ __forceinline__ vec pack(const float *o)
    {
        vec v = {bf16_pack(o[0], o[1]), bf16_pack(o[2], o[3]), bf16_pack(o[4], o[5]),
                 bf16_pack(o[6], o[7])};
        return v;
    }
    static __device__ __forceinline__ float load1(const elem *p)
    {
        return __builtin_bit_cast(float, (uint32_t)(*p) << 16);
    }
    static __device__ __forceinline__ void store1(elem *p, float v)
    {
        *p = (uint16_t)(bf16_pack(v, 0.f) & 0xFFFFu);
    }
    static __device__ __forceinline__ vec zero() { vec v = {0u, 0u, 0u, 0u}; return v; }
};

struct BF16x1 {  // bf16, element-wise
    static constexpr bool kIntExp = true;  // which ExtExp evaluator: see extexp.h
    using elem = uint16_t;
    using vec = uint16_t;
    static constexpr int V = 1;
    static __device__ __forceinline__ void unpack(vec v, float *o)
    {
        o[0] = __builtin_bit_cast(float, (uint32_t)v << 16);
    }
    static __device__ __forceinline__ vec pack(const float *o)
    {
        return (uint16_t)(bf16_pack(o[0], 0.f) & 0xFFFFu);
    }
    static __device__ __forceinline__ float load1(const elem *p) { return BF16x8::load1(p); }
    static __device__ __forceinline__ void store1(elem *p, float v) { BF16x8::store1(p, v); }
    static __device__ __forceinline__ vec zero() { return 0; }
};

// IEEE binary16 widens to fp32 exactly (its subnormals too: the conversion instructions
// honour them in the default floating-point mode) and narrows with round to nearest even.
__device__ __forceinline__ void f16_unpack(uint32_t w, float &lo, float &hi)
{
    const f32x2 p = __builtin_convertvector(__builtin_bit_cast(f16x2, w), f32x2);
    lo = p.x;
    hi = p.y;
}
__device__ __forceinline__ uint32_t f16_pack(float lo, float hi)
{
    f32x2 p = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(p, f16x2));
}

struct F16x8 {  // fp16 in and out, 16-byte vectors, fp32 arithmetic
    static constexpr bool kIntExp = true;  // which ExtExp evaluator: see extexp.h
    using elem = uint16_t;
    using vec = u32x4;
    static constexpr int V = 8;
    static __device__ __forceinline__ void unpack(vec v, float *o)
    {
        f16_unpack(v.x, o[0], o[1]);
        f16_unpack(v.y, o[2], o[3]);
        f16_unpack(v.z, o[4], o[5]);
        f16_unpack(v.w, o[6], o[7]);
    }
    static __device__ __forceinline__ vec pack(const float *o)
    {
        vec v = {f16_pack(o[0], o[1]), f16_pack(o[2], o[3]), f16_pack(o[4], o[5]),
                 f16_pack(o[6], o[7])};
        return v;
    }
    static __device__ __forceinline__ float load1(const elem *p)
    {
        return (float)__builtin_bit_cast(_Float16, *p);
    }
    static __device__ __forceinline__ void store1(elem *p, float v)
    {
        *p = __builtin_bit_cast(uint16_t, (_Float16)v);
    }
    static __device__ __forceinline__ vec zero() { vec v = {0u, 0u, 0u, 0u}; return v; }
};

struct F16x1 {  // fp16, element-wise
    static constexpr bool kIntExp = true;  // which ExtExp evaluator: see extexp.h
    using elem = uint16_t;
    using vec = uint16_t;
    static constexpr int V = 1;
    static __device__ __forceinline__ void unpack(vec v, float *o)
    {
        o[0] = (float)__builtin_bit_cast(_Float16, v);
    }
    static __device__ __forceinline__ vec pack(const float *o)
    {
        return __builtin_bit_cast(uint16_t, (_Float16)o[0]);
    }
    static __device__ __forceinline__ float load1(const elem *p) { return F16x8::load1(p); }
    static __device__ __forceinline__ void store1(elem *p, float v) { F16x8::store1(p, v); }
    static __device__ __forceinline__ vec zero() { return 0; }
};

// ---------------------------------------------------------------------------
// the part of one row that one workgroup streams
// ---------------------------------------------------------------------------
//
// A row starts `a` elements past a 16-byte boundary.  Vector j of the row's frame
// holds row elements [j V - a, j V - a + V); vectors jlo..jhi-1 lie wholly inside
// the row and are moved with 128-bit accesses.  The at most V-1 elements before
// and V-1 after them (or the whole row when it holds no full vector) are "edge"
// elements handled one per lane.  x and y must be congruent modulo 16 bytes for
// the vector formats; the host picks the element-wise formats otherwise.

template <class IO>
struct Seg {
    const typename IO::vec *xv;  // frame vector 0 of the row in x (16-byte aligned)
    typename IO::vec *yv;        // the same for y
    const typename IO::elem *xrow;
    typename IO::elem *yrow;
    int64_t vb;     // first frame vector of this workgroup
    uint32_t cnt;   // number of vectors of this workgroup (< 2^31 / 16)
    int head;       // edge elements [0, head) ...
    int64_t tail0;  // ... and [tail0, n), if `edges`
    int64_t n;
    bool edges;
};

template <class IO>
__device__ __forceinline__ Seg<IO> make_seg(const typename IO::elem *x, typename IO::elem *y,
                                            int64_t n, int64_t row, int64_t chunk,
                                            int64_t chunk_vecs)
{
    using elem = typename IO::elem;
    constexpr int V = IO::V;
    Seg<IO> s;
    s.xrow = x + row * n;
    s.yrow = y ? y + row * n : nullptr;
    s.n = n;
    const int a = (int)(((uintptr_t)s.xrow / sizeof(elem)) % V);
    const int64_t jlo = a ? 1 : 0;
    int64_t jhi = (a + n) / V;
    if (jhi < jlo)
        jhi = jlo;
    s.head = a ? (int)(n < (int64_t)(V - a) ? n : (int64_t)(V - a)) : 0;
    s.tail0 = jhi > jlo ? jhi * V - a : (int64_t)s.head;
    // plain pointer arithmetic (no integer round trip) so the compiler keeps treating these
    // as global-memory pointers and emits global_load / global_store, not flat accesses
    s.xv = reinterpret_cast<const typename IO::vec *>(s.xrow - a);
    s.yv = y ? reinterpret_cast<typename IO::vec *>(s.yrow - a) : nullptr;
    int64_t vb = jlo + chunk * chunk_vecs;
    int64_t ve = vb + chunk_vecs;
    if (vb > jhi) vb = jhi;
    if (ve > jhi) ve = jhi;
    s.vb = vb;
    s.cnt = (uint32_t)(ve - vb);
    s.edges = chunk == 0;
    return s;
}

// True if the predicate holds in every active lane of the wave.
__device__ __forceinline__ bool wave_all(bool p)
{
    return __builtin_amdgcn_ballot_w64(p) == __builtin_amdgcn_ballot_w64(true);
}

template <bool NT, class VEC>
__device__ __forceinline__ VEC ld(const VEC *p)
{
    if constexpr (NT)
        return __builtin_nontemporal_load(p);
    else
        return *p;
}

template <bool NT, class VEC>
__device__ __forceinline__ void st(VEC *p, VEC v)
{
    if constexpr (NT)
        __builtin_nontemporal_store(v, p);
    else
        *p = v;
}

// Streams a segment through policy P.  Each thread keeps U independent 16-byte
// loads in flight; consecutive lanes touch consecutive vectors, so one wave
// instruction moves 1 KiB contiguously.  P provides
//     static constexpr bool kWrite;
//     template <int G> void group(const float *f, float *o);
// which consumes G elements (and, if kWrite, produces G outputs).  Full rounds
// hand over G = U*V elements at once; the last, partly filled round hands over
// the vectors that exist one at a time.
// `tid` is the thread's index among the BLOCK threads that share the segment (the
// workgroup by default; a single wave when one wave owns a row).
template <class IO, int BLOCK, int U, bool NT_LOAD, bool NT_STORE, class P>
__device__ __forceinline__ void stream(const Seg<IO> &s, P &p, uint32_t tid = threadIdx.x)
{
    using vec = typename IO::vec;
    constexpr int V = IO::V;
    constexpr int G = U * V;
    const vec *xb = s.xv + s.vb;
    vec *yb = s.yv + s.vb;
    const uint32_t cnt = s.cnt;
    uint32_t k = tid;
    // Lane groups (BLOCK <= 64, several rows per wave): full rounds as long as every lane of the
    // wave has one.  A wave whose lanes disagree would run this loop body for some and the partly
    // filled round below for the others, one after the other, and with a few rounds per row that
    // is most of the time.  When the vote fails a lane has at most U vectors left (the lanes of a
    // wave are in the same round, and rows that share a wave differ by at most one vector).
    // Workgroups decide per lane: only the wave that holds the end of the row ever disagrees, and
    // the vote in the loop cost the arithmetic-heavy read-only passes 2 %.
    auto full_round = [&](uint32_t at) {
        const bool mine = at + (uint32_t)((U - 1) * BLOCK) < cnt;
        if constexpr (BLOCK <= 64)
            return wave_all(mine);
        else
            return mine;
    };
    for (; full_round(k); k += (uint32_t)(U * BLOCK)) {
        vec v[U];
#pragma unroll
        for (int u = 0; u < U; ++u)
            v[u] = ld<NT_LOAD>(xb + (k + (uint32_t)(u * BLOCK)));
        float f[G], o[G];
#pragma unroll
        for (int u = 0; u < U; ++u)
            IO::unpack(v[u], f + u * V);
        p.template group<G>(f, o);
        if constexpr (P::kWrite) {
#pragma unroll
            for (int u = 0; u < U; ++u)
                st<NT_STORE>(yb + (k + (uint32_t)(u * BLOCK)), IO::pack(o + u * V));
        }
    }
    if (k < cnt) {  // last, partly filled round of this thread
        vec v[U];
        bool ok[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            ok[u] = k + (uint32_t)(u * BLOCK) < cnt;
            v[u] = ok[u] ? ld<NT_LOAD>(xb + (k + (uint32_t)(u * BLOCK))) : IO::zero();
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (ok[u]) {
                float f[V], o[V];
                IO::unpack(v[u], f);
                p.template group<V>(f, o);
                if constexpr (P::kWrite)
                    st<NT_STORE>(yb + (k + (uint32_t)(u * BLOCK)), IO::pack(o));
            }
        }
    }
    if (s.edges) {  // at most 2 (V - 1) elements: one round, except for lane groups of four
        const int nedge = s.head + (int)(s.n - s.tail0);
        for (int e = (int)tid; e < nedge; e += BLOCK) {
            const int64_t i = e < s.head ? (int64_t)e : s.tail0 + (e - s.head);
            float f = IO::load1(s.xrow + i), o;
            p.template group<1>(&f, &o);
            if constexpr (P::kWrite)
                IO::store1(s.yrow + i, o);
        }
    }
}

// ---------------------------------------------------------------------------
// policies: what happens to each element in a pass
// ---------------------------------------------------------------------------

template <int G>
__device__ __forceinline__ float tree_sum(float *v)
{
#pragma unroll
    for (int w = 1; w < G; w *= 2)
#pragma unroll
        for (int i = 0; i + w < G; i += 2 * w)
            v[i] += v[i + w];
    return v[0];
}

// Two-Pass, pass 1 (Algorithm 3): accumulate ExtExp pairs.  A whole group is
// brought to the largest exponent among the group and the running sum, then added.
struct PairSum {
    static constexpr bool kWrite = false;
    float m = 0.f, n = kNIdent;
    // If `e` is given, the group's mantissas are left there scaled to the exponent `n` holds
    // after the call.
    template <int G>
    __device__ __forceinline__ void group(const float *f, float *e)
    {
        float mi[G], ni[G];
        float nmax = n;
#pragma unroll
        for (int i = 0; i < G; ++i) {
            tp_extexp(f[i], &mi[i], &ni[i]);
            nmax = fmaxf(nmax, ni[i]);
        }
        float acc = scale_pow2(m, n - nmax);
#pragma unroll
        for (int i = 0; i < G; ++i) {
            mi[i] = scale_pow2(mi[i], ni[i] - nmax);
            if (e)
                e[i] = mi[i];
        }
        m = acc + tree_sum<G>(mi);
        n = nmax;
    }
    __device__ __forceinline__ void finish(float &m_out, float &n_out) const
    {
        m_out = m;
        n_out = n;
    }
    // For a caller that keeps the scaled mantissas of a group: the exponent they were scaled
    // to, and the factor that takes them from there to lambda * 2^(that exponent - n_sum).
    using token = float;
    __device__ __forceinline__ token exponent() const { return n; }
    static __device__ __forceinline__ float factor(float lambda, token g, float n_sum)
    {
        return scale_pow2(lambda, g - n_sum);
    }
};

// The same on the integer-exponent evaluator (16-bit storage formats): the running exponent
// is the bit pattern of z, the group maximum an integer maximum, and each rescale one integer
// subtraction and one v_ldexp_f32.  If `e` is given, the group's mantissas are left there
// scaled to the exponent in `z` after the call, for a caller that keeps them.
struct PairSumI {
    static constexpr bool kWrite = false;
    float m = 0.f;
    int z = kZIdent;
    template <int G>
    __device__ __forceinline__ void group(const float *f, float *e)
    {
        float mi[G], zf[G];
        int zmax = z;
#pragma unroll
        for (int i = 0; i < G; ++i) {
            tp_extexp_bits(f[i], &mi[i], &zf[i]);
            zmax = max(zmax, tp_float_bits(zf[i]));
        }
        const float acc = __builtin_ldexpf(m, sub_sat(z, zmax));
#pragma unroll
        for (int i = 0; i < G; ++i) {
            mi[i] = __builtin_ldexpf(mi[i], sub_sat(tp_float_bits(zf[i]), zmax));
            if (e)
                e[i] = mi[i];
        }
        m = acc + tree_sum<G>(mi);
        z = zmax;
    }
    // the pair in the float form every merge level above the thread works on
    __device__ __forceinline__ void finish(float &m_out, float &n_out) const
    {
        m_out = m;
        n_out = (float)sub_sat(z, TP_MAGIC_BITS);
    }
    using token = int;
    __device__ __forceinline__ token exponent() const { return z; }
    static __device__ __forceinline__ float factor(float lambda, token g, float n_sum)
    {
        return __builtin_ldexpf(lambda, sub_sat(g, add_sat(TP_MAGIC_BITS, cvt_i32_sat(n_sum))));
    }
};

// Two-Pass, pass 2: Y_i = m_i * lambda * 2^(n_i - n_sum).  lambda is folded into the
// polynomial's coefficients once per thread, so m_i * lambda comes out of the Horner chain.
struct PairOut {
    static constexpr bool kWrite = true;
    float cs[6];
    float n_sum;
    __device__ __forceinline__ PairOut(float lambda, float n_sum_) : n_sum(n_sum_)
    {
        tp_scale_coeffs(lambda, cs);
    }
    template <int G>
    __device__ __forceinline__ void group(const float *f, float *o)
    {
#pragma unroll
        for (int i = 0; i < G; ++i) {
            float ml, ni;
            tp_extexp_scaled(f[i], cs, &ml, &ni);
            o[i] = scale_pow2(ml, ni - n_sum);
        }
    }
};

struct PairOutI {
    static constexpr bool kWrite = true;
    float cs[6];
    int k;  // the bit pattern z would have for n = n_sum
    __device__ __forceinline__ PairOutI(float lambda, float n_sum)
        : k(add_sat(TP_MAGIC_BITS, cvt_i32_sat(n_sum)))
    {
        tp_scale_coeffs(lambda, cs);
    }
    template <int G>
    __device__ __forceinline__ void group(const float *f, float *o)
    {
#pragma unroll
        for (int i = 0; i < G; ++i) {
            float ml, z;
            tp_extexp_bits_scaled(f[i], cs, &ml, &z);
            o[i] = __builtin_ldexpf(ml, sub_sat(tp_float_bits(z), k));
        }
    }
};

template <class IO>
using PairSumOf = std::conditional_t<IO::kIntExp, PairSumI, PairSum>;
template <class IO>
using PairOutOf = std::conditional_t<IO::kIntExp, PairOutI, PairOut>;

// Three-Pass, pass 1: running maximum.
struct MaxOf {
    static constexpr bool kWrite = false;
    float mx = -__builtin_inff();
    template <int G>
    __device__ __forceinline__ void group(const float *f, float *)
    {
#pragma unroll
        for (int i = 0; i < G; ++i)
            mx = fmaxf(mx, f[i]);
    }
};

// Three-Pass (recompute), pass 2: sigma += Exp(x - mu).  INT_EXP picks the evaluator (all
// three-pass policies): both families always share one, as in the paper (Section 6.3).
template <bool INT_EXP>
struct SumExp {
    static constexpr bool kWrite = false;
    float mu;
    float s = 0.f;
    template <int G>
    __device__ __forceinline__ void group(const float *f, float *)
    {
        float e[G];
#pragma unroll
        for (int i = 0; i < G; ++i)
            e[i] = exp_nonpos_as<INT_EXP>(f[i] - mu);
        s += tree_sum<G>(e);
    }
};

// Three-Pass (recompute), pass 3: Y_i = lambda * Exp(x - mu), lambda folded into the
// polynomial as in PairOut so both families pay the same per element.
template <bool INT_EXP>
struct ExpScale {
    static constexpr bool kWrite = true;
    float cs[6];
    float mu;
    __device__ __forceinline__ ExpScale(float mu_, float lambda) : mu(mu_)
    {
        tp_scale_coeffs(lambda, cs);
    }
    template <int G>
    __device__ __forceinline__ void group(const float *f, float *o)
    {
#pragma unroll
        for (int i = 0; i < G; ++i) {
            if constexpr (INT_EXP) {
                float ml, z;
                tp_extexp_bits_scaled(f[i] - mu, cs, &ml, &z);
                o[i] = __builtin_ldexpf(ml, sub_sat(tp_float_bits(z), TP_MAGIC_BITS));
            } else {
                float ml, ni;
                tp_extexp_scaled(f[i] - mu, cs, &ml, &ni);
                o[i] = scale_pow2(ml, ni);
            }
        }
    }
};

// Three-Pass (reload), pass 2: Y_i = Exp(x - mu), sigma += Y_i.
template <bool INT_EXP>
struct ExpStoreSum {
    static constexpr bool kWrite = true;
    float mu;
    float s = 0.f;
    template <int G>
    __device__ __forceinline__ void group(const float *f, float *o)
    {
        float e[G];
#pragma unroll
        for (int i = 0; i < G; ++i)
            e[i] = o[i] = exp_nonpos_as<INT_EXP>(f[i] - mu);
        s += tree_sum<G>(e);
    }
};

// Three-Pass (reload), pass 3 and the STREAM-Scale calibration: Y_i = lambda * Y_i.
struct Scale {
    static constexpr bool kWrite = true;
    float lambda;
    template <int G>
    __device__ __forceinline__ void group(const float *f, float *o)
    {
#pragma unroll
        for (int i = 0; i < G; ++i)
            o[i] = lambda * f[i];
    }
};

// Calibration: plain sum (read-only stream) and copy.
struct SumOf {
    static constexpr bool kWrite = false;
    float s = 0.f;
    template <int G>
    __device__ __forceinline__ void group(const float *f, float *)
    {
        float e[G];
#pragma unroll
        for (int i = 0; i < G; ++i)
            e[i] = f[i];
        s += tree_sum<G>(e);
    }
};

struct Copy {
    static constexpr bool kWrite = true;
    template <int G>
    __device__ __forceinline__ void group(const float *f, float *o)
    {
#pragma unroll
        for (int i = 0; i < G; ++i)
            o[i] = f[i];
    }
};

}  // namespace tp
