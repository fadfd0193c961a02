// ExtExp: e^x as a (mantissa, exponent) pair, and Exp with reconstruction.
//
// Section 4 keeps e^x = m * 2^n as the pair (m, n) by dropping the reconstruction
// step of Algorithm 4 (Section 6.3): n = round(x log2 e), t = x - n ln 2 by a
// two-constant Cody-Waite reduction, m = 1 + t (c1 + t (c2 + t (c3 + t (c4 + t c5))))
// in Horner form with fused multiply-adds.  n is an integer held in a float.
// Both softmax families use this same reduction and polynomial (Section 6.3, last
// paragraph).
//
// The functions are plain scalar code: hipcc compiles them for gfx950
// (v_rndne_f32, v_fma_f32); a host C compiler can include the file as well so the
// arithmetic can be swept exhaustively against libm without a GPU.
#pragma once
#include "expconst.h"

#if defined(__HIPCC__)
#define TP_FN __host__ __device__ __forceinline__
#else
#define TP_FN static inline
#endif

TP_FN void tp_extexp(float x, float *m, float *n)
{
    float nn = __builtin_rintf(x * TP_LOG2E);        // round to nearest, ties to even
    float t = __builtin_fmaf(nn, -TP_LN2_HI, x);     // product exact inside the FMA
    t = __builtin_fmaf(nn, -TP_LN2_LO, t);
    float p = __builtin_fmaf(TP_EXP_C5, t, TP_EXP_C4);
    p = __builtin_fmaf(p, t, TP_EXP_C3);
    p = __builtin_fmaf(p, t, TP_EXP_C2);
    p = __builtin_fmaf(p, t, TP_EXP_C1);
    p = __builtin_fmaf(p, t, 1.0f);
    *m = p;
    *n = nn;
}

// The same evaluation with the polynomial pre-multiplied by a factor s: cs[0] = s and
// cs[k] = fl(c_k * s), so the Horner chain ends in s * m instead of m at no extra cost per
// element.  Pass 2 of Algorithm 3 uses it with s = lambda_sum = 1 / m_sum; the 2^(n - n_sum)
// factor is applied afterwards.  Costs one rounding per coefficient (about 0.3 ULP in all).
TP_FN void tp_scale_coeffs(float s, float *cs)
{
    cs[0] = s;
    cs[1] = TP_EXP_C1 * s;
    cs[2] = TP_EXP_C2 * s;
    cs[3] = TP_EXP_C3 * s;
    cs[4] = TP_EXP_C4 * s;
    cs[5] = TP_EXP_C5 * s;
}

TP_FN void tp_extexp_scaled(float x, const float *cs, float *ms, float *n)
{
    float nn = __builtin_rintf(x * TP_LOG2E);
    float t = __builtin_fmaf(nn, -TP_LN2_HI, x);
    t = __builtin_fmaf(nn, -TP_LN2_LO, t);
    float p = __builtin_fmaf(cs[5], t, cs[4]);
    p = __builtin_fmaf(p, t, cs[3]);
    p = __builtin_fmaf(p, t, cs[2]);
    p = __builtin_fmaf(p, t, cs[1]);
    p = __builtin_fmaf(p, t, cs[0]);
    *ms = p;
    *n = nn;
}

// ---------------------------------------------------------------------------------------
// The evaluator of the 16-bit storage formats: same steps, exponent taken as an integer.
//
// Rows of bf16 / fp16 elements are bound by vector instructions, not by memory, so every
// instruction per element counts.  Two changes to the evaluation above, neither to its steps:
//
//  * n comes out of the rounding itself.  z = fl(x log2 e + 1.5 * 2^23) is an integer for
//    |x log2 e| < 2^22 (the addition rounds to nearest even at unit spacing), n = z - 1.5 * 2^23
//    is exact, and the low mantissa bits of z hold n in two's complement: the bit pattern of z
//    minus that of another such z is the difference of the two exponents.  This is the
//    exponent-field reconstruction that Section 6.3 describes for AVX2, taken one step
//    earlier; the float -> integer conversion per element goes away, and the multiply and the
//    rounding become one fused multiply-add and one subtraction.  The price is the range:
//    |x| < 2^22 ln 2 = 2.9e6, which binary16 cannot exceed (bfloat16 can: beyond it results are
//    meaningless, as they already are beyond 1e5 for want of accuracy in x log2 e).
//  * the reduction t = x - n ln 2 uses the single constant fl(ln 2).  What is left out,
//    n * TP_LN2_LO, multiplies e^x by e^(n * 1.9e-9): a softmax output only sees
//    e^((n_i - n_sum) * 1.9e-9), and an output that is not flushed to zero has
//    |n_i - n_sum| < 150, so the cost is below 2.9e-7 relative, against 4.9e-4 (binary16) or
//    3.9e-3 (bfloat16) for the rounding of the output itself.
#define TP_MAGIC 12582912.0f   /* 1.5 * 2^23 */
#define TP_MAGIC_BITS 0x4B400000

TP_FN int tp_float_bits(float f)
{
    int i;
    __builtin_memcpy(&i, &f, sizeof i);
    return i;
}

// z of the first bullet above (its bit pattern carries n) and the mantissa m.
TP_FN void tp_extexp_bits(float x, float *m, float *z)
{
    float zz = __builtin_fmaf(x, TP_LOG2E, TP_MAGIC);
    float nn = zz - TP_MAGIC;
    float t = __builtin_fmaf(nn, -TP_LN2_HI, x);
    float p = __builtin_fmaf(TP_EXP_C5, t, TP_EXP_C4);
    p = __builtin_fmaf(p, t, TP_EXP_C3);
    p = __builtin_fmaf(p, t, TP_EXP_C2);
    p = __builtin_fmaf(p, t, TP_EXP_C1);
    p = __builtin_fmaf(p, t, 1.0f);
    *m = p;
    *z = zz;
}

// The same with the polynomial pre-multiplied by a factor (cs from tp_scale_coeffs).
TP_FN void tp_extexp_bits_scaled(float x, const float *cs, float *ms, float *z)
{
    float zz = __builtin_fmaf(x, TP_LOG2E, TP_MAGIC);
    float nn = zz - TP_MAGIC;
    float t = __builtin_fmaf(nn, -TP_LN2_HI, x);
    float p = __builtin_fmaf(cs[5], t, cs[4]);
    p = __builtin_fmaf(p, t, cs[3]);
    p = __builtin_fmaf(p, t, cs[2]);
    p = __builtin_fmaf(p, t, cs[1]);
    p = __builtin_fmaf(p, t, cs[0]);
    *ms = p;
    *z = zz;
}

#if defined(__HIPCC__)
// The alternative the paper leaves open for step 2 of the exponential (Section 4: the
// function on the reduced argument may also come from a table or another approximation):
// reduce in base 2, f = x log2 e - n with log2 e split in two fp32 terms (the first product
// is exact inside the FMA), and take 2^f from the hardware's v_exp_f32.  Same n as
// tp_extexp, so the two are interchangeable per element.  Built into the softmax kernels it
// gained 2-3 % on rows of 16-bit elements, which are bound by vector instructions, nothing
// on fp32 and cost the on-chip fp32 kernel its register budget, so the kernels keep the
// polynomial; this evaluator stays exported on its own for the accuracy test.
__device__ __forceinline__ void tp_extexp_hw(float x, float *m, float *n)
{
    float nn = __builtin_rintf(x * TP_LOG2E);
    float f = __builtin_fmaf(x, TP_LOG2E, -nn);
    f = __builtin_fmaf(x, TP_LOG2E_LO, f);
    *m = __builtin_amdgcn_exp2f(f);
    *n = nn;
}
#endif
