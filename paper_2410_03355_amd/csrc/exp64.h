// exp(d) for d <= 0 in fp64: argument reduction by ln 2 in two pieces
// (Cody-Waite) and the degree-13 Taylor polynomial on |r| <= ln(2)/2, whose
// truncation error is below 2^-57; the result is within one ulp of libm.
// Branch-free.  The same source compiles for the device and, for testing
// against libm, for the host.
#pragma once

#include <math.h>

#if defined(__HIPCC__)
#define LANTERN_HD __host__ __device__ __forceinline__
#else
#define LANTERN_HD inline
#endif

namespace lantern {

// One Horner step acc*r + c.  On the device the constant stays in a scalar
// register pair and the step is a single v_fma_f64 (the compiler otherwise
// copies the constant into the accumulator register first).
LANTERN_HD double horner_step(double acc, double r, double c) {
#if defined(__HIP_DEVICE_COMPILE__)
    double out;
    asm("v_fma_f64 %0, %1, %2, %3" : "=v"(out) : "v"(acc), "v"(r), "s"(c));
    return out;
#else
    return __builtin_fma(acc, r, c);
#endif
}

// d <= 0, or -inf (result 0).  Arguments below -1000, and NaN, give 0.
LANTERN_HD double exp_nonpos(double d) {
    const double LOG2E = 1.4426950408889634074;          // 1/ln 2
    const double LN2_HI = 6.93147180369123816490e-01;    // ln 2 with the low 21 mantissa bits zero
    const double LN2_LO = 1.90821492927058770002e-10;    // ln 2 - LN2_HI
    d = fmax(d, -1000.0);                                 // 2^-1443 scales to exactly 0 below
    const double n = __builtin_rint(d * LOG2E);
    double r = __builtin_fma(-n, LN2_HI, d);
    r = __builtin_fma(-n, LN2_LO, r);
    double p = 1.6059043836821614599e-10;                 // 1/13!
    p = horner_step(p, r, 2.0876756987868098979e-09);     // 1/12!
    p = horner_step(p, r, 2.5052108385441718775e-08);     // 1/11!
    p = horner_step(p, r, 2.7557319223985890653e-07);     // 1/10!
    p = horner_step(p, r, 2.7557319223985892511e-06);     // 1/9!
    p = horner_step(p, r, 2.4801587301587301566e-05);     // 1/8!
    p = horner_step(p, r, 1.9841269841269841253e-04);     // 1/7!
    p = horner_step(p, r, 1.3888888888888889419e-03);     // 1/6!
    p = horner_step(p, r, 8.3333333333333332177e-03);     // 1/5!
    p = horner_step(p, r, 4.1666666666666664354e-02);     // 1/4!
    p = horner_step(p, r, 1.6666666666666665741e-01);     // 1/3!
    p = __builtin_fma(p, r, 0.5);
    p = __builtin_fma(p, r, 1.0);
    p = __builtin_fma(p, r, 1.0);
    return ldexp(p, (int)n);
}

// exp(d) for d in [-1000, 700] from a table of 2^(j/128): d = (128 n + j) ln2/128 + r with
// |r| <= ln2/256, exp(d) = 2^n * T[j] * e^r.  The reduction multiplies the integer 128 n + j
// (below 2^18 in magnitude) by a 32-bit piece of ln2/128, which is exact, and by the remainder;
// e^r - 1 is the degree-5 Taylor polynomial (truncation below 6e-19); the table entry is a pair
// hi + lo, so the result is within 0.6 ulp of the exact value: within one ulp of libm.  Half the
// arithmetic of exp_nonpos.  tab: EXP_TABLE_HILO, on the device a copy of it in LDS.
// Arguments below -1000, and NaN, give 0.  Branch-free.
LANTERN_HD double exp_poly5(double r) {                     // e^r - 1 for |r| <= ln2/256
    double q = __builtin_fma(r, 8.3333333333333332177e-03, 4.1666666666666664354e-02);   // 1/5!, 1/4!
    q = __builtin_fma(q, r, 1.6666666666666665741e-01);                                  // 1/3!
    q = __builtin_fma(q, r, 0.5);
    q = __builtin_fma(q, r, 1.0);
    return q * r;
}

LANTERN_HD double exp_tab(double d, const double* tab) {
    const double INV_STEP = 184.6649652337873;             // 128 / ln 2
    const double STEP_HI = 0x1.62e42fee00000p-8;           // ln2/128 with the low 21 mantissa bits zero
    const double STEP_LO = 0x1.a39ef35793c76p-40;          // ln2/128 - STEP_HI
    d = fmin(fmax(d, -1000.0), 700.0);
    const double m = __builtin_rint(d * INV_STEP);
    double r = __builtin_fma(-m, STEP_HI, d);
    r = __builtin_fma(-m, STEP_LO, r);
    const int mi = (int)m;
    const int j = mi & 127;
    const int n = mi >> 7;                                  // floor division: j >= 0
    const double hi = tab[2 * j], lo = tab[2 * j + 1];
    const double p = exp_poly5(r);                          // e^r - 1
    const double res = hi + __builtin_fma(hi, p, lo);
    return ldexp(res, n);
}

// exp_tab for arguments known to lie in [-700, 700], with fewer instructions: the rounding to an
// integer is one fused multiply-add onto 1.5 * 2^52 (the integer then sits in the low word of
// the sum), and the scaling by 2^n is an integer addition to the exponent field (the result
// stays a normal number on this range).  Same reduction, table and polynomial as exp_tab: the
// same value.  The caller clamps; outside the range the result is meaningless.
// tab_bytes: the table as bytes (on the device an LDS address: placed at offset 0 of the
// workgroup's LDS, the lookup's address is the masked integer itself).
LANTERN_HD double exp_tab_core(double d, const unsigned char* tab_bytes) {
    const double INV_STEP = 184.6649652337873;
    const double STEP_HI = 0x1.62e42fee00000p-8;
    const double STEP_LO = 0x1.a39ef35793c76p-40;
    const double MAGIC = 6755399441055744.0;               // 1.5 * 2^52
    const double t = __builtin_fma(d, INV_STEP, MAGIC);
    unsigned long long tb;
    __builtin_memcpy(&tb, &t, 8);
    const unsigned mi = (unsigned)tb;                       // low word: the rounded integer, two's complement
    const double m = t - MAGIC;
    double r = __builtin_fma(-m, STEP_HI, d);
    r = __builtin_fma(-m, STEP_LO, r);
    const double* entry = reinterpret_cast<const double*>(tab_bytes + ((mi & 127u) << 4));
    const double hi = entry[0], lo = entry[1];
    const double p = exp_poly5(r);
    const double res = hi + __builtin_fma(hi, p, lo);
    unsigned long long rb;
    __builtin_memcpy(&rb, &res, 8);
    // n = mi >> 7 (arithmetic) into the exponent field: bits 52.. of the double, 20.. of its high word
    const unsigned hi_word = (unsigned)(rb >> 32) + ((mi & ~127u) << 13);
    rb = ((unsigned long long)hi_word << 32) | (unsigned)rb;
    double out;
    __builtin_memcpy(&out, &rb, 8);
    return out;
}

}  // namespace lantern
