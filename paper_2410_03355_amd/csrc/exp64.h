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

}  // namespace lantern
