// q8_math.h -- sigmoid, tanh and exp of the float parts of the model (Section 3 keeps them in
// floating point): each is evaluated in double to about 1e-15 relative accuracy and rounded
// once to float, so the float result is the correctly rounded one except for arguments
// whose exact value lies within ~1e-15 (relative) of a rounding boundary.  Plain fma / add /
// divide only, the same on the host and on the device (but for how the quotient is formed, see
// q8_div_pos); no library calls on the device.
#pragma once

#include <math.h>

#if defined(__HIPCC__)
#define Q8_MATH_FN __host__ __device__ __forceinline__
#else
#define Q8_MATH_FN static inline
#endif

// a / b for finite a >= 0 and b in [1, 2^120].  On the host: a / b.  On the device the compiler's
// division is twelve instructions, five of them operand scaling and special cases that cannot
// occur here and two a second Newton step; this form keeps the hardware's reciprocal estimate, one
// Newton step and the correction of the quotient by its exact residual.  With y = (1 + e) / b the
// corrected quotient is (a / b)(1 - e^2) before its one rounding: e is below 2^-40 after the
// Newton step even for an estimate good to 20 bits only, so the result is within 0.5 ulp + 2^-80
// of a / b, far inside the 1e-15 these functions promise; on the GPU the float results of tanh and
// sigmoid equal the host's on every sample tried (tests/test_gpu_device_math.py).
Q8_MATH_FN double q8_div_pos(double a, double b)
{
#if defined(__HIP_DEVICE_COMPILE__)
    double y = __builtin_amdgcn_rcp(b);
    y = fma(fma(-b, y, 1.0), y, y);
    const double q = a * y;
    return fma(fma(-b, q, a), y, q);
#else
    return a / b;
#endif
}

// exp(r) - 1 for |r| <= ln 2 / 2 as r (1 + r h(r)), h a polynomial of degree 9 that interpolates
// (expm1(r) / r - 1) / r at the Chebyshev points of the interval (near-minimax: in exact arithmetic the
// result is within 4.1e-17 relative of expm1(r), below the rounding of the evaluation itself; the
// Taylor polynomial needs three more terms for that).  The constant term 1 is exact, so the result
// keeps its relative accuracy down to r = 0.
Q8_MATH_FN double q8_expm1_small(double r)
{
    double p = 2.51003758422236995e-08;
    p = fma(p, r, 2.76200758925481640e-07);
    p = fma(p, r, 2.75572684802897162e-06);
    p = fma(p, r, 2.48015213223422815e-05);
    p = fma(p, r, 1.98412698630405585e-04);
    p = fma(p, r, 1.38888889171967359e-03);
    p = fma(p, r, 8.33333333333006500e-03);
    p = fma(p, r, 4.16666666666241636e-02);
    p = fma(p, r, 1.66666666666666685e-01);
    p = fma(p, r, 5.00000000000000111e-01);
    p = fma(p, r, 1.0);
    return p * r;
}

// Splits y (|y| <= 700) as y = k ln 2 + r with k integral and |r| <= 0.347; returns r.
Q8_MATH_FN double q8_reduce_ln2(double y, int *k_out)
{
    const double k = rint(y * 1.44269504088896338700e+00);
    double r = fma(k, -6.93147180369123816490e-01, y);       // high part of ln 2: 32 significant bits, k times it is exact
    r = fma(k, -1.90821492927058770002e-10, r);
    *k_out = (int)k;
    return r;
}

// exp(y) in double for |y| <= 700 (callers clamp).
Q8_MATH_FN double q8_exp_d(double y)
{
    int k;
    const double r = q8_reduce_ln2(y, &k);
    return ldexp(1.0 + q8_expm1_small(r), k);
}

// tanh(a) = (e^{2|a|} - 1) / (e^{2|a|} + 1) with the sign of a.  With e^{y} = 2^k (1 + m),
// m = expm1(r), the numerator is 2^k m + (2^k - 1), which keeps full accuracy for small |a|.
Q8_MATH_FN float q8_tanh_rn(float a)
{
    const double x = (double)a;
    const double y = fmin(2.0 * fabs(x), 80.0);               // tanh is 1 to double precision long before
    int k;
    const double r = q8_reduce_ln2(y, &k);
    const double m = q8_expm1_small(r);
    const double s = ldexp(1.0, k);
    const double num = fma(s, m, s - 1.0);
    const double t = q8_div_pos(num, num + 2.0);
    return (float)copysign(t, x);
}

// sigmoid(a) = 1 / (1 + e^{-a}); with E = e^{-|a|} in (0, 1]: 1 / (1 + E) for a >= 0, E / (1 + E) below.
Q8_MATH_FN float q8_sigmoid_rn(float a)
{
    const double x = (double)a;
    const double E = q8_exp_d(-fmin(fabs(x), 700.0));
    const double num = x >= 0.0 ? 1.0 : E;
    return (float)q8_div_pos(num, 1.0 + E);
}
