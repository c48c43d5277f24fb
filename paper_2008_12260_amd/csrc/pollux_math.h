// fp64 elementary functions for the last pass of Eq. 10 of the Pollux paper
// (arXiv 2008.12260, Sec. 3.2): T_iter(a, m, 0) = (T_grad^g + T_sync^g)^(1/g).
//
// gfx950 has no fp64 transcendental unit beyond v_rcp_f64, so exp and log are
// fused-multiply-add polynomial chains.  The kernel evaluates Eq. 10 with the
// larger term factored out,
//     big * exp( log1p( exp(-g * |ln T_grad - ln T_sync|) ) / g ),
// so the only arguments that occur are: exp of a non-positive number,
// log1p on [0, 1], and exp on [0, ln 2].  Each function below is accurate to
// about one unit in the last place on that domain.
//
// The file also compiles for the host (PX_MATH_HOST) so that the CPU test-suite
// can measure the error of exactly these polynomials against libm.
#pragma once

#if defined(PX_MATH_HOST)
#include <cmath>
#define PX_DEV inline
namespace px {
inline double px_fma(double a, double b, double c) { return std::fma(a, b, c); }
inline double px_rcp_seed(double x) { return (double)(1.0f / (float)x); }   // ~2^-23, like the hardware seed
inline double px_ldexp(double x, int k) { return std::ldexp(x, k); }
inline double px_rint(double x) { return std::nearbyint(x); }
}  // namespace px
#else
#include <hip/hip_runtime.h>
#define PX_DEV __device__ __forceinline__
namespace px {
PX_DEV double px_fma(double a, double b, double c) { return __builtin_fma(a, b, c); }
PX_DEV double px_rcp_seed(double x) { return __builtin_amdgcn_rcp(x); }             // v_rcp_f64
PX_DEV double px_ldexp(double x, int k) { return __builtin_amdgcn_ldexp(x, k); }    // v_ldexp_f64
PX_DEV double px_rint(double x) { return __builtin_rint(x); }                       // v_rndne_f64
}  // namespace px
#endif

namespace px {

// a / b for finite b != 0 well inside the exponent range: reciprocal seed, two
// Newton steps, one residual correction of the quotient.
PX_DEV double px_div(double a, double b)
{
    double r = px_rcp_seed(b);
    r = px_fma(px_fma(-b, r, 1.0), r, r);
    r = px_fma(px_fma(-b, r, 1.0), r, r);
    double q = a * r;
    return px_fma(px_fma(-b, q, a), r, q);
}

// exp(t) for t <= 1 (any negative t, -inf included): t = k ln2 + r, |r| <= ln2/2,
// Taylor polynomial of degree 13 in r (remainder below 2^-57), scaled by 2^k.
PX_DEV double px_exp(double t)
{
    t = t > -745.5 ? t : -745.5;                                   // exp underflows to 0 below this
    const double k = px_rint(t * 1.4426950408889634);              // log2(e)
    double r = px_fma(-k, 0.6931471805599453, t);                  // ln2 high part
    r = px_fma(-k, 2.3190468138462996e-17, r);                     // ln2 low part
    double p = 1.6059043836821613e-10;                             // 1/13!
    p = px_fma(p, r, 2.08767569878681e-09);                        // 1/12!
    p = px_fma(p, r, 2.505210838544172e-08);                       // 1/11!
    p = px_fma(p, r, 2.755731922398589e-07);                       // 1/10!
    p = px_fma(p, r, 2.7557319223985893e-06);                      // 1/9!
    p = px_fma(p, r, 2.48015873015873e-05);                        // 1/8!
    p = px_fma(p, r, 0.0001984126984126984);                       // 1/7!
    p = px_fma(p, r, 0.001388888888888889);                        // 1/6!
    p = px_fma(p, r, 0.008333333333333333);                        // 1/5!
    p = px_fma(p, r, 0.041666666666666664);                        // 1/4!
    p = px_fma(p, r, 0.16666666666666666);                         // 1/3!
    p = px_fma(p, r, 0.5);
    p = px_fma(p, r, 1.0);
    p = px_fma(p, r, 1.0);
    return px_ldexp(p, (int)k);
}

// 2 atanh(z) = log((1+z)/(1-z)) for |z| <= 0.1716 (z^2 <= 0.0295): odd series up to z^23.
PX_DEV double px_two_atanh(double z)
{
    const double w = z * z;
    double p = 0.08695652173913043;                                // 2/23
    p = px_fma(p, w, 0.09523809523809523);                         // 2/21
    p = px_fma(p, w, 0.10526315789473684);                         // 2/19
    p = px_fma(p, w, 0.11764705882352941);                         // 2/17
    p = px_fma(p, w, 0.13333333333333333);                         // 2/15
    p = px_fma(p, w, 0.15384615384615385);                         // 2/13
    p = px_fma(p, w, 0.18181818181818182);                         // 2/11
    p = px_fma(p, w, 0.2222222222222222);                          // 2/9
    p = px_fma(p, w, 0.2857142857142857);                          // 2/7
    p = px_fma(p, w, 0.4);                                         // 2/5
    p = px_fma(p, w, 0.6666666666666666);                          // 2/3
    return px_fma(z * w, p, z + z);
}

// log(1 + e) for 0 <= e <= 1.  For e > sqrt(2) - 1 the argument is halved first:
// log(1+e) = ln2 + log(1 + f), f = (e - 1)/2; in both cases log(1+f) = 2 atanh(f/(2+f)).
PX_DEV double px_log1p_unit(double e)
{
    const bool big = e > 0.41421356237309503;
    const double f = big ? (e - 1.0) * 0.5 : e;
    const double l = px_two_atanh(px_div(f, 2.0 + f));
    return big ? l + 0.6931471805599453 : l;
}

// log(x) for positive, finite, normal x.  x = 2^k * m with m in [sqrt(1/2), sqrt(2)).
PX_DEV double px_log(double x)
{
#if defined(PX_MATH_HOST)
    int k;
    double m = std::frexp(x, &k);
#else
    int k = __builtin_amdgcn_frexp_exp(x);
    double m = __builtin_amdgcn_frexp_mant(x);
#endif
    if (m < 0.7071067811865476) { m += m; k -= 1; }
    const double f = m - 1.0;
    const double l = px_two_atanh(px_div(f, 2.0 + f));
    const double kd = (double)k;
    return px_fma(kd, 0.6931471805599453, px_fma(kd, 2.3190468138462996e-17, l));
}

}  // namespace px
