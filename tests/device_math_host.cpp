// Host build of the device polynomial kernels, for error measurement against libm (long double).
#define PX_MATH_HOST 1
#include "../paper_2008_12260_amd/csrc/pollux_math.h"

#include <cmath>

static double ulp_err(double got, long double want)
{
    if (want == 0.0L) return got == 0.0 ? 0.0 : 1e300;
    int e;
    std::frexp((double)want, &e);
    long double ulp = std::ldexp(1.0L, e - 53);
    return (double)(std::fabs((long double)got - want) / ulp);
}

extern "C" {
// which: 0 exp, 1 log1p on [0,1], 2 log, 3 the whole last pass of Eq. 10 (x = T_grad, y = T_sync, g = gamma)
double px_host_eval(int which, double x, double y, double g)
{
    switch (which) {
        case 0: return px::px_exp(x);
        case 1: return px::px_log1p_unit(x);
        case 2: return px::px_log(x);
        default: {
            double d = px::px_log(x) - px::px_log(y);
            double e = px::px_exp(-g * std::fabs(d));
            return std::fmax(x, y) * px::px_exp(px::px_log1p_unit(e) * (1.0 / g));
        }
    }
}
double px_host_max_ulp(int which, const double *x, const double *y, const double *g, long n)
{
    double worst = 0.0;
    for (long i = 0; i < n; ++i) {
        long double want;
        if (which == 0) want = expl((long double)x[i]);
        else if (which == 1) want = log1pl((long double)x[i]);
        else if (which == 2) want = logl((long double)x[i]);
        else want = powl(powl((long double)x[i], (long double)g[i]) + powl((long double)y[i], (long double)g[i]),
                         1.0L / (long double)g[i]);
        double err = ulp_err(px_host_eval(which, x[i], which == 3 ? y[i] : 0.0, which == 3 ? g[i] : 1.0), want);
        if (err > worst) worst = err;
    }
    return worst;
}
}
