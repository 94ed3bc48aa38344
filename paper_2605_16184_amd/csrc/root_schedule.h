// Coefficients of the coupled inverse p-th root iteration  T = a I - g M,  X <- X T,  M <- T^p M.
//
// Every eigenvalue mu of M moves by the scalar map f(mu) = (a - g mu)^p mu.  The classical
// Newton choice a = (p + 1) / p, g = 1 / p grows a small eigenvalue by only ((p + 1) / p)^p per
// step (2.44 for p = 4).  When the spectrum of M is known to lie in [lo, hi] the pair (a, g) can
// instead be chosen so that f maps the whole interval as close to 1 as possible: write
// f(mu) = g^p (c - mu)^p mu with c = a / g (the zero of T); the minimax choice equalises
// f(lo) = f(hi) = 1 - E and f(c / (p + 1)) = 1 + E (the interior maximum), which has the closed
// form below.  c is kept >= (1 + theta) hi so that T stays safely positive definite even if hi
// was underestimated.  As the interval contracts to {1} the pair tends to the Newton pair.
// The same routine runs on the host (iteration budget, precision switch) and on the device
// (per-factor coefficients).
#pragma once
#include <math.h>

#ifdef __HIPCC__
#define ASTERIA_HD __host__ __device__
#else
#define ASTERIA_HD
#endif

namespace asteria {

struct RootInterval { double lo, hi; };

ASTERIA_HD inline double ipow(double x, int p)
{
    double r = 1.0;
    for (int i = 0; i < p; ++i) r *= x;
    return r;
}

// (a, g) for a spectrum in [lo, hi]; adapted = false gives the classical Newton pair.
ASTERIA_HD inline void root_coefficients(double lo, double hi, int p, bool adapted, double theta,
                                         double &a, double &g)
{
    a = (p + 1.0) / p;
    g = 1.0 / p;
    if (!adapted || !(lo > 0.0) || !(hi > lo)) return;
    const double rho = pow(hi / lo, 1.0 / p);
    if (!(rho > 1.0 + 1e-9)) return;
    double c = (rho * hi - lo) / (rho - 1.0);
    if (c < hi * (1.0 + theta)) c = hi * (1.0 + theta);
    if (!(c < 1e6)) return;
    const double flo = ipow(c - lo, p) * lo, fhi = ipow(c - hi, p) * hi;
    double fmin = flo < fhi ? flo : fhi, fmax = flo > fhi ? flo : fhi;
    const double ms = c / (p + 1.0);
    if (ms > lo && ms < hi) {
        const double fm = ipow(c - ms, p) * ms;
        if (fm > fmax) fmax = fm;
        if (fm < fmin) fmin = fm;
    }
    g = pow(2.0 / (fmin + fmax), 1.0 / p);
    a = g * c;
}

// image of [lo, hi] under mu -> (a - g mu)^p mu
ASTERIA_HD inline RootInterval root_image(double lo, double hi, int p, double a, double g)
{
    const double flo = ipow(a - g * lo, p) * lo, fhi = ipow(a - g * hi, p) * hi;
    RootInterval r;
    r.lo = flo < fhi ? flo : fhi;
    r.hi = flo > fhi ? flo : fhi;
    const double ms = a / ((p + 1.0) * g);
    if (ms > lo && ms < hi) {
        const double fm = ipow(a - g * ms, p) * ms;
        if (fm > r.hi) r.hi = fm;
        if (fm < r.lo) r.lo = fm;
    }
    return r;
}

constexpr double ROOT_THETA = 0.1;   // safety margin of T's positivity: zero of T >= 1.1 hi

}  // namespace asteria
