// Tolerance ladder and error-aware speedup scores.
//
// Paper Sec. 3.4: per-subgraph rectified speedup (Eq. 2), its geometric mean
// ES_t (Eq. 3) and the weighted geometric mean AS over the tolerance index
// t = -10 .. |E|+1 (Eq. 4, weights in Appendix E); Appendix F gives atol(t) and
// rtol(t) as 10^(k t) per dtype.  |E| = 3 error categories: accuracy 1,
// compilation 2, runtime 3.  For t <= 0 a subgraph is correct when it ran and
// no element violates the tolerance of index t; for t > 0 the numerical test
// of t = 0 applies and error categories c <= t are forgiven.
#include "metric.h"

#include <cmath>

#include "pf_internal.h"

namespace pf {

void tolerance_at(pf_dtype dtype, int t, double* rtol, double* atol) {
    if (t > 0) t = 0;
    double kr, ka;
    switch (dtype) {
        case PF_BF16: kr = 1.796 / 5.0; ka = 1.0; break;
        case PF_F16: kr = 3.0 / 5.0; ka = 1.0; break;
        case PF_F32: kr = 5.886 / 5.0; ka = 1.0; break;
        case PF_F64: kr = 7.0 / 5.0; ka = 7.0 / 5.0; break;
        default: fail(PF_E_INVALID, "no tolerance table for dtype %d", (int)dtype);
    }
    *rtol = std::pow(10.0, kr * t);
    *atol = std::pow(10.0, ka * t);
}

namespace {

constexpr int kTMin = -10, kTMax = 4;

double weight(int t) {
    if (t <= -6 || t >= 4) return 0.001;
    if (t <= -3) return 1.0;
    return std::pow(0.8, t + 3);
}

bool correct_at(const pf_case& c, int t) {
    if (c.error_class != 0) return false;
    const int level = (t > 0 ? 0 : t) - kTMin;
    return c.n_viol[level] == 0;
}

double rectified(const pf_case& c, int t, double b, double p) {
    if (correct_at(c, t)) return c.speedup >= 1.0 ? c.speedup : std::pow(c.speedup, p + 1.0);
    const int cat = c.error_class != 0 ? c.error_class : 1;
    return t < cat ? b : 1.0;
}

}  // namespace

void aggregate(const pf_case* cases, int n, double b, double p, pf_metrics* out) {
    if (!(b > 0.0)) fail(PF_E_INVALID, "base penalty b must be positive");
    for (int i = 0; i < n; ++i) {
        if (cases[i].error_class != 0 && (cases[i].error_class < 2 || cases[i].error_class > 3))
            fail(PF_E_INVALID, "case %d: error_class must be 0, 2 or 3", i);
        if (cases[i].error_class == 0 && !(cases[i].speedup > 0.0)) fail(PF_E_INVALID, "case %d: speedup must be positive", i);
    }
    double wsum = 0.0, acc = 0.0;
    for (int t = kTMin; t <= kTMax; ++t) {
        double logsum = 0.0;
        for (int i = 0; i < n; ++i) logsum += std::log(rectified(cases[i], t, b, p));
        const double es = std::exp(logsum / n);
        out->es[t - kTMin] = es;
        wsum += weight(t);
        acc += weight(t) * (logsum / n);
    }
    out->as = std::exp(acc / wsum);
}

double fast_p(const pf_case* cases, int n, double threshold, int t) {
    int hit = 0;
    for (int i = 0; i < n; ++i) hit += correct_at(cases[i], t) && cases[i].speedup > threshold;
    return (double)hit / n;
}

}  // namespace pf
