// Tolerance ladder and error-aware speedup scores (host side).
#pragma once
#include "pf.h"

namespace pf {

// atol(t), rtol(t) of the paper's Appendix F for a storage dtype; t > 0 uses t = 0.
void tolerance_at(pf_dtype dtype, int t, double* rtol, double* atol);
// ES_t for t = -10 .. 4 and AS (paper Eq. 2-4, weights of Appendix E).
void aggregate(const pf_case* cases, int n, double b, double p, pf_metrics* out);
double fast_p(const pf_case* cases, int n, double threshold, int t);

}  // namespace pf
