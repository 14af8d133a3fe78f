// Checkpointing configuration model of Sec. V-C: the expected wasted GPU time T_w(f, b)
// (Eq. (10)), the interval f_c(b) at which it is stationary in f (Eq. (11)) and the discrete
// selection over candidate pairs (Eq. (12)). Host arithmetic only (a few flops per call): the
// costs it is fed - C_B(b), R_B(b), ... - are what the kernels of this library are measured for.
#include <math.h>

#include "ld_common.h"

namespace {
bool bad(double x) { return !(x == x) || x == HUGE_VAL || x == -HUGE_VAL; }
}  // namespace

extern "C" double ld_config_wasted_time(const ld_config_params* p, double f, double b, double R_B, double C_B) {
    if (!p || bad(f) || bad(b) || !(b >= 1.0) || !(f >= b) || !(p->tau > 0.0) || !(p->M > 0.0)) return NAN;
    const double failures = p->N * p->T / p->M;
    const double diffs_per_full = f / b - 1.0;
    const double lost = 0.5 * b * p->tau + p->R_F + 0.5 * R_B * diffs_per_full;
    const double writes = (p->N * p->T / (f * p->tau)) * (p->C_F + C_B * diffs_per_full);
    return failures * lost + writes;
}

extern "C" double ld_config_critical_interval(const ld_config_params* p, double b, double R_B, double C_B) {
    if (!p || !(b >= 1.0) || !(p->tau > 0.0) || !(R_B > 0.0) || !(p->C_F > C_B)) return NAN;
    return sqrt(2.0 * p->M * b * (p->C_F - C_B) / (p->tau * R_B));
}

extern "C" int32_t ld_config_select(const ld_config_params* p, int32_t n_cand, const int32_t* f, const int32_t* b,
                                    const double* R_B, const double* C_B, double* wasted) {
    if (!p || n_cand <= 0 || !f || !b || !R_B || !C_B) return -1;
    int32_t best = -1;
    double best_t = 0.0;
    for (int32_t i = 0; i < n_cand; ++i) {
        const double t = ld_config_wasted_time(p, static_cast<double>(f[i]), static_cast<double>(b[i]), R_B[i], C_B[i]);
        if (wasted) wasted[i] = t;
        if (t == t && (best < 0 || t < best_t)) {
            best = i;
            best_t = t;
        }
    }
    return best;
}
