// lnmod_sched.cpp -- host-side dual-constraint bucket sizing (Eq. 2) and the cost-model fit of
// Sec. 3.2, declared in include/lnmod_sched.h.  Plain double arithmetic, no device code.
#include "lnmod_sched.h"

#include <cmath>

extern "C" {

int64_t lnmod_bucket_batch_size(int64_t S, double M_mem, double M_comp, double p) {
    if (S < 1 || !std::isfinite(M_mem) || !std::isfinite(M_comp) || !std::isfinite(p)) return 0;
    if (M_mem < 0.0 || M_comp < 0.0) return 0;
    const double s = static_cast<double>(S);
    const double by_mem = std::floor(M_mem / s);
    const double by_comp = std::floor(M_comp / std::pow(s, p));
    double b = by_mem < by_comp ? by_mem : by_comp;
    if (!(b >= 1.0)) b = 1.0;                               // also catches a NaN quotient
    if (b > 9.0e18) b = 9.0e18;
    return static_cast<int64_t>(b);
}

int lnmod_bucket_batch_sizes(const int64_t* S, int64_t n, double M_mem, double M_comp, double p,
                             int64_t* out) {
    if (n < 0 || (n > 0 && (!S || !out))) return 1;
    for (int64_t i = 0; i < n; ++i) out[i] = lnmod_bucket_batch_size(S[i], M_mem, M_comp, p);
    return 0;
}

int lnmod_fit_cost_model(const int64_t* B, const int64_t* S, const double* t, int64_t n,
                         double p_lo, double p_hi, double p_step, double* a_out, double* b_out,
                         double* p_out, double* r2_out) {
    if (!B || !S || !t || !a_out || !b_out || !p_out || !r2_out) return 1;
    if (n < 2 || !(p_step > 0.0) || !(p_hi >= p_lo) || !std::isfinite(p_lo) || !std::isfinite(p_hi) ||
        !std::isfinite(p_step))
        return 1;
    double t_mean = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        if (B[i] < 1 || S[i] < 1 || !std::isfinite(t[i])) return 1;
        t_mean += t[i];
    }
    t_mean /= static_cast<double>(n);
    double sst = 0.0;
    for (int64_t i = 0; i < n; ++i) sst += (t[i] - t_mean) * (t[i] - t_mean);
    if (!(sst > 0.0)) return 2;

    bool found = false;
    double best_r2 = 0.0;
    const int64_t steps = static_cast<int64_t>(std::floor((p_hi - p_lo) / p_step + 1e-9));
    for (int64_t g = 0; g <= steps; ++g) {
        const double p = p_lo + static_cast<double>(g) * p_step;
        // least squares of t on z = B * S^p, centred sums
        double z_mean = 0.0, z_min = 0.0, z_max = 0.0;
        for (int64_t i = 0; i < n; ++i) {
            const double z = static_cast<double>(B[i]) * std::pow(static_cast<double>(S[i]), p);
            z_mean += z;
            if (i == 0 || z < z_min) z_min = z;
            if (i == 0 || z > z_max) z_max = z;
        }
        if (!(z_max > z_min)) continue;                     // no line through one abscissa
        z_mean /= static_cast<double>(n);
        double szz = 0.0, szt = 0.0;
        for (int64_t i = 0; i < n; ++i) {
            const double z = static_cast<double>(B[i]) * std::pow(static_cast<double>(S[i]), p) - z_mean;
            szz += z * z;
            szt += z * (t[i] - t_mean);
        }
        if (!(szz > 0.0) || !std::isfinite(szz)) continue;
        const double b = szt / szz;
        const double a = t_mean - b * z_mean;
        double sse = 0.0;
        for (int64_t i = 0; i < n; ++i) {
            const double z = static_cast<double>(B[i]) * std::pow(static_cast<double>(S[i]), p);
            const double r = t[i] - (a + b * z);
            sse += r * r;
        }
        const double r2 = 1.0 - sse / sst;
        if (!found || r2 > best_r2) {
            found = true;
            best_r2 = r2;
            *a_out = a;
            *b_out = b;
            *p_out = p;
            *r2_out = r2;
        }
    }
    return found ? 0 : 2;
}

double lnmod_comp_bound(double target_sync, double a, double b) {
    if (!(b > 0.0)) return 0.0;
    const double m = (target_sync - a) / b;
    return (std::isfinite(m) && m > 0.0) ? m : 0.0;
}

}  // extern "C"
