// Host-only helpers of libadatopk: the bandwidth-adaptive ratio rule of the paper's
// Sec. 5.2 (Eq. "adacompress") and the ratio -> element-count conversion.
#include <cmath>
#include <cstdint>

#include "adatopk.h"

extern "C" {

adatopk_status adatopk_adaptive_ratios(const double *R, int32_t m, double r_user, double coeff, double *r_out) {
    if (!R || !r_out || m <= 0 || !(r_user > 0.0) || !(coeff > 0.0)) return ADATOPK_EINVAL;
    double slowest = 0.0;
    for (int32_t i = 0; i < m; ++i) {
        if (!(R[i] >= 0.0) || std::isinf(R[i])) return ADATOPK_EINVAL;
        slowest = std::fmax(slowest, R[i]);
    }
    if (!(slowest > 0.0)) return ADATOPK_EINVAL;
    const double scale = coeff * r_user;
    for (int32_t i = 0; i < m; ++i) r_out[i] = std::fmax(1.0, scale * R[i] / slowest);
    return ADATOPK_OK;
}

int64_t adatopk_k_for_ratio(int64_t n, double r_i) {
    if (n <= 0) return 0;
    if (!(r_i >= 1.0)) return -1;
    const double kept = std::floor(static_cast<double>(n) / r_i);
    if (kept < 1.0) return 1;
    if (kept >= static_cast<double>(n)) return n;
    return static_cast<int64_t>(kept);
}

namespace {
bool times_ok(const double *C, const double *R, int32_t m) {
    if (!C || !R || m <= 0) return false;
    for (int32_t p = 0; p < m; ++p)
        if (!(C[p] >= 0.0) || !(R[p] >= 0.0) || std::isinf(C[p]) || std::isinf(R[p])) return false;
    return true;
}
}  // namespace

double adatopk_link_time(double alpha, double beta, double message_bytes) {
    if (!(alpha >= 0.0) || !(beta >= 0.0) || !(message_bytes >= 0.0)) return std::nan("");
    return alpha + beta * message_bytes;
}

double adatopk_pipeline_time(const double *C, const double *R, int32_t m, int32_t n_b) {
    if (!times_ok(C, R, m) || n_b < 1) return std::nan("");
    double latency = 0.0, bottleneck = 0.0;
    for (int32_t p = 0; p < m; ++p) {
        latency += C[p] + R[p];
        bottleneck = std::fmax(bottleneck, std::fmax(C[p], R[p]));
    }
    return latency + (n_b - 1) * bottleneck;
}

double adatopk_pipeline_time_compressed(const double *C, const double *R, int32_t m, int32_t n_b, double r_user,
                                        double coeff, int32_t variant) {
    if (!times_ok(C, R, m) || n_b < 1 || (variant != 0 && variant != 1)) return std::nan("");
    double slowest = 0.0;
    for (int32_t p = 0; p < m; ++p) slowest = std::fmax(slowest, R[p]);
    if (!(r_user > 0.0) || !(coeff > 0.0)) return std::nan("");
    double latency = 0.0, printed = 0.0, own = 0.0;
    for (int32_t p = 0; p < m; ++p) {
        // a pipeline without communication has nothing to compress: every ratio is 1
        const double r_p = slowest > 0.0 ? std::fmax(1.0, coeff * r_user * R[p] / slowest) : 1.0;
        const double sent = coeff * R[p] / r_p;
        latency += C[p] + sent;
        printed = std::fmax(printed, std::fmax(C[p], R[p]));
        own = std::fmax(own, std::fmax(C[p], sent));
    }
    return latency + (n_b - 1) * (variant == 0 ? coeff * printed / r_user : own);
}

adatopk_status adatopk_plan_keep_counts(const double *alpha, const double *beta, const int64_t *n, int32_t m,
                                        adatopk_dtype dt, double r_user, double coeff, double *r_out,
                                        int64_t *k_out) {
    if (!alpha || !beta || !n || !k_out || m <= 0 || (dt != ADATOPK_F32 && dt != ADATOPK_BF16 && dt != ADATOPK_F16))
        return ADATOPK_EINVAL;
    if (!(r_user > 0.0) || !(coeff > 0.0)) return ADATOPK_EINVAL;
    const double bytes_per_value = dt == ADATOPK_F32 ? 4.0 : 2.0;
    double slowest = 0.0;
    for (int32_t s = 0; s < m; ++s) {
        if (n[s] < 0) return ADATOPK_EINVAL;
        const double t = adatopk_link_time(alpha[s], beta[s], bytes_per_value * static_cast<double>(n[s]));
        if (std::isnan(t) || std::isinf(t)) return ADATOPK_EINVAL;
        slowest = std::fmax(slowest, t);
    }
    if (!(slowest > 0.0)) return ADATOPK_EINVAL;
    for (int32_t s = 0; s < m; ++s) {
        const double t = alpha[s] + beta[s] * bytes_per_value * static_cast<double>(n[s]);
        const double r_s = std::fmax(1.0, coeff * r_user * t / slowest);
        if (r_out) r_out[s] = r_s;
        k_out[s] = adatopk_k_for_ratio(n[s], r_s);
    }
    return ADATOPK_OK;
}

}  // extern "C"
