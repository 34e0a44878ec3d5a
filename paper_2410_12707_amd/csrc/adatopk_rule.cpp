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

}  // extern "C"
