// Host-only entry points of libadatopk (no device is touched, nothing here needs hipcc): the
// bandwidth-adaptive ratio rule of the paper's Sec. 5.2 (Eq. "adacompress"), the ratio ->
// element-count conversion, the link and pipeline time estimates that feed the rule (Sec. 3.5,
// 3.6), and the size arithmetic and header check of the wire message.
#include <cmath>
#include <cstdint>
#include <cstring>

#include "adatopk.h"
#include "wire_layout.h"

using adatopk_internal::dtype_ok;
using adatopk_internal::elem_size;
using adatopk_internal::wire_val_offset;

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
static bool times_ok(const double *C, const double *R, int32_t m) {
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

// ---- wire message
size_t adatopk_wire_bytes(int64_t k, adatopk_dtype dt, int32_t index_bytes) {
    if (k < 0 || k >= (static_cast<int64_t>(1) << 31) || !dtype_ok(dt) || (index_bytes != 4 && index_bytes != 8)) return 0;
    return wire_val_offset(k, index_bytes) + static_cast<size_t>(k) * elem_size(dt);
}

int64_t adatopk_wire_keep_count(size_t wire_bytes, adatopk_dtype dt, int32_t index_bytes) {
    if (!dtype_ok(dt) || (index_bytes != 4 && index_bytes != 8) || wire_bytes < sizeof(adatopk_wire_header)) return -1;
    // bytes(k) grows by index_bytes + element size per pair plus padding of at most 15: start from
    // the estimate without padding and walk down to the k whose size matches
    const size_t per = static_cast<size_t>(index_bytes) + elem_size(dt);
    int64_t k = static_cast<int64_t>((wire_bytes - sizeof(adatopk_wire_header)) / per);
    if (k >= (static_cast<int64_t>(1) << 31)) return -1;
    for (int step = 0; step < 16 && k >= 0; ++step, --k)
        if (adatopk_wire_bytes(k, dt, index_bytes) == wire_bytes) return k;
    return -1;
}

adatopk_status adatopk_wire_parse_header(const void *host_bytes, size_t wire_bytes, adatopk_wire_header *out) {
    if (!host_bytes || !out || wire_bytes < sizeof(adatopk_wire_header)) return ADATOPK_EINVAL;
    adatopk_wire_header h;
    std::memcpy(&h, host_bytes, sizeof h);
    if (h.magic != ADATOPK_WIRE_MAGIC || h.version != ADATOPK_WIRE_VERSION || h.algorithm != ADATOPK_WIRE_TOPK)
        return ADATOPK_EINVAL;
    const adatopk_dtype dt = static_cast<adatopk_dtype>(h.dtype);
    if (!dtype_ok(dt) || (h.index_bytes != 4 && h.index_bytes != 8)) return ADATOPK_EINVAL;
    if (h.n < 0 || h.n >= (static_cast<int64_t>(1) << 31) || h.k < 0 || h.k > h.n) return ADATOPK_EINVAL;
    if (h.idx_offset != static_cast<int64_t>(sizeof(adatopk_wire_header)) ||
        h.val_offset != static_cast<int64_t>(wire_val_offset(h.k, h.index_bytes)) ||
        adatopk_wire_bytes(h.k, dt, h.index_bytes) != wire_bytes)
        return ADATOPK_EINVAL;
    *out = h;
    return ADATOPK_OK;
}

}  // extern "C"
