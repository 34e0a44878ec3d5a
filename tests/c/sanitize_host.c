/* Host code under AddressSanitizer and UndefinedBehaviorSanitizer: the CPU oracle and the host-only
 * entry points of the library (ratio rule, time estimates, wire-message arithmetic), compiled from
 * source with -fsanitize=address,undefined into this one program and driven through their edge cases
 * with exactly sized heap buffers, so that a read or write one element past any of them, a signed
 * overflow or a misaligned access stops the run.  No device is involved.  Built and run by
 * tests/test_sanitizers.py.  Where both sides state the same equation of the paper (Sec. 3.5, 3.6,
 * 5.2) their answers are compared as well. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "adatopk.h"

int oracle_compress_f32(const float *x, int64_t n, int64_t k, int32_t *idx, float *val, float *err);
int oracle_compress_bf16(const uint16_t *x, int64_t n, int64_t k, int32_t *idx, uint16_t *val, float *err);
int oracle_compress_f16(const uint16_t *x, int64_t n, int64_t k, int32_t *idx, uint16_t *val, float *err);
int oracle_decompress_f32(const int32_t *idx, const float *val, int64_t k, float *y, int64_t n);
int oracle_decompress_bf16(const int32_t *idx, const uint16_t *val, int64_t k, uint16_t *y, int64_t n);
int oracle_decompress_accumulate_f32(const int32_t *idx, const float *val, int64_t k, float *y, int64_t n);
int oracle_decompress_accumulate_bf16(const int32_t *idx, const uint16_t *val, int64_t k, uint16_t *y, int64_t n);
int oracle_decompress_accumulate_f16(const int32_t *idx, const uint16_t *val, int64_t k, uint16_t *y, int64_t n);
int oracle_compress_segmented_f32(const float *x, const int64_t *in_offset, const int64_t *k, int32_t S, int32_t *idx,
                                  float *val, const int64_t *out_offset, float *err);
int oracle_compress_segmented_bf16(const uint16_t *x, const int64_t *in_offset, const int64_t *k, int32_t S,
                                   int32_t *idx, uint16_t *val, const int64_t *out_offset, float *err);
int oracle_compress_segmented_f16(const uint16_t *x, const int64_t *in_offset, const int64_t *k, int32_t S,
                                  int32_t *idx, uint16_t *val, const int64_t *out_offset, float *err);
float oracle_f16_to_f32(uint16_t h);
uint16_t oracle_round_bf16(double s);
uint16_t oracle_round_f16(double s);
int oracle_adaptive_ratios(const double *R, int32_t m, double r, double coeff, double *r_out);
int64_t oracle_k_for_ratio(int64_t n, double r_i);
double oracle_link_time(double alpha, double beta, double bytes);
double oracle_pipeline_time(const double *C, const double *R, int32_t m, int32_t n_b);
double oracle_pipeline_time_compressed(const double *C, const double *R, int32_t m, int32_t n_b, double r,
                                       double coeff, int32_t variant);

#define CHECK(cond)                                                       \
    do {                                                                  \
        if (!(cond)) {                                                    \
            fprintf(stderr, "line %d: %s\n", __LINE__, #cond);            \
            return 1;                                                     \
        }                                                                 \
    } while (0)

static uint32_t rng_state = 12707u;
static uint32_t next_u32(void) { /* xorshift: structure does not matter here, coverage of patterns does */
    rng_state ^= rng_state << 13;
    rng_state ^= rng_state >> 17;
    rng_state ^= rng_state << 5;
    return rng_state;
}

/* n == 0 still gets a real (one-byte) allocation so that a stray access is caught */
static void *exact(size_t bytes) { return malloc(bytes ? bytes : 1); }

static int run_f32(int64_t n, int64_t k, int pattern) {
    float *x = exact((size_t)n * 4), *val = exact((size_t)k * 4), *y = exact((size_t)n * 4), err = -1.0f;
    int32_t *idx = exact((size_t)k * 4);
    for (int64_t i = 0; i < n; ++i) {
        uint32_t u = pattern == 0 ? next_u32() : (pattern == 1 ? 0x3FC00000u ^ ((next_u32() & 1u) << 31) : (next_u32() % 5u) << 23);
        memcpy(&x[i], &u, 4);
    }
    CHECK(oracle_compress_f32(x, n, k, idx, val, &err) == 0);
    for (int64_t j = 1; j < k; ++j) CHECK(idx[j - 1] < idx[j]);
    for (int64_t j = 0; j < k; ++j) CHECK(idx[j] >= 0 && idx[j] < n && memcmp(&val[j], &x[idx[j]], 4) == 0);
    CHECK(oracle_decompress_f32(idx, val, k, y, n) == 0);
    CHECK(oracle_decompress_accumulate_f32(idx, val, k, y, n) == 0);
    CHECK(oracle_compress_f32(x, n, n + 1, idx, val, &err) != 0); /* k > n is refused, nothing is written */
    free(x); free(val); free(y); free(idx);
    return 0;
}

static int run_16(int64_t n, int64_t k, int pattern, int half) {
    uint16_t *x = exact((size_t)n * 2), *val = exact((size_t)k * 2), *y = exact((size_t)n * 2);
    int32_t *idx = exact((size_t)k * 4);
    float err = -1.0f;
    for (int64_t i = 0; i < n; ++i)
        x[i] = (uint16_t)(pattern == 0 ? next_u32() : (pattern == 1 ? 0x3FC0u : (next_u32() % 7u) << 7));
    CHECK((half ? oracle_compress_f16 : oracle_compress_bf16)(x, n, k, idx, val, &err) == 0);
    for (int64_t j = 1; j < k; ++j) CHECK(idx[j - 1] < idx[j]);
    for (int64_t j = 0; j < k; ++j) CHECK(idx[j] >= 0 && idx[j] < n && val[j] == x[idx[j]]);
    CHECK(oracle_decompress_bf16(idx, val, k, y, n) == 0);
    CHECK((half ? oracle_decompress_accumulate_f16 : oracle_decompress_accumulate_bf16)(idx, val, k, y, n) == 0);
    free(x); free(val); free(y); free(idx);
    return 0;
}

static int run_segmented(void) {
    const int64_t in_off[6] = {0, 0, 7, 8, 8, 300}, k[5] = {0, 7, 0, 0, 31}, out_off[6] = {0, 0, 7, 7, 7, 38};
    float *xf = exact(300 * 4), *vf = exact(38 * 4), *ef = exact(5 * 4);
    uint16_t *xh = exact(300 * 2), *vh = exact(38 * 2);
    int32_t *idx = exact(38 * 4);
    for (int i = 0; i < 300; ++i) {
        uint32_t u = next_u32();
        memcpy(&xf[i], &u, 4);
        xh[i] = (uint16_t)(u >> 16);
    }
    CHECK(oracle_compress_segmented_f32(xf, in_off, k, 5, idx, vf, out_off, ef) == 0);
    CHECK(oracle_compress_segmented_bf16(xh, in_off, k, 5, idx, vh, out_off, ef) == 0);
    CHECK(oracle_compress_segmented_f16(xh, in_off, k, 5, idx, vh, out_off, NULL) == 0);
    free(xf); free(vf); free(ef); free(xh); free(vh); free(idx);
    return 0;
}

static int run_rule(void) {
    enum { M = 6 };
    const double alpha[M] = {4.2e-2, 1e-4, 3e-3, 0.0, 5e-3, 2e-4}, beta[M] = {1e-6, 8e-10, 1.4e-8, 1e-7, 0.0, 9e-10};
    const int64_t n[M] = {8388608, 8388608, 1, 0, 12345, 1 << 30};
    double *R = exact(M * 8), *r_lib = exact(M * 8), *r_ora = exact(M * 8), *r_plan = exact(M * 8);
    int64_t *k_plan = exact(M * 8);
    for (int i = 0; i < M; ++i) {
        R[i] = adatopk_link_time(alpha[i], beta[i], 4.0 * (double)n[i]);
        CHECK(R[i] == oracle_link_time(alpha[i], beta[i], 4.0 * (double)n[i]));
    }
    CHECK(adatopk_adaptive_ratios(R, M, 100.0, 3.0, r_lib) == ADATOPK_OK);
    CHECK(oracle_adaptive_ratios(R, M, 100.0, 3.0, r_ora) == 0);
    CHECK(adatopk_plan_keep_counts(alpha, beta, n, M, ADATOPK_F32, 100.0, 3.0, r_plan, k_plan) == ADATOPK_OK);
    for (int i = 0; i < M; ++i) {
        CHECK(fabs(r_lib[i] - r_ora[i]) <= 1e-12 * r_ora[i] && r_plan[i] == r_lib[i]);
        CHECK(adatopk_k_for_ratio(n[i], r_lib[i]) == oracle_k_for_ratio(n[i], r_ora[i]) && k_plan[i] == adatopk_k_for_ratio(n[i], r_lib[i]));
    }
    CHECK(adatopk_plan_keep_counts(alpha, beta, n, M, ADATOPK_BF16, 100.0, 3.0, NULL, k_plan) == ADATOPK_OK);
    CHECK(adatopk_adaptive_ratios(R, 0, 100.0, 3.0, r_lib) == ADATOPK_EINVAL);
    CHECK(adatopk_adaptive_ratios(NULL, M, 100.0, 3.0, r_lib) == ADATOPK_EINVAL);
    CHECK(adatopk_k_for_ratio(INT64_MAX, 1.0) == INT64_MAX && adatopk_k_for_ratio(INT64_MAX, 1e300) == 1);
    CHECK(adatopk_k_for_ratio(10, NAN) == -1 && oracle_k_for_ratio(10, NAN) == -1);
    const double C[3] = {0.3, 0.7, 0.2}, Rp[3] = {2.0, 0.5, 4.0};
    for (int n_b = 1; n_b <= 5; ++n_b) {
        CHECK(fabs(adatopk_pipeline_time(C, Rp, 3, n_b) - oracle_pipeline_time(C, Rp, 3, n_b)) < 1e-12);
        for (int v = 0; v < 2; ++v)
            CHECK(fabs(adatopk_pipeline_time_compressed(C, Rp, 3, n_b, 100.0, 3.0, v) -
                       oracle_pipeline_time_compressed(C, Rp, 3, n_b, 100.0, 3.0, v)) < 1e-12);
    }
    CHECK(isnan(adatopk_pipeline_time(C, Rp, 0, 2)) && isnan(adatopk_pipeline_time_compressed(C, Rp, 3, 2, 100.0, 3.0, 2)));
    free(R); free(r_lib); free(r_ora); free(r_plan); free(k_plan);
    return 0;
}

static int run_wire(void) {
    for (int64_t k = 0; k < 70; ++k)
        for (int dt = 0; dt < 3; ++dt)
            for (int ib = 4; ib <= 8; ib += 4) {
                const size_t bytes = adatopk_wire_bytes(k, (adatopk_dtype)dt, ib);
                CHECK(bytes >= 64 && adatopk_wire_keep_count(bytes, (adatopk_dtype)dt, ib) == k);
                unsigned char *msg = exact(bytes); /* header check reads 64 bytes of an exactly sized message */
                memset(msg, 0, bytes);
                adatopk_wire_header h, out;
                memset(&h, 0, sizeof h);
                h.magic = ADATOPK_WIRE_MAGIC; h.version = ADATOPK_WIRE_VERSION; h.algorithm = ADATOPK_WIRE_TOPK;
                h.dtype = (uint8_t)dt; h.index_bytes = (uint8_t)ib; h.n = k + 3; h.k = k; h.idx_offset = 64;
                h.val_offset = (int64_t)(bytes - (size_t)k * (dt == 0 ? 4 : 2));
                memcpy(msg, &h, sizeof h);
                CHECK(adatopk_wire_parse_header(msg, bytes, &out) == ADATOPK_OK && out.k == k);
                CHECK(adatopk_wire_parse_header(msg + 1, bytes - 1, &out) == ADATOPK_EINVAL); /* unaligned source */
                CHECK(adatopk_wire_parse_header(msg, bytes + 1, &out) == ADATOPK_EINVAL);
                free(msg);
            }
    CHECK(adatopk_wire_bytes(-1, ADATOPK_F32, 4) == 0 && adatopk_wire_bytes((int64_t)1 << 31, ADATOPK_F32, 4) == 0);
    CHECK(adatopk_wire_keep_count(63, ADATOPK_F32, 4) == -1 && adatopk_wire_keep_count(65, ADATOPK_F32, 4) == -1);
    CHECK(adatopk_wire_keep_count(SIZE_MAX, ADATOPK_BF16, 4) == -1);
    return 0;
}

int main(void) {
    static const int64_t sizes[] = {0, 1, 2, 3, 17, 64, 65, 1000, 4097};
    for (unsigned a = 0; a < sizeof sizes / sizeof sizes[0]; ++a)
        for (int pattern = 0; pattern < 3; ++pattern) {
            const int64_t n = sizes[a];
            const int64_t ks[] = {0, 1, n / 3, n > 0 ? n - 1 : 0, n};
            for (unsigned b = 0; b < 5; ++b) {
                if (ks[b] > n) continue;
                if (run_f32(n, ks[b], pattern) || run_16(n, ks[b], pattern, 0) || run_16(n, ks[b], pattern, 1)) return 1;
            }
        }
    for (uint32_t h = 0; h < 65536; ++h) { /* every binary16 pattern through the widening and both roundings */
        const float f = oracle_f16_to_f32((uint16_t)h);
        if (f == f) { (void)oracle_round_f16((double)f); (void)oracle_round_bf16((double)f); }
    }
    (void)oracle_round_f16(1e300); (void)oracle_round_bf16(-1e300); (void)oracle_round_f16(NAN); (void)oracle_round_bf16(5e-324);
    if (run_segmented() || run_rule() || run_wire()) return 1;
    printf("sanitized host run ok\n");
    return 0;
}
