/*
 * CPU oracle for the AdaTopK compress / decompress path.
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is the slow, plain statement of what the
 * path computes, used only by the tests, the smoke check and the benchmark's CPU
 * baseline leg.  The product library never links, loads or calls it, and it shares
 * no code with the HIP kernels.
 *
 * What it computes (paper Sec. 5.1, caption of the Top-K sparsification figure:
 * of a d-vector the k entries of largest absolute value are communicated as
 * (index, value) pairs and every other entry is zero after decompression;
 * Sec. 5.2, Eq. "adacompress": the per-link ratio rule):
 *
 *   1. key_i  = bit pattern of x_i with the sign bit cleared, read as an unsigned
 *               integer (31 bits for fp32, 15 bits for bf16 and fp16).  Ordering keys is
 *               ordering |x| for every finite value, and extends it to Inf / NaN.
 *   2. sort all (key_i, i) by key descending, then index ascending  (full sort).
 *   3. the first k pairs are the selected set.
 *   4. sort the selected set by index ascending; emit idx[j] and val[j] = the
 *      untouched bits of x[idx[j]].
 *   5. err = (float) sqrt( sum over the non-selected i of (double)x_i^2 ),
 *      summed in index order in fp64.
 *   6. decompress: y = n entries of +0.0, then y[idx[j]] = val[j].
 *
 * Readings where the paper is silent: ties at the threshold go to the lowest
 * index; output is in ascending index order; indices are 32-bit; the error norm
 * is the L2 norm of the residual x - decompress(compress(x)).
 *
 * Pins (tests, CPU only): brute-force repeated arg-max and exhaustive subsets on
 * tiny inputs, selection invariants, agreement with numpy lexsort / torch.topk on
 * distinct magnitudes, closed forms (all-equal, k = n, k = 1, pre-sorted input),
 * err^2 = |x|^2 - |val|^2, the Gaussian closed form of the relative error, the
 * paper's wire-size arithmetic and a hand-worked example of Eq. "adacompress".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    uint32_t key;
    int32_t idx;
} oracle_pair;

static int cmp_key_desc_idx_asc(const void *pa, const void *pb) {
    const oracle_pair *a = (const oracle_pair *)pa;
    const oracle_pair *b = (const oracle_pair *)pb;
    if (a->key != b->key) return (a->key > b->key) ? -1 : 1;
    if (a->idx != b->idx) return (a->idx < b->idx) ? -1 : 1;
    return 0;
}

static int cmp_idx_asc(const void *pa, const void *pb) {
    const int32_t a = *(const int32_t *)pa, b = *(const int32_t *)pb;
    return (a > b) - (a < b);
}

static float bf16_to_f32(uint16_t h) {
    uint32_t u = ((uint32_t)h) << 16; /* exact widening */
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

/* IEEE binary16 -> fp32, exact: 1 sign, 5 exponent (bias 15), 10 fraction bits. */
float oracle_f16_to_f32(uint16_t h) {
    const int sign = (h >> 15) & 1, e = (h >> 10) & 0x1F, m = h & 0x3FF;
    double v;
    if (e == 0) v = ldexp((double)m, -24);                   /* zero and denormals: m * 2^-24 */
    else if (e == 31) v = m ? (double)NAN : (double)INFINITY;
    else v = ldexp((double)(1024 + m), e - 25);              /* (1 + m/1024) * 2^(e-15) */
    return (float)(sign ? -v : v);
}

/* Steps 1-4: fills idx[k] (ascending).  keys[] holds key_i for all i.  The caller
 * owns every buffer.  Returns 0, or -1 on bad arguments / out of memory. */
static int select_topk(const uint32_t *keys, int64_t n, int64_t k, int32_t *idx) {
    if (n < 0 || k < 0 || k > n || n > INT32_MAX) return -1;
    if (k == 0) return 0;
    oracle_pair *p = (oracle_pair *)malloc((size_t)n * sizeof *p);
    if (!p) return -1;
    for (int64_t i = 0; i < n; ++i) {
        p[i].key = keys[i];
        p[i].idx = (int32_t)i;
    }
    qsort(p, (size_t)n, sizeof *p, cmp_key_desc_idx_asc);
    for (int64_t j = 0; j < k; ++j) idx[j] = p[j].idx;
    free(p);
    qsort(idx, (size_t)k, sizeof *idx, cmp_idx_asc);
    return 0;
}

int oracle_compress_f32(const float *x, int64_t n, int64_t k, int32_t *idx, float *val, float *err) {
    if (n < 0 || k < 0 || k > n || n > INT32_MAX) return -1;
    uint32_t *keys = (uint32_t *)malloc((size_t)(n > 0 ? n : 1) * sizeof *keys);
    uint8_t *sel = (uint8_t *)calloc((size_t)(n > 0 ? n : 1), 1);
    if (!keys || !sel) { free(keys); free(sel); return -1; }
    for (int64_t i = 0; i < n; ++i) {
        uint32_t u;
        memcpy(&u, &x[i], sizeof u);
        keys[i] = u & 0x7FFFFFFFu;
    }
    int rc = select_topk(keys, n, k, idx);
    if (rc == 0) {
        for (int64_t j = 0; j < k; ++j) {
            memcpy(&val[j], &x[idx[j]], sizeof(float)); /* bits, not a float move */
            sel[idx[j]] = 1;
        }
        if (err) {
            double s = 0.0;
            for (int64_t i = 0; i < n; ++i)
                if (!sel[i]) s += (double)x[i] * (double)x[i];
            *err = (float)sqrt(s);
        }
    }
    free(keys);
    free(sel);
    return rc;
}

int oracle_compress_bf16(const uint16_t *x, int64_t n, int64_t k, int32_t *idx, uint16_t *val, float *err) {
    if (n < 0 || k < 0 || k > n || n > INT32_MAX) return -1;
    uint32_t *keys = (uint32_t *)malloc((size_t)(n > 0 ? n : 1) * sizeof *keys);
    uint8_t *sel = (uint8_t *)calloc((size_t)(n > 0 ? n : 1), 1);
    if (!keys || !sel) { free(keys); free(sel); return -1; }
    for (int64_t i = 0; i < n; ++i) keys[i] = (uint32_t)(x[i] & 0x7FFFu);
    int rc = select_topk(keys, n, k, idx);
    if (rc == 0) {
        for (int64_t j = 0; j < k; ++j) {
            val[j] = x[idx[j]];
            sel[idx[j]] = 1;
        }
        if (err) {
            double s = 0.0;
            for (int64_t i = 0; i < n; ++i)
                if (!sel[i]) {
                    double v = (double)bf16_to_f32(x[i]);
                    s += v * v;
                }
            *err = (float)sqrt(s);
        }
    }
    free(keys);
    free(sel);
    return rc;
}

/* fp16: the key is again the 15 bits below the sign; only the widening for step 5 differs. */
int oracle_compress_f16(const uint16_t *x, int64_t n, int64_t k, int32_t *idx, uint16_t *val, float *err) {
    if (n < 0 || k < 0 || k > n || n > INT32_MAX) return -1;
    uint32_t *keys = (uint32_t *)malloc((size_t)(n > 0 ? n : 1) * sizeof *keys);
    uint8_t *sel = (uint8_t *)calloc((size_t)(n > 0 ? n : 1), 1);
    if (!keys || !sel) { free(keys); free(sel); return -1; }
    for (int64_t i = 0; i < n; ++i) keys[i] = (uint32_t)(x[i] & 0x7FFFu);
    int rc = select_topk(keys, n, k, idx);
    if (rc == 0) {
        for (int64_t j = 0; j < k; ++j) {
            val[j] = x[idx[j]];
            sel[idx[j]] = 1;
        }
        if (err) {
            double s = 0.0;
            for (int64_t i = 0; i < n; ++i)
                if (!sel[i]) {
                    double v = (double)oracle_f16_to_f32(x[i]);
                    s += v * v;
                }
            *err = (float)sqrt(s);
        }
    }
    free(keys);
    free(sel);
    return rc;
}

/* Step 6.  Indices must be unique and inside [0, n); anything else is an error. */
int oracle_decompress_f32(const int32_t *idx, const float *val, int64_t k, float *y, int64_t n) {
    if (n < 0 || k < 0) return -1;
    memset(y, 0, (size_t)n * sizeof *y);
    for (int64_t j = 0; j < k; ++j) {
        if (idx[j] < 0 || (int64_t)idx[j] >= n) return -1;
        memcpy(&y[idx[j]], &val[j], sizeof(float));
    }
    return 0;
}

/* Any 16-bit type (bf16, fp16): patterns are moved, never interpreted. */
int oracle_decompress_bf16(const int32_t *idx, const uint16_t *val, int64_t k, uint16_t *y, int64_t n) {
    if (n < 0 || k < 0) return -1;
    memset(y, 0, (size_t)n * sizeof *y);
    for (int64_t j = 0; j < k; ++j) {
        if (idx[j] < 0 || (int64_t)idx[j] >= n) return -1;
        y[idx[j]] = val[j];
    }
    return 0;
}

/* Rounding of a real number to a binary format with p significand bits (hidden bit included) and
 * normal exponents emin..emax, to nearest, ties to even, by the format's definition: the spacing of
 * representable numbers around s is 2^(e - p + 1) with e = max(floor(log2 |s|), emin). */
static double round_to_format(double s, int p, int emin, int emax) {
    if (s == 0.0 || isnan(s) || isinf(s)) return s;
    int e;
    (void)frexp(fabs(s), &e);
    e -= 1; /* 2^e <= |s| < 2^(e+1) */
    if (e < emin) e = emin;
    double quantum = ldexp(1.0, e - (p - 1));
    double r = rint(s / quantum) * quantum; /* rint: nearest, ties to even, in the default rounding mode */
    if (fabs(r) >= ldexp(1.0, emax + 1)) r = copysign(INFINITY, s);
    return r;
}

/* bf16: 8 significand bits, exponents -126..127; its values are fp32 values with 16 zero low bits. */
uint16_t oracle_round_bf16(double s) {
    if (isnan(s)) return 0x7FC0;
    float f = (float)round_to_format(s, 8, -126, 127); /* exact: every bf16 value is an fp32 value */
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    return (uint16_t)(u >> 16);
}

/* fp16: 11 significand bits, exponents -14..15. */
uint16_t oracle_round_f16(double s) {
    if (isnan(s)) return 0x7E00;
    double r = round_to_format(s, 11, -14, 15);
    uint16_t sign = signbit(r) ? 0x8000 : 0;
    double a = fabs(r);
    if (isinf(a)) return (uint16_t)(sign | 0x7C00);
    if (a < ldexp(1.0, -14)) return (uint16_t)(sign | (uint16_t)(a * 16777216.0)); /* a = m * 2^-24 */
    int e;
    double f = frexp(a, &e); /* a = f * 2^e with f in [0.5, 1) = (1 + m/1024) * 2^(e-1) */
    return (uint16_t)(sign | ((uint16_t)(e - 1 + 15) << 10) | (uint16_t)((f * 2.0 - 1.0) * 1024.0));
}

/* Accumulating decompress: y[idx[j]] += val[j], the exact sum rounded once to the type (to nearest,
 * ties to even); everything else in y is left alone.  Indices unique and inside [0, n). */
int oracle_decompress_accumulate_f32(const int32_t *idx, const float *val, int64_t k, float *y, int64_t n) {
    if (n < 0 || k < 0) return -1;
    for (int64_t j = 0; j < k; ++j) {
        if (idx[j] < 0 || (int64_t)idx[j] >= n) return -1;
        y[idx[j]] = (float)((double)y[idx[j]] + (double)val[j]); /* 53 bits hold the sum well enough to round once */
    }
    return 0;
}

int oracle_decompress_accumulate_bf16(const int32_t *idx, const uint16_t *val, int64_t k, uint16_t *y, int64_t n) {
    if (n < 0 || k < 0) return -1;
    for (int64_t j = 0; j < k; ++j) {
        if (idx[j] < 0 || (int64_t)idx[j] >= n) return -1;
        y[idx[j]] = oracle_round_bf16((double)bf16_to_f32(y[idx[j]]) + (double)bf16_to_f32(val[j]));
    }
    return 0;
}

int oracle_decompress_accumulate_f16(const int32_t *idx, const uint16_t *val, int64_t k, uint16_t *y, int64_t n) {
    if (n < 0 || k < 0) return -1;
    for (int64_t j = 0; j < k; ++j) {
        if (idx[j] < 0 || (int64_t)idx[j] >= n) return -1;
        y[idx[j]] = oracle_round_f16((double)oracle_f16_to_f32(y[idx[j]]) + (double)oracle_f16_to_f32(val[j]));
    }
    return 0;
}

/* Segmented variant: the single-tensor routine once per tensor.  x is the
 * concatenation of the S tensors; tensor s starts at in_offset[s] (S+1 entries) and
 * its outputs start at out_offset[s] (S+1 entries, the exclusive scan of k). */
int oracle_compress_segmented_f32(const float *x, const int64_t *in_offset, const int64_t *k, int32_t S,
                                  int32_t *idx, float *val, const int64_t *out_offset, float *err) {
    for (int32_t s = 0; s < S; ++s) {
        int rc = oracle_compress_f32(x + in_offset[s], in_offset[s + 1] - in_offset[s], k[s],
                                     idx + out_offset[s], val + out_offset[s], err ? err + s : NULL);
        if (rc) return rc;
    }
    return 0;
}

int oracle_compress_segmented_bf16(const uint16_t *x, const int64_t *in_offset, const int64_t *k, int32_t S,
                                   int32_t *idx, uint16_t *val, const int64_t *out_offset, float *err) {
    for (int32_t s = 0; s < S; ++s) {
        int rc = oracle_compress_bf16(x + in_offset[s], in_offset[s + 1] - in_offset[s], k[s],
                                      idx + out_offset[s], val + out_offset[s], err ? err + s : NULL);
        if (rc) return rc;
    }
    return 0;
}

int oracle_compress_segmented_f16(const uint16_t *x, const int64_t *in_offset, const int64_t *k, int32_t S,
                                  int32_t *idx, uint16_t *val, const int64_t *out_offset, float *err) {
    for (int32_t s = 0; s < S; ++s) {
        int rc = oracle_compress_f16(x + in_offset[s], in_offset[s + 1] - in_offset[s], k[s],
                                     idx + out_offset[s], val + out_offset[s], err ? err + s : NULL);
        if (rc) return rc;
    }
    return 0;
}

/* Sec. 5.2, Eq. "adacompress": r_i = max(1, coeff * r * R_i / max_p R_p); the paper's
 * coefficient is 3 (fp32 value + int64 index).  R are the estimated uncompressed
 * communication times of the m links. */
int oracle_adaptive_ratios(const double *R, int32_t m, double r, double coeff, double *r_out) {
    if (m <= 0 || !(r > 0.0) || !(coeff > 0.0)) return -1;
    double Rmax = R[0];
    for (int32_t i = 0; i < m; ++i) {
        if (!(R[i] >= 0.0)) return -1;
        if (R[i] > Rmax) Rmax = R[i];
    }
    if (!(Rmax > 0.0)) return -1;
    for (int32_t i = 0; i < m; ++i) {
        double v = coeff * r * R[i] / Rmax;
        r_out[i] = v > 1.0 ? v : 1.0;
    }
    return 0;
}

/* A ratio r_i keeps one element in r_i: k = max(1, floor(n / r_i)), at most n. */
int64_t oracle_k_for_ratio(int64_t n, double r_i) {
    if (n <= 0 || !(r_i >= 1.0)) return n <= 0 ? 0 : -1;
    double q = floor((double)n / r_i);
    int64_t k = (int64_t)q;
    if (k < 1) k = 1;
    if (k > n) k = n;
    return k;
}

/* Sec. 3.5, alpha-beta model of one link: T = alpha + beta * M. */
double oracle_link_time(double alpha, double beta, double bytes) { return alpha + beta * bytes; }

/* Sec. 3.6, Eq. "time_pipe": sum_p (C_p + R_p) + (n_b - 1) * max_p max(C_p, R_p). */
double oracle_pipeline_time(const double *C, const double *R, int32_t m, int32_t n_b) {
    double sum = 0.0, worst = 0.0;
    for (int32_t p = 0; p < m; ++p) {
        sum += C[p] + R[p];
        if (C[p] > worst) worst = C[p];
        if (R[p] > worst) worst = R[p];
    }
    return sum + (double)(n_b - 1) * worst;
}

/* Sec. 5.2, Eq. "time_pipe_compress" with r_p from Eq. "adacompress".
 * variant 0 is the equation as printed (bottleneck term 3 (n_b - 1) max(C_p, R_p) / r);
 * variant 1 puts each link's own compressed time coeff R_p / r_p into the bottleneck term. */
double oracle_pipeline_time_compressed(const double *C, const double *R, int32_t m, int32_t n_b, double r,
                                       double coeff, int32_t variant) {
    double Rmax = 0.0;
    for (int32_t p = 0; p < m; ++p)
        if (R[p] > Rmax) Rmax = R[p];
    double sum = 0.0, worst_printed = 0.0, worst_own = 0.0;
    for (int32_t p = 0; p < m; ++p) {
        double rp = Rmax > 0.0 ? coeff * r * R[p] / Rmax : 1.0;
        if (rp < 1.0) rp = 1.0;
        double sent = coeff * R[p] / rp;
        sum += C[p] + sent;
        double a = C[p] > R[p] ? C[p] : R[p];
        double b = C[p] > sent ? C[p] : sent;
        if (a > worst_printed) worst_printed = a;
        if (b > worst_own) worst_own = b;
    }
    if (variant == 0) return sum + coeff * (double)(n_b - 1) * worst_printed / r;
    return sum + (double)(n_b - 1) * worst_own;
}
