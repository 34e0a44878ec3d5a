/* The headers must compile as plain C, and the host-only entry points must link and answer from a C
 * program that never touches a device.  Built and run by tests/test_abi_host.py. */
#include <math.h>
#include <stdio.h>
#include <string.h>

#include "adatopk.h"
#ifdef WITH_MEASURE /* linked against the measuring build, which also exports the benchmark's hooks */
#include "adatopk_measure.h"
#endif

int main(void) {
    /* Eq. "adacompress" by hand: R = {1, 4, 2}, r = 10, coeff = 3 -> {7.5, 30, 15} */
    const double R[3] = {1.0, 4.0, 2.0};
    double r[3];
    if (adatopk_adaptive_ratios(R, 3, 10.0, 3.0, r) != ADATOPK_OK) return 1;
    if (fabs(r[0] - 7.5) > 1e-12 || fabs(r[1] - 30.0) > 1e-12 || fabs(r[2] - 15.0) > 1e-12) return 2;
    if (adatopk_k_for_ratio(1000, 30.0) != 33) return 3;
    if (adatopk_wire_bytes(3, ADATOPK_F32, 4) != 64 + 16 + 12) return 4;
    if (adatopk_wire_keep_count(64 + 32 + 12, ADATOPK_F32, 8) != 3) return 5;
    if (sizeof(adatopk_wire_header) != 64) return 6;
    if (adatopk_workspace_bytes(1000, 1, ADATOPK_BF16) == 0) return 7;
    /* bad arguments are refused before any device is touched */
    if (adatopk_compress(NULL, 10, ADATOPK_F32, 1, NULL, NULL, NULL, NULL, 0, NULL) != ADATOPK_EINVAL) return 8;
    if (fabs(adatopk_link_time(0.5, 2.0, 3.0) - 6.5) > 1e-12) return 9;
    adatopk_wire_header h;
    unsigned char raw[64];
    memset(raw, 0, sizeof raw);
    if (adatopk_wire_parse_header(raw, 64, &h) != ADATOPK_EINVAL) return 10; /* no magic */
#ifdef WITH_MEASURE
    if (adatopk_measure_stage_count() < 5 || adatopk_measure_stage_name(0) == NULL) return 11;
#endif
    /* the call without a workspace refuses a tensor whose scratch would not fit its resident array,
     * and bad arguments, before any device is touched */
    if (adatopk_compress_noalloc(raw, (int64_t)1 << 30, ADATOPK_F32, 1, NULL, NULL, NULL, NULL) != ADATOPK_EWORKSPACE) return 12;
    if (adatopk_compress_noalloc(raw, -1, ADATOPK_F32, 0, NULL, NULL, NULL, NULL) != ADATOPK_EINVAL) return 13;
    if (adatopk_decompress(NULL, NULL, 11, ADATOPK_F32, raw, 10, NULL) != ADATOPK_EINVAL) return 14; /* k > n */
    printf("c abi host check ok\n");
    return 0;
}
