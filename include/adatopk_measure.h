/*
 * adatopk_measure.h -- measurement hooks of libadatopk (benchmark and profiling only).
 *
 * Not part of the compressor's contract: these calls exist so that a benchmark can
 * time the individual kernels of a compress / decompress call with HIP events on the
 * caller's stream, and can measure plain streaming kernels (the ceilings that the
 * HBM roofline fractions are compared with, and the known-size copy that hardware
 * counter readings are scaled by).  They keep process-global state, create HIP events
 * and synchronise; none of them may be used concurrently with another call.
 */
#ifndef ADATOPK_MEASURE_H
#define ADATOPK_MEASURE_H

#include <stddef.h>
#include <stdint.h>

#include "adatopk.h"

#ifdef __cplusplus
extern "C" {
#endif

/* on != 0: from now on every kernel of a compress / decompress call is launched with a
 * start and a stop HIP event that carry the timestamps of the dispatch itself (events are
 * created on the first enable).  on == 0: plain launches.  Returns ADATOPK_OK or
 * ADATOPK_ERUNTIME. */
adatopk_status adatopk_measure_enable(int32_t on);

/* Number of kernel stages a timed call can report, and their names (static strings):
 * the kernels of compress in launch order, then those of the two decompress calls. */
int32_t adatopk_measure_stage_count(void);
const char *adatopk_measure_stage_name(int32_t stage);

/* Waits for the stop events of the kernels launched since the last read and stores the
 * duration of the most recent launch of every stage in milliseconds into
 * ms_out[adatopk_measure_stage_count()] (host memory); stages that did not run since
 * the last read are reported as -1.  Returns ADATOPK_OK or ADATOPK_ERUNTIME. */
adatopk_status adatopk_measure_read(float *ms_out);

/* Plain streaming kernels on `hip_stream`; all pointers are device memory, 16-byte
 * aligned; bytes must be a multiple of 16.
 *   copy:      dst[i] = src[i]                        (reads bytes, writes bytes)
 *   read_only: folds src into one word at sink[0]     (reads bytes)
 *   fill:      dst[i] = 0, the kernel decompress uses (writes bytes) */
adatopk_status adatopk_measure_copy(void *dst, const void *src, size_t bytes, void *hip_stream);
adatopk_status adatopk_measure_read_only(const void *src, size_t bytes, uint32_t *sink, void *hip_stream);
adatopk_status adatopk_measure_fill(void *dst, size_t bytes, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* ADATOPK_MEASURE_H */
