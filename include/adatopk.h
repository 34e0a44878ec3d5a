/*
 * adatopk.h -- C ABI of the MI355X (gfx950) AdaTopK compressor.
 *
 * The operation is the Top-K sparsification of the paper's Sec. 5.1 (caption of the
 * Top-K figure): of a d-vector, the k entries of largest absolute value are sent as
 * (index, value) pairs and every other entry is 0 after decompression.  Sec. 5.2
 * (Eq. "adacompress") gives every slow link its own ratio, hence the segmented call
 * with one k per tensor.
 *
 * Result, fixed where the paper is silent:
 *   - key(x) = bit pattern of x with the sign bit cleared, compared as an unsigned
 *     integer (so NaN > Inf > finite, and -0 ties with +0);
 *   - the k largest keys are kept; ties at the k-th key go to the lowest indices;
 *   - outputs are in ascending index order; values are the untouched bits of the input;
 *   - err = L2 norm of (x - decompress(compress(x))) = sqrt(sum of squares of the
 *     dropped entries), accumulated in fp64, returned as fp32;
 *   - decompress writes +0.0 (all-zero bits) everywhere except at the given indices.
 *
 * Conventions for every call:
 *   - "device" pointers are HIP device memory of the current device; "host" pointers
 *     are ordinary process memory.  The caller owns every buffer.  The library never
 *     allocates or frees device memory, never synchronises, and copies nothing back to the host: all
 *     work is enqueued on `hip_stream` (a hipStream_t, NULL = the default stream)
 *     and the call returns at once.  Output sizes are known beforehand (exactly k).
 *   - a tensor is its flat contiguous buffer; indices are int32 and local to the
 *     tensor (to the segment in the segmented call), so n must be below 2^31.
 *   - bf16 and fp16 (IEEE binary16) values travel as 16-bit patterns; the paper's tensors are
 *     fp32 (Sec. 5.2), the 16-bit types are the half-width forms of the same operation.
 *   - the workspace is scratch: contents are undefined between calls and it may be
 *     reused by the next call on the same stream.  Calls that share a workspace
 *     must be ordered by the stream.
 *   - errors are returned as adatopk_status; nothing is enqueued when the status is
 *     ADATOPK_EINVAL or ADATOPK_EWORKSPACE.
 *   - the library keeps no state between calls (adatopk_compress_noalloc's device array aside):
 *     calls from several host threads are fine as long
 *     as calls that share a workspace or an output are ordered by their stream.  Every call can be
 *     captured into a HIP graph (kernel launches only; no memset or copy nodes).
 */
#ifndef ADATOPK_H
#define ADATOPK_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { ADATOPK_F32 = 0, ADATOPK_BF16 = 1, ADATOPK_F16 = 2 } adatopk_dtype;

typedef enum {
    ADATOPK_OK = 0,
    ADATOPK_EINVAL = 1,     /* bad n / k / dtype / offsets, NULL or misaligned pointer */
    ADATOPK_EWORKSPACE = 2, /* workspace smaller than adatopk_workspace_bytes() */
    ADATOPK_ERUNTIME = 3,   /* a HIP launch failed */
    ADATOPK_ENOTIMPL = 4
} adatopk_status;

/* Bytes of device workspace that a compress call over `num_segments` tensors holding
 * `n_total` elements in all needs (single-tensor call: num_segments = 1): the scratch of the
 * threshold search and of the ordered compaction of Sec. 5.1's Top-K step (per-chunk digit counts,
 * the candidate list).  Returns 0 for invalid arguments.  Host-only; touches no device. */
size_t adatopk_workspace_bytes(int64_t n_total, int32_t num_segments, adatopk_dtype dt);

/* Top-K sparsification of one tensor (Sec. 5.1).
 *   dense         device, n values of type dt, aligned to the element size
 *   k             0 <= k <= n; k == 0 or n == 0 keep nothing
 *   idx_out       device, k int32: kept indices, ascending
 *   val_out       device, k values of type dt: val_out[j] = bits of dense[idx_out[j]]
 *   err_norm_out  device, 1 float, or NULL to skip the store
 *   workspace     device, 256-byte aligned, at least adatopk_workspace_bytes(n, 1, dt)
 * EINVAL: n < 0, k < 0, k > n, n >= 2^31, unknown dt, NULL where a buffer is needed,
 * misaligned pointer.  EWORKSPACE: workspace too small. */
adatopk_status adatopk_compress(const void *dense, int64_t n, adatopk_dtype dt, int64_t k,
                                int32_t *idx_out, void *val_out, float *err_norm_out,
                                void *workspace, size_t workspace_bytes, void *hip_stream);

/* adatopk_compress for callers that cannot allocate device memory or carry a workspace around: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * result and errors as adatopk_compress, without the workspace: the scratch is an array of
 * ADATOPK_NOALLOC_MAX_WORKSPACE bytes (64 MiB) that lives in the library's device image, on every GPU
 * the library is loaded on, until the process ends.  The call allocates and frees nothing (its first
 * call on a device looks up the array's address there, once).
 *   ADATOPK_EWORKSPACE  adatopk_workspace_bytes(n, 1, dt) is larger than ADATOPK_NOALLOC_MAX_WORKSPACE
 *                       (nothing is enqueued)
 * All calls on one GPU share that GPU's array: calls that may overlap on one GPU (different streams
 * without an ordering between them, several host threads) race on it and must be ordered by the
 * caller; calls on one stream are ordered by the stream. */
#define ADATOPK_NOALLOC_MAX_WORKSPACE ((size_t)64 << 20)
adatopk_status adatopk_compress_noalloc(const void *dense, int64_t n, adatopk_dtype dt, int64_t k,
                                        int32_t *idx_out, void *val_out, float *err_norm_out,
                                        void *hip_stream);

/* Decompression (Sec. 5.1): dense_out = +0.0 everywhere, then dense_out[idx[j]] = val[j].
 *   idx, val   device, k entries; indices unique; any order (ascending is fastest)
 *   dense_out  device, n values of type dt
 * Indices outside [0, n) are skipped; with duplicate indices one of the values wins.
 * k == 0 gives all zeros.  EINVAL as for compress (k > n included). */
adatopk_status adatopk_decompress(const int32_t *idx, const void *val, int64_t k, adatopk_dtype dt,
                                  void *dense_out, int64_t n, void *hip_stream);

/* Decompression when idx is strictly ascending, which is how adatopk_compress writes it: the
 * same result as adatopk_decompress from one kernel that writes every output line once.  The
 * order is the caller's promise and is not checked: with idx not ascending every store still
 * stays inside dense_out, but entries may be dropped.  Arguments and errors as above. */
adatopk_status adatopk_decompress_sorted(const int32_t *idx, const void *val, int64_t k, adatopk_dtype dt,
                                         void *dense_out, int64_t n, void *hip_stream);

/* Accumulating decompression: dense_inout[idx[j]] += val[j], every other entry untouched.  A node
 * whose gradient is the sum of what several users send back (backward pass of Sec. 3.3: gradients
 * return to the argument nodes) calls it once per incoming message on a zeroed or running buffer.
 *   fp32: the fp32 sum.  bf16 / fp16: the exact sum of the two values rounded once to the type,
 *   to nearest, ties to even.  A NaN sum is stored as some NaN pattern of the type.
 *   idx, val     device, k entries, indices unique within the call; any order
 *   dense_inout  device, n values of type dt
 * Indices outside [0, n) are skipped; with duplicate indices in one call one of the additions may be
 * lost.  Calls on one buffer must be ordered by the stream.  EINVAL as for decompress. */
adatopk_status adatopk_decompress_accumulate(const int32_t *idx, const void *val, int64_t k, adatopk_dtype dt,
                                             void *dense_inout, int64_t n, void *hip_stream);

/* Segmented compress: S independent tensors, tensor s with its own k[s] (the per-link
 * ratios of Sec. 5.2), every pass launched once for all of them.
 *   dense       host array of S device pointers
 *   n, k        host arrays of S entries
 *   out_offset  host array of S+1 entries, the exclusive scan of k: tensor s writes
 *               idx_out / val_out entries [out_offset[s], out_offset[s+1])
 *   idx_out, val_out  device, out_offset[S] entries
 *   err_norm_out      device, S floats, or NULL
 *   workspace   device, at least adatopk_workspace_bytes(sum of n, S, dt)
 * The host arrays are read before the call returns.  EINVAL additionally when S < 0 or
 * out_offset is not the scan of k. */
adatopk_status adatopk_compress_segmented(const void *const *dense, const int64_t *n, const int64_t *k,
                                          int32_t S, adatopk_dtype dt, int32_t *idx_out, void *val_out,
                                          const int64_t *out_offset, float *err_norm_out,
                                          void *workspace, size_t workspace_bytes, void *hip_stream);

/* Segmented decompress, the counterpart of adatopk_compress_segmented: S tensors in as few
 * launches as fit, tensor s from the pairs [out_offset[s], out_offset[s+1]) of idx / val, which
 * must be strictly ascending within each tensor (as adatopk_compress_segmented writes them; the
 * same promise, and the same memory safety without it, as adatopk_decompress_sorted).
 *   idx, val    device, out_offset[S] entries
 *   out_offset  host array of S+1 entries, out_offset[0] = 0, non-decreasing
 *   dense_out   host array of S device pointers; tensor s has n[s] values of type dt
 *   n           host array of S entries
 * The host arrays are read before the call returns.  EINVAL: S < 0, offsets that decrease or give
 * more pairs than elements, n[s] outside [0, 2^31), NULL or misaligned buffers. */
adatopk_status adatopk_decompress_segmented(const int32_t *idx, const void *val, const int64_t *out_offset, int32_t S,
                                            adatopk_dtype dt, void *const *dense_out, const int64_t *n,
                                            void *hip_stream);

/* ---- Wire message.  What one compressed tensor looks like on the link: the (index, value) pairs
 * of Sec. 5.1 behind a fixed header that carries what the paper's message descriptor keeps for
 * compression (its Compress_cfg field, Sec. 3.4: the algorithm, the ratio, further parameters).
 * One contiguous buffer, little-endian:
 *     [0, 64)                         adatopk_wire_header
 *     [64, 64 + k * index_bytes)      indices, ascending; int32, or int64 as in the paper's own
 *                                     accounting (fp32 value + int64 index = 3 x the kept values, Sec. 5.2)
 *     padding with zeros to a multiple of 16
 *     [val_offset, val_offset + k * sizeof(value))   values
 * so the message of k pairs is adatopk_wire_bytes(k, dt, index_bytes) long and k follows from the
 * length (adatopk_wire_keep_count). */
#define ADATOPK_WIRE_MAGIC 0x314B5441u /* "ATK1" */
#define ADATOPK_WIRE_VERSION 1
#define ADATOPK_WIRE_TOPK 1 /* algorithm: top-k by magnitude */

typedef struct {
    uint32_t magic;
    uint16_t version;
    uint8_t algorithm;
    uint8_t dtype;       /* adatopk_dtype of the values */
    uint8_t index_bytes; /* 4 or 8 */
    uint8_t reserved0[3];
    float err_norm;      /* L2 norm of the dropped part, written by the compress kernels */
    int64_t n;           /* elements of the dense tensor */
    int64_t k;           /* pairs in the message */
    double ratio;        /* the link's ratio r_i (Eq. "adacompress") that k was derived from; informational */
    int64_t idx_offset;  /* = 64 */
    int64_t val_offset;
    uint8_t reserved1[8];
} adatopk_wire_header; /* 64 bytes */

/* Host-only.  Message length for k pairs; 0 for invalid arguments (k < 0, k >= 2^31, unknown dt,
 * index_bytes not 4 or 8). */
size_t adatopk_wire_bytes(int64_t k, adatopk_dtype dt, int32_t index_bytes);

/* Host-only.  The k whose message is exactly wire_bytes long, or -1 if there is none. */
int64_t adatopk_wire_keep_count(size_t wire_bytes, adatopk_dtype dt, int32_t index_bytes);

/* Host-only.  Checks the first 64 bytes of a message held in HOST memory (a receiver has them
 * there before it uploads the message) against the message length and copies them to *out.
 * EINVAL: wrong magic / version / algorithm / dtype / index width, k > n, offsets or length that
 * do not fit k. */
adatopk_status adatopk_wire_parse_header(const void *host_bytes, size_t wire_bytes, adatopk_wire_header *out);

/* adatopk_compress with the outputs laid out as one wire message.
 *   wire_out       device, 16-byte aligned, wire_capacity >= adatopk_wire_bytes(k, dt, index_bytes) bytes.
 *                  May also be pinned host memory that the device addresses (hipHostMalloc): the kernels
 *                  then write the message over the bus and no device-to-host copy is needed before the
 *                  host sends it (measured: 95 us per call on the 25 M element tensor at k = 1 %,
 *                  against 60 us into device memory and 141 us with a copy behind it on the same stream).
 *   index_bytes    4, or 8 for int64 indices
 *   ratio          stored in the header as given
 * Everything else as adatopk_compress; EINVAL also for a buffer that is too small or misaligned. */
adatopk_status adatopk_compress_wire(const void *dense, int64_t n, adatopk_dtype dt, int64_t k, int32_t index_bytes,
                                     double ratio, void *wire_out, size_t wire_capacity, void *workspace,
                                     size_t workspace_bytes, void *hip_stream);

/* adatopk_compress_segmented with every tensor written as its own wire message into one buffer:
 * a node that feeds several links compresses all its outgoing tensors in one call and hands each
 * link its message.
 *   ratio        host array of S entries stored in the headers, or NULL to store n[s] / k[s]
 *   wire_out     device, 16-byte aligned
 *   wire_offset  host array of S entries: message s starts at byte wire_offset[s] (a multiple of
 *                16) and is adatopk_wire_bytes(k[s], dt, index_bytes) long; ascending, no overlap,
 *                the last one ends within wire_capacity
 * Everything else as adatopk_compress_segmented. */
adatopk_status adatopk_compress_wire_segmented(const void *const *dense, const int64_t *n, const int64_t *k, int32_t S,
                                               adatopk_dtype dt, int32_t index_bytes, const double *ratio,
                                               void *wire_out, const int64_t *wire_offset, size_t wire_capacity,
                                               void *workspace, size_t workspace_bytes, void *hip_stream);

/* Decompression of a wire message in device memory.  The receiver knows dt, index_bytes and n (the
 * tensor's shape is part of the graph); k follows from wire_bytes.  The device-side header is not
 * read: parse it on the host before the upload if it is to be checked.
 *   accumulate == 0   dense = decompress(message)  (as adatopk_decompress_sorted)
 *   accumulate != 0   dense += decompress(message) (as adatopk_decompress_accumulate)
 * EINVAL: no k fits wire_bytes, k > n, misaligned or NULL buffers. */
adatopk_status adatopk_decompress_wire(const void *wire, size_t wire_bytes, adatopk_dtype dt, int32_t index_bytes,
                                       int64_t n, int32_t accumulate, void *dense, void *hip_stream);

/* Host-only: the adaptive ratio rule, Sec. 5.2, Eq. "adacompress":
 *   r_out[i] = max(1, coeff * r_user * R[i] / max_p R[p])
 * R = estimated uncompressed communication time of each of the m links (>= 0, not all
 * zero); coeff = 3 in the paper (fp32 value + int64 index).  EINVAL otherwise. */
adatopk_status adatopk_adaptive_ratios(const double *R, int32_t m, double r_user, double coeff,
                                       double *r_out);

/* Host-only: elements kept at ratio r_i >= 1 (Sec. 5.2: a link with ratio r_i sends one element in
 * r_i; ratio 1 sends the tensor as it is): max(1, floor(n / r_i)), at most n; 0 when n <= 0; -1 when
 * r_i < 1 or is NaN. */
int64_t adatopk_k_for_ratio(int64_t n, double r_i);

/* Host-only: the estimates that feed the rule (paper Sec. 3.5 and 3.6) and what the rule does to
 * the pipeline (Sec. 5.2).  All return NaN for invalid arguments (m <= 0, n_b < 1, NULL, negative
 * or non-finite times).
 *   adatopk_link_time             alpha-beta model, Sec. 3.5: T_comm(M) = alpha + beta * M
 *   adatopk_pipeline_time         Eq. "time_pipe", Sec. 3.6:
 *                                 sum_p (C_p + R_p) + (n_b - 1) * max_p max(C_p, R_p)
 *   adatopk_pipeline_time_compressed   Eq. "time_pipe_compress", Sec. 5.2, with r_p from Eq. "adacompress":
 *       variant 0, as printed:    sum_p (C_p + coeff R_p / r_p) + coeff (n_b - 1) max_p max(C_p, R_p) / r_user
 *       variant 1, every link with its own ratio also in the bottleneck term:
 *                                 sum_p (C_p + coeff R_p / r_p) + (n_b - 1) max_p max(C_p, coeff R_p / r_p)
 * C, R: computation and uncompressed communication time of each of the m pipeline stages. */
double adatopk_link_time(double alpha, double beta, double message_bytes);
double adatopk_pipeline_time(const double *C, const double *R, int32_t m, int32_t n_b);
double adatopk_pipeline_time_compressed(const double *C, const double *R, int32_t m, int32_t n_b, double r_user,
                                        double coeff, int32_t variant);

/* Host-only: from link parameters to the k array of a segmented compress call.  Tensor s of n[s]
 * values of type dt crosses a link with latency alpha[s] and inverse bandwidth beta[s] (seconds per
 * byte): R_s = alpha_s + beta_s * bytes(tensor s) (Sec. 3.5), r_s from Eq. "adacompress",
 * k_out[s] = adatopk_k_for_ratio(n[s], r_s).  r_out may be NULL.  EINVAL as for the rule. */
adatopk_status adatopk_plan_keep_counts(const double *alpha, const double *beta, const int64_t *n, int32_t m,
                                        adatopk_dtype dt, double r_user, double coeff, double *r_out,
                                        int64_t *k_out);

#ifdef __cplusplus
}
#endif
#endif /* ADATOPK_H */
