// AdaTopK compress / decompress for MI355X (gfx950, wave64): kernels, launch planner and C ABI.
//
// Operation (paper Sec. 5.1, Top-K sparsification figure): keep the k entries of largest
// absolute value of a flat tensor as (int32 index, value) pairs; decompression writes them
// back into zeros.  Sec. 5.2 (Eq. "adacompress") gives every slow link its own ratio, so
// the launch is segmented: S tensors, each with its own k, one launch per pass for all.
//
// Method.  key(x) = bits(x) with the sign cleared (bf16 is widened to the fp32 pattern, so
// both types share one 31-bit key).  The exact k-th largest key T is found by a 3-level
// MSD radix select with digits of 11 / 10 / 10 bits:
//   k_init    zero the per-segment state and the three global histograms
//   k_hist1   one read of the input: per-chunk LDS histogram of the top digit, added into the
//             segment's global histogram G1; every chunk also stores the suffix sums of its
//             own histogram (one row per chunk)
//   k_gather  prologue (every block, redundantly): G1 -> digit bucket B1 holding the k-th key;
//             the chunk's slot range in the candidate list L = sum over the earlier chunks of
//             their stored count of digits >= B1.  Then the second read of the input: every
//             element whose top digit is >= B1 goes, in index order, into L (index, value);
//             members of bucket B1 are histogrammed on the second digit (G2); squares of the
//             elements below the bucket are summed in fp64 per chunk
//   k_hist3   over L only (about k + the bucket population).  Prologue: G2 -> second digit B2.
//             Histogram of the third digit of the entries matching (B1,B2) into G3, one row of
//             suffix sums per list block
//   k_emit    over L.  Prologue: G3 -> threshold key T and tie quota q; output offsets of the
//             list block from the rows of the earlier blocks.  Stable compaction into idx_out /
//             val_out (key > T, plus the first q keys equal to T); squares of dropped entries;
//             the block that finishes last adds all error partials in a fixed order
// Cross-block order comes only from counts that an EARLIER kernel stored and that every block
// of the next kernel scans for itself: no block waits for another block (no launch can hang),
// no block needs a release fence (on this chip an agent-scope fence writes back the L2 of its
// XCD, about 1.5 us per workgroup, serialised), and every result, the fp64 error sum included,
// is the same from run to run.
//
// Decompress: k_fill (16-byte zero stores) then k_scatter.
#include <hip/hip_runtime.h>

#include <stdint.h>

#include "adatopk.h"
#include "adatopk_measure.h"

namespace {

constexpr int BLOCK = 512;          // threads per workgroup (8 wavefronts)
constexpr int NW = BLOCK / 64;      // wavefronts per workgroup
constexpr int U = 4;                // 16-byte groups per thread per tile
constexpr int LU = 4;               // list elements per thread per tile in the list kernels
constexpr int BITS1 = 11, BITS2 = 10, BITS3 = 10;
constexpr int NB1 = 1 << BITS1, NB2 = 1 << BITS2, NB3 = 1 << BITS3;
constexpr int SH1 = BITS2 + BITS3;  // key >> SH1 = first digit
constexpr int SH2 = BITS3;
constexpr int MAXSEG = 32;          // segments per launch (the table travels as kernel arguments)
constexpr int CTARGET = 512;        // chunks aimed at per launch (2 workgroups per CU)
constexpr int LB_ELEMS = 16384;     // input elements per list block when sizing the list grid
static_assert(U * NW <= 64 && LU * NW <= 64, "per-tile wave counts must fit one wavefront scan");
static_assert(NB1 % BLOCK == 0 && NB2 % BLOCK == 0 && NB3 % BLOCK == 0, "bins split evenly over threads");
static_assert(BITS1 + BITS2 + BITS3 == 31, "digits cover the 31-bit key");
static_assert(BLOCK >= 256, "k_emit scans the list blocks of a segment with one thread each");

struct SegState {  // one per segment, zeroed by k_init; 64 bytes
    uint32_t ticket;        // list blocks that have published their error partial
    uint32_t B1, c_gt1, m;  // bucket of level 1, #keys above it, length of the candidate list
    uint32_t B2, c_gt2;     // bucket of level 2, #keys above (B1,B2)
    uint32_t T, q, c_gt;    // threshold key, tie quota, #keys above T
    uint32_t pad[7];
};
static_assert(sizeof(SegState) == 64, "state record size");

struct SegDesc {
    const void *x;       // device pointer of the tensor
    int64_t out_off;     // first output slot of this segment
    int64_t l_base;      // first candidate-list slot of this segment
    int32_t n, k;
    int32_t chunk_begin, nchunks;
    int32_t lb_begin, lb_count;
    uint32_t aligned16;  // tensor base is 16-byte aligned
    uint32_t pad;
};

struct Launch {
    SegDesc seg[MAXSEG];
    int32_t S;
    int32_t E;  // elements per chunk (multiple of the tile)
    SegState *state;
    uint32_t *G1, *G2, *G3;                    // [MAXSEG][NBx] global histograms
    uint32_t *rows1;                           // [chunks][NB1] suffix sums of the chunk histograms
    double *chunk_err;                         // [chunks] sum of squares below the bucket
    uint32_t *rows3;                           // [list blocks][NB3] suffix sums
    uint32_t *ldef;                            // [list blocks] #keys above the 21-bit prefix
    double *lerr;                              // [list blocks]
    int32_t *L_idx;
    void *L_val;
    int32_t *idx_out;
    void *val_out;
    float *err_out;
};

// ------------------------------------------------------------------ element access
template <int VEC> struct Raw;
template <> struct Raw<4> { using type = uint32_t; };  // fp32
template <> struct Raw<8> { using type = uint16_t; };  // bf16

template <int VEC> __device__ __forceinline__ uint32_t key_of(uint32_t raw) {
    return VEC == 4 ? (raw & 0x7FFFFFFFu) : ((raw & 0x7FFFu) << 16);
}
template <int VEC> __device__ __forceinline__ float value_of(uint32_t raw) {
    return __uint_as_float(VEC == 4 ? raw : (raw << 16));
}

// One 16-byte group (VEC consecutive elements starting at element i0) -> raw[].
template <int VEC> __device__ __forceinline__ void load_vec(const void *x, int64_t i0, uint32_t (&raw)[VEC]) {
    const uint4 v = *reinterpret_cast<const uint4 *>(static_cast<const char *>(x) + i0 * (16 / VEC));
    if (VEC == 4) {
        raw[0] = v.x; raw[1] = v.y; raw[2] = v.z; raw[3] = v.w;
    } else {
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int e = 0; e < VEC; ++e) raw[e] = (w[e >> 1] >> ((e & 1) * 16)) & 0xFFFFu;
    }
}
// Guarded element-wise variant; returns the mask of elements below `end`.
template <int VEC> __device__ __forceinline__ uint32_t load_guarded(const void *x, int64_t i0, int64_t end,
                                                                      uint32_t (&raw)[VEC]) {
    using R = typename Raw<VEC>::type;
    const R *p = static_cast<const R *>(x);
    uint32_t m = 0;
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
        raw[e] = 0;
        if (i0 + e < end) {
            raw[e] = p[i0 + e];
            m |= 1u << e;
        }
    }
    return m;
}

// ------------------------------------------------------------------ wave / block helpers
__device__ __forceinline__ uint32_t lanes_below(uint64_t mask) {
    return __builtin_amdgcn_mbcnt_hi(static_cast<uint32_t>(mask >> 32),
                                     __builtin_amdgcn_mbcnt_lo(static_cast<uint32_t>(mask), 0u));
}

__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t v) {
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t t = __shfl_up(v, d);
        if (lane >= d) v += t;
    }
    return v;
}

// Inclusive prefix sum over the block in thread order; *total = block sum.  sm holds NW words.
__device__ __forceinline__ uint32_t block_incl_scan(uint32_t v, uint32_t *sm, uint32_t *total) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const uint32_t inc = wave_incl_scan(v);
    __syncthreads();
    if (lane == 63) sm[w] = inc;
    __syncthreads();
    uint32_t pre = 0, tot = 0;
#pragma unroll
    for (int i = 0; i < NW; ++i) {
        const uint32_t t = sm[i];
        pre += (i < w) ? t : 0u;
        tot += t;
    }
    *total = tot;
    return inc + pre;
}

// Block sum of doubles in a fixed order (same grouping every run).  sm holds NW doubles.
__device__ __forceinline__ double block_sum_f64(double v, double *sm) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) v += __shfl_down(v, d);
    __syncthreads();
    if (lane == 0) sm[w] = v;
    __syncthreads();
    double s = 0.0;
#pragma unroll
    for (int i = 0; i < NW; ++i) s += sm[i];
    return s;
}

// h[NB] raw counts -> inclusive suffix sums in place (h[b] = sum of counts of bins >= b).
template <int NB> __device__ __forceinline__ void block_suffix_inplace(uint32_t *h, uint32_t *sm) {
    constexpr int PER = NB / BLOCK;
    const int b0 = threadIdx.x * PER;
    uint32_t s = 0;
#pragma unroll
    for (int j = 0; j < PER; ++j) s += h[b0 + j];
    uint32_t total;
    const uint32_t inc = block_incl_scan(s, sm, &total);
    uint32_t run = total - inc;  // counts owned by higher threads
#pragma unroll
    for (int j = PER - 1; j >= 0; --j) {
        run += h[b0 + j];
        h[b0 + j] = run;
    }
    __syncthreads();
}

// On suffix sums suf[NB]: the bucket B with suf[B] >= krem > suf[B+1]; out[0] = B, out[1] = suf[B+1].
// krem == 0 selects nothing: B = NB.  out[] is in LDS; every thread calls; the caller syncs before reading it.
template <int NB> __device__ __forceinline__ void block_pick_bucket(const uint32_t *suf, uint32_t krem, uint32_t *out) {
    constexpr int PER = NB / BLOCK;
    if (threadIdx.x == 0) {  // also what stays when no bin qualifies (counts that do not add up)
        out[0] = NB;
        out[1] = 0;
    }
    __syncthreads();
    if (krem != 0) {
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            const int b = threadIdx.x * PER + j;
            const uint32_t above = (b + 1 < NB) ? suf[b + 1] : 0u;
            if (suf[b] >= krem && above < krem) {
                out[0] = b;
                out[1] = above;
            }
        }
    }
}

// Adds the non-zero bins of an LDS histogram into a global one.
template <int NB> __device__ __forceinline__ void flush_bins(const uint32_t *h, uint32_t *G) {
    for (int b = threadIdx.x; b < NB; b += BLOCK) {
        const uint32_t c = h[b];
        if (c) __hip_atomic_fetch_add(&G[b], c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}
// Error-norm hand-off without cache maintenance: thread 0 of every list block publishes its
// partial with a device-coherent store, waits until the store is acknowledged, and takes a
// ticket; the block that draws the last ticket reads all partials with device-coherent loads.
// (A release fence here would write back the whole L2 once per block.)  No block waits.
__device__ __forceinline__ void coherent_store_f64(double *p, double v) {
    __hip_atomic_store(reinterpret_cast<unsigned long long *>(p), static_cast<unsigned long long>(__double_as_longlong(v)),
                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ double coherent_load_f64(const double *p) {
    return __longlong_as_double(static_cast<long long>(__hip_atomic_load(
        reinterpret_cast<const unsigned long long *>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)));
}
__device__ __forceinline__ bool publish_and_take_ticket(double *slot, double v, uint32_t *ticket, uint32_t nblocks,
                                                        uint32_t *s_flag) {
    if (threadIdx.x == 0) {
        coherent_store_f64(slot, v);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        const uint32_t t = __hip_atomic_fetch_add(ticket, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        *s_flag = (t == nblocks - 1u) ? 1u : 0u;
    }
    __syncthreads();
    return *s_flag != 0u;
}

__device__ __forceinline__ int find_segment_by(const Launch &a, int g, bool by_chunk) {
    int s = 0;
    for (int i = 1; i < a.S; ++i) {
        const int begin = by_chunk ? a.seg[i].chunk_begin : a.seg[i].lb_begin;
        if (g >= begin) s = i;
    }
    return s;
}

// Global histogram G[NB] (complete: written by an earlier kernel) -> bucket B holding the
// krem-th largest digit and the count `above` it.  h[NB], sm[NW], s_pick[2] are LDS scratch.
template <int NB>
__device__ __forceinline__ void pick_from_global(const uint32_t *G, uint32_t krem, uint32_t *h, uint32_t *sm,
                                                 uint32_t *s_pick, uint32_t &B, uint32_t &above) {
    for (int b = threadIdx.x; b < NB; b += BLOCK) h[b] = G[b];
    __syncthreads();
    block_suffix_inplace<NB>(h, sm);
    block_pick_bucket<NB>(h, krem, s_pick);
    __syncthreads();
    B = s_pick[0];
    above = s_pick[1];
    __syncthreads();
}

// ------------------------------------------------------------------ k_init
__global__ __launch_bounds__(BLOCK) void k_init(Launch a) {
    const int s = blockIdx.x;
    uint32_t *st = reinterpret_cast<uint32_t *>(&a.state[s]);
    if (threadIdx.x < sizeof(SegState) / 4) st[threadIdx.x] = 0;
    for (int b = threadIdx.x; b < NB1; b += BLOCK) a.G1[s * NB1 + b] = 0;
    for (int b = threadIdx.x; b < NB2; b += BLOCK) a.G2[s * NB2 + b] = 0;
    for (int b = threadIdx.x; b < NB3; b += BLOCK) a.G3[s * NB3 + b] = 0;
}

// ------------------------------------------------------------------ k_hist1
template <int VEC, bool FULL>
__device__ __forceinline__ void hist1_tile(const void *x, int64_t t0, int64_t end, uint32_t *h) {
    uint32_t raw[U][VEC];
    uint32_t vm[U];
#pragma unroll
    for (int j = 0; j < U; ++j) {
        const int64_t i0 = t0 + (static_cast<int64_t>(j) * BLOCK + threadIdx.x) * VEC;
        if (FULL) {
            load_vec<VEC>(x, i0, raw[j]);
            vm[j] = (1u << VEC) - 1u;
        } else {
            vm[j] = load_guarded<VEC>(x, i0, end, raw[j]);
        }
    }
#pragma unroll
    for (int j = 0; j < U; ++j)
#pragma unroll
        for (int e = 0; e < VEC; ++e)
            if (FULL || ((vm[j] >> e) & 1u)) atomicAdd(&h[key_of<VEC>(raw[j][e]) >> SH1], 1u);
}

template <int VEC> __global__ __launch_bounds__(BLOCK) void k_hist1(Launch a) {
    __shared__ uint32_t h[NB1];
    __shared__ uint32_t sm[NW];
    constexpr int TILE = BLOCK * U * VEC;

    const int g = blockIdx.x;
    const int s = find_segment_by(a, g, true);
    const SegDesc &sg = a.seg[s];
    const int c = g - sg.chunk_begin;
    const int64_t beg = static_cast<int64_t>(c) * a.E;
    const int64_t end = (beg + a.E < sg.n) ? beg + a.E : sg.n;

    for (int b = threadIdx.x; b < NB1; b += BLOCK) h[b] = 0;
    __syncthreads();

    int64_t t0 = beg;
    if (sg.aligned16)
        for (; t0 + TILE <= end; t0 += TILE) hist1_tile<VEC, true>(sg.x, t0, end, h);
    for (; t0 < end; t0 += TILE) hist1_tile<VEC, false>(sg.x, t0, end, h);
    __syncthreads();

    flush_bins<NB1>(h, a.G1 + s * NB1);
    __syncthreads();
    block_suffix_inplace<NB1>(h, sm);
    uint32_t *row = a.rows1 + static_cast<size_t>(g) * NB1;
    for (int b = threadIdx.x; b < NB1; b += BLOCK) row[b] = h[b];
}

// ------------------------------------------------------------------ k_gather
template <int VEC, bool FULL>
__device__ __forceinline__ void gather_tile(const void *x, int64_t t0, int64_t end, uint32_t B1, uint32_t *h2,
                                            uint32_t *wcnt, uint32_t &running, uint32_t cnt, int32_t *Li,
                                            typename Raw<VEC>::type *Lv, double &acc) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    uint32_t raw[U][VEC];
    uint32_t vm[U];
#pragma unroll
    for (int j = 0; j < U; ++j) {
        const int64_t i0 = t0 + (static_cast<int64_t>(j) * BLOCK + threadIdx.x) * VEC;
        if (FULL) {
            load_vec<VEC>(x, i0, raw[j]);
            vm[j] = (1u << VEC) - 1u;
        } else {
            vm[j] = load_guarded<VEC>(x, i0, end, raw[j]);
        }
    }
    uint32_t keepbits[U], lane_pre[U];
#pragma unroll
    for (int j = 0; j < U; ++j) {
        uint32_t kb = 0, lp = 0, wc = 0;
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            const bool valid = FULL || ((vm[j] >> e) & 1u);
            const uint32_t key = key_of<VEC>(raw[j][e]);
            const uint32_t d = key >> SH1;
            const bool keep = valid && d >= B1;
            if (valid && d == B1) atomicAdd(&h2[(key >> SH2) & (NB2 - 1)], 1u);
            const double xd = (valid && d < B1) ? static_cast<double>(value_of<VEC>(raw[j][e])) : 0.0;
            acc = fma(xd, xd, acc);
            const uint64_t bal = __ballot(keep);
            lp += lanes_below(bal);
            wc += __popcll(bal);
            kb |= (keep ? 1u : 0u) << e;
        }
        keepbits[j] = kb;
        lane_pre[j] = lp;
        if (lane == 0) wcnt[j * NW + w] = wc;
    }
    __syncthreads();
    const uint32_t c = (lane < U * NW) ? wcnt[lane] : 0u;
    const uint32_t inc = wave_incl_scan(c);
    const uint32_t tot = __shfl(inc, 63);
    const uint32_t exc = inc - c;
#pragma unroll
    for (int j = 0; j < U; ++j) {
        uint32_t pos = running + __shfl(exc, j * NW + w) + lane_pre[j];
        const int64_t i0 = t0 + (static_cast<int64_t>(j) * BLOCK + threadIdx.x) * VEC;
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            if ((keepbits[j] >> e) & 1u) {
                if (pos < cnt) {
                    Li[pos] = static_cast<int32_t>(i0 + e);
                    Lv[pos] = static_cast<typename Raw<VEC>::type>(raw[j][e]);
                }
                ++pos;
            }
        }
    }
    running += tot;
}

template <int VEC> __global__ __launch_bounds__(BLOCK) void k_gather(Launch a) {
    using R = typename Raw<VEC>::type;
    __shared__ uint32_t h[NB1];  // top-digit histogram during the prologue, then the second-digit one
    __shared__ uint32_t wcnt[2][U * NW];
    __shared__ uint32_t sm[NW];
    __shared__ double smd[NW];
    __shared__ uint32_t s_pick[2];
    constexpr int TILE = BLOCK * U * VEC;

    const int g = blockIdx.x;
    const int s = find_segment_by(a, g, true);
    const SegDesc &sg = a.seg[s];
    const int c = g - sg.chunk_begin;
    const int64_t beg = static_cast<int64_t>(c) * a.E;
    const int64_t end = (beg + a.E < sg.n) ? beg + a.E : sg.n;

    // Prologue, the same in every block of the segment: bucket of the top digit, then this
    // chunk's slot range in the list = scan of the earlier chunks' counts of digits >= B1.
    uint32_t B1, c_gt1;
    pick_from_global<NB1>(a.G1 + s * NB1, static_cast<uint32_t>(sg.k), h, sm, s_pick, B1, c_gt1);
    uint32_t part = 0, cnt = 0;
    if (B1 < NB1) {
        const uint32_t *col = a.rows1 + static_cast<size_t>(sg.chunk_begin) * NB1 + B1;
        for (int cc = threadIdx.x; cc < c; cc += BLOCK) part += col[static_cast<size_t>(cc) * NB1];
        cnt = col[static_cast<size_t>(c) * NB1];
    }
    uint32_t off;
    block_incl_scan(part, sm, &off);
    if (c == sg.nchunks - 1 && threadIdx.x == 0) {
        a.state[s].B1 = B1;
        a.state[s].c_gt1 = c_gt1;
        a.state[s].m = off + cnt;
    }
    const int64_t lo = sg.l_base + off;
    int32_t *Li = a.L_idx + lo;
    R *Lv = static_cast<R *>(a.L_val) + lo;

    uint32_t *h2 = h;
    for (int b = threadIdx.x; b < NB2; b += BLOCK) h2[b] = 0;
    __syncthreads();

    double acc = 0.0;
    uint32_t running = 0;
    int buf = 0;
    int64_t t0 = beg;
    if (sg.aligned16)
        for (; t0 + TILE <= end; t0 += TILE, buf ^= 1)
            gather_tile<VEC, true>(sg.x, t0, end, B1, h2, wcnt[buf], running, cnt, Li, Lv, acc);
    for (; t0 < end; t0 += TILE, buf ^= 1)
        gather_tile<VEC, false>(sg.x, t0, end, B1, h2, wcnt[buf], running, cnt, Li, Lv, acc);

    const double bsum = block_sum_f64(acc, smd);
    if (threadIdx.x == 0) a.chunk_err[g] = bsum;
    __syncthreads();
    flush_bins<NB2>(h2, a.G2 + s * NB2);
}

// ------------------------------------------------------------------ list kernels
// Slot range of list block lb of a segment whose list holds m entries.
__device__ __forceinline__ void list_range(uint32_t m, int lb, int lb_count, uint32_t &beg, uint32_t &end) {
    constexpr uint32_t LT = BLOCK * LU;
    const uint32_t per = ((m + lb_count - 1) / lb_count + LT - 1) / LT * LT;  // whole tiles per block
    const uint64_t b = static_cast<uint64_t>(per) * lb;
    beg = b < m ? static_cast<uint32_t>(b) : m;
    end = (b + per < m) ? static_cast<uint32_t>(b + per) : m;
}

template <int VEC> __global__ __launch_bounds__(BLOCK) void k_hist3(Launch a) {
    using R = typename Raw<VEC>::type;
    __shared__ uint32_t h[NB2 > NB3 ? NB2 : NB3];
    __shared__ uint32_t sm[NW];
    __shared__ uint32_t s_pick[2];

    const int g = blockIdx.x;
    const int s = find_segment_by(a, g, false);
    const SegDesc &sg = a.seg[s];
    const int lb = g - sg.lb_begin;
    const uint32_t m = a.state[s].m;
    const uint32_t B1 = a.state[s].B1, c_gt1 = a.state[s].c_gt1;

    // Prologue: bucket of the second digit among the members of bucket B1.
    uint32_t B2, above2;
    pick_from_global<NB2>(a.G2 + s * NB2, static_cast<uint32_t>(sg.k) - c_gt1, h, sm, s_pick, B2, above2);
    if (lb == 0 && threadIdx.x == 0) {
        a.state[s].B2 = B2;
        a.state[s].c_gt2 = c_gt1 + above2;
    }
    const uint32_t P = (B1 << BITS2) | B2;  // 21-bit prefix of the threshold
    const R *Lv = static_cast<const R *>(a.L_val) + sg.l_base;
    uint32_t beg, end;
    list_range(m, lb, sg.lb_count, beg, end);

    uint32_t *h3 = h;
    for (int b = threadIdx.x; b < NB3; b += BLOCK) h3[b] = 0;
    __syncthreads();
    uint32_t def = 0;  // keys above the prefix: kept whatever the last digit is
    for (uint32_t i = beg + threadIdx.x; i < end; i += BLOCK) {
        const uint32_t key = key_of<VEC>(Lv[i]);
        const uint32_t p = key >> SH2;
        def += (p > P) ? 1u : 0u;
        if (p == P) atomicAdd(&h3[key & (NB3 - 1)], 1u);
    }
    __syncthreads();
    flush_bins<NB3>(h3, a.G3 + s * NB3);
    __syncthreads();
    block_suffix_inplace<NB3>(h3, sm);
    uint32_t *row = a.rows3 + static_cast<size_t>(g) * NB3;
    for (int b = threadIdx.x; b < NB3; b += BLOCK) row[b] = h3[b];
    uint32_t deftot;
    block_incl_scan(def, sm, &deftot);
    if (threadIdx.x == 0) a.ldef[g] = deftot;
}

template <int VEC> __global__ __launch_bounds__(BLOCK) void k_emit(Launch a) {
    using R = typename Raw<VEC>::type;
    __shared__ uint32_t h[NB3];
    __shared__ uint32_t wcnt[2][2][LU * NW];
    __shared__ uint32_t sm[NW];
    __shared__ double smd[NW];
    __shared__ uint32_t s_pick[2];
    __shared__ uint32_t s_off[2];
    __shared__ uint32_t s_flag;

    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int g = blockIdx.x;
    const int s = find_segment_by(a, g, false);
    const SegDesc &sg = a.seg[s];
    const int lb = g - sg.lb_begin;
    const uint32_t m = a.state[s].m;
    const uint32_t P = (a.state[s].B1 << BITS2) | a.state[s].B2;
    const uint32_t c_gt2 = a.state[s].c_gt2;
    const uint32_t kout = static_cast<uint32_t>(sg.k);

    // Prologue: last digit -> threshold key T and tie quota q; then this block's output
    // offsets = scan over the earlier list blocks of (#keys above T, #keys equal to T).
    uint32_t B3, above3;
    pick_from_global<NB3>(a.G3 + s * NB3, kout - c_gt2, h, sm, s_pick, B3, above3);
    const uint32_t T = (B3 < NB3) ? ((P << BITS3) | B3) : 0xFFFFFFFFu;
    const uint32_t q = kout - (c_gt2 + above3);
    {
        uint32_t gt = 0, eq = 0;
        if (static_cast<int>(threadIdx.x) < sg.lb_count && B3 < NB3) {
            const uint32_t *r = a.rows3 + static_cast<size_t>(sg.lb_begin + threadIdx.x) * NB3;
            const uint32_t above = (B3 + 1 < NB3) ? r[B3 + 1] : 0u;
            gt = a.ldef[sg.lb_begin + threadIdx.x] + above;
            eq = r[B3] - above;
        }
        uint32_t tot;
        const uint32_t inc_gt = block_incl_scan(gt, sm, &tot);
        const uint32_t inc_eq = block_incl_scan(eq, sm, &tot);
        if (static_cast<int>(threadIdx.x) == lb) {
            s_off[0] = inc_gt - gt;
            s_off[1] = inc_eq - eq;
        }
        __syncthreads();
    }
    uint32_t run_gt = s_off[0], run_eq = s_off[1];

    const int32_t *Li = a.L_idx + sg.l_base;
    const R *Lv = static_cast<const R *>(a.L_val) + sg.l_base;
    int32_t *oi = a.idx_out + sg.out_off;
    R *ov = static_cast<R *>(a.val_out) + sg.out_off;
    uint32_t beg, end;
    list_range(m, lb, sg.lb_count, beg, end);

    double acc = 0.0;
    int buf = 0;
    for (uint32_t t0 = beg; t0 < end; t0 += BLOCK * LU, buf ^= 1) {
        uint32_t raw[LU];
        int32_t id[LU];
        uint32_t pre_gt[LU], pre_eq[LU], cls[LU];  // cls: 0 below T, 1 equal, 2 above, 3 no element
#pragma unroll
        for (int j = 0; j < LU; ++j) {
            const uint32_t i = t0 + j * BLOCK + threadIdx.x;
            const bool valid = i < end;
            raw[j] = valid ? static_cast<uint32_t>(Lv[i]) : 0u;
            id[j] = valid ? Li[i] : 0;
            const uint32_t key = key_of<VEC>(raw[j]);
            const bool gt = valid && key > T, eq = valid && key == T;
            cls[j] = valid ? (gt ? 2u : (eq ? 1u : 0u)) : 3u;
            const uint64_t bg = __ballot(gt), be = __ballot(eq);
            pre_gt[j] = lanes_below(bg);
            pre_eq[j] = lanes_below(be);
            if (lane == 0) {
                wcnt[buf][0][j * NW + w] = __popcll(bg);
                wcnt[buf][1][j * NW + w] = __popcll(be);
            }
        }
        __syncthreads();
        const uint32_t cg = (lane < LU * NW) ? wcnt[buf][0][lane] : 0u;
        const uint32_t ce = (lane < LU * NW) ? wcnt[buf][1][lane] : 0u;
        const uint32_t ig = wave_incl_scan(cg), ie = wave_incl_scan(ce);
        const uint32_t tg = __shfl(ig, 63), te = __shfl(ie, 63);
#pragma unroll
        for (int j = 0; j < LU; ++j) {
            const uint32_t gt_before = run_gt + __shfl(ig - cg, j * NW + w) + pre_gt[j];
            const uint32_t eq_before = run_eq + __shfl(ie - ce, j * NW + w) + pre_eq[j];
            const bool keep = cls[j] == 2u || (cls[j] == 1u && eq_before < q);
            if (keep) {
                const uint32_t pos = gt_before + (eq_before < q ? eq_before : q);
                if (pos < kout) {
                    oi[pos] = id[j];
                    ov[pos] = static_cast<R>(raw[j]);
                }
            } else if (cls[j] != 3u) {
                const double xd = static_cast<double>(value_of<VEC>(raw[j]));
                acc = fma(xd, xd, acc);
            }
        }
        run_gt += tg;
        run_eq += te;
    }
    if (a.err_out == nullptr) return;

    // Error norm of the segment: the block that draws the last ticket adds the chunk partials,
    // then the list-block partials, in a fixed order.
    const double bsum = block_sum_f64(acc, smd);
    if (!publish_and_take_ticket(a.lerr + g, bsum, &a.state[s].ticket, sg.lb_count, &s_flag)) return;
    double part = 0.0;
    for (int cc = threadIdx.x; cc < sg.nchunks; cc += BLOCK) part += a.chunk_err[sg.chunk_begin + cc];
    for (int bb = threadIdx.x; bb < sg.lb_count; bb += BLOCK) part += coherent_load_f64(a.lerr + sg.lb_begin + bb);
    const double tot = block_sum_f64(part, smd);
    if (threadIdx.x == 0) a.err_out[s] = static_cast<float>(sqrt(tot));
}

// ------------------------------------------------------------------ decompress / streaming kernels
// Zero `bytes` bytes at dst.  [head, head + 16 * body16) is the 16-byte aligned body.
__global__ __launch_bounds__(BLOCK) void k_fill(unsigned char *dst, size_t bytes, size_t head, size_t body16) {
    uint4 *body = reinterpret_cast<uint4 *>(dst + head);
    const uint4 z = make_uint4(0, 0, 0, 0);
    const size_t stride = static_cast<size_t>(gridDim.x) * BLOCK;
    for (size_t i = static_cast<size_t>(blockIdx.x) * BLOCK + threadIdx.x; i < body16; i += stride) body[i] = z;
    if (blockIdx.x == 0) {  // ragged ends, byte-wise (at most 15 + 15 bytes)
        const size_t tail0 = head + body16 * 16;
        for (size_t i = threadIdx.x; i < head; i += BLOCK) dst[i] = 0;
        for (size_t i = tail0 + threadIdx.x; i < bytes; i += BLOCK) dst[i] = 0;
    }
}

template <typename R>
__global__ __launch_bounds__(BLOCK) void k_scatter(const int32_t *idx, const R *val, int64_t k, R *y, int64_t n) {
    const int64_t j = static_cast<int64_t>(blockIdx.x) * BLOCK + threadIdx.x;
    if (j >= k) return;
    const int64_t i = idx[j];
    if (i >= 0 && i < n) y[i] = val[j];
}

__global__ __launch_bounds__(BLOCK) void k_copy16(uint4 *dst, const uint4 *src, size_t n16) {
    const size_t stride = static_cast<size_t>(gridDim.x) * BLOCK;
    for (size_t i = static_cast<size_t>(blockIdx.x) * BLOCK + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

__global__ __launch_bounds__(BLOCK) void k_read16(const uint4 *src, size_t n16, uint32_t *sink) {
    const size_t stride = static_cast<size_t>(gridDim.x) * BLOCK;
    uint32_t f = 0;
    for (size_t i = static_cast<size_t>(blockIdx.x) * BLOCK + threadIdx.x; i < n16; i += stride) {
        const uint4 v = src[i];
        f ^= v.x ^ v.y ^ v.z ^ v.w;
    }
    if (f == 0x9E3779B9u) sink[0] = f;  // keeps the loads alive; practically never true
}

// ------------------------------------------------------------------ host side: plan and launch
inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

inline int elem_size(adatopk_dtype dt) { return dt == ADATOPK_F32 ? 4 : 2; }
inline bool dtype_ok(adatopk_dtype dt) { return dt == ADATOPK_F32 || dt == ADATOPK_BF16; }

int64_t chunk_elems(int64_t n_total, adatopk_dtype dt) {
    const int64_t tile = static_cast<int64_t>(BLOCK) * U * (16 / elem_size(dt));
    int64_t e = (n_total + CTARGET - 1) / CTARGET;
    if (e < tile) e = tile;
    e = (e + tile - 1) / tile * tile;
    const int64_t cap = (static_cast<int64_t>(1) << 30) / tile * tile;
    return e < cap ? e : cap;
}

int32_t list_blocks_cap(int32_t S) {
    int32_t c = 1024 / (S < 1 ? 1 : (S > MAXSEG ? MAXSEG : S));
    if (c < 16) c = 16;
    if (c > 256) c = 256;
    return c;
}

int32_t list_blocks(int64_t n, int32_t S) {
    int64_t b = (n + LB_ELEMS - 1) / LB_ELEMS;
    const int32_t cap = list_blocks_cap(S);
    if (b < 1) b = 1;
    return b > cap ? cap : static_cast<int32_t>(b);
}

struct Carve {
    size_t state, G1, G2, G3, rows1, chunk_err, rows3, ldef, lerr, L_idx, L_val, total;
};

// Workspace layout for up to max_chunks chunks, max_lb list blocks and n_total list slots.
Carve carve(int64_t max_chunks, int64_t max_lb, int64_t n_total, adatopk_dtype dt) {
    Carve c;
    size_t p = 0;
    auto take = [&](size_t bytes) {
        const size_t at = p;
        p = align_up(p + bytes, 256);
        return at;
    };
    c.state = take(sizeof(SegState) * MAXSEG);
    c.G1 = take(sizeof(uint32_t) * NB1 * MAXSEG);
    c.G2 = take(sizeof(uint32_t) * NB2 * MAXSEG);
    c.G3 = take(sizeof(uint32_t) * NB3 * MAXSEG);
    c.rows1 = take(sizeof(uint32_t) * NB1 * max_chunks);
    c.chunk_err = take(sizeof(double) * max_chunks);
    c.rows3 = take(sizeof(uint32_t) * NB3 * max_lb);
    c.ldef = take(sizeof(uint32_t) * max_lb);
    c.lerr = take(sizeof(double) * max_lb);
    c.L_idx = take(sizeof(int32_t) * static_cast<size_t>(n_total));
    c.L_val = take(static_cast<size_t>(elem_size(dt)) * static_cast<size_t>(n_total));
    c.total = p;
    return c;
}

void bounds_for(int64_t n_total, int32_t S, adatopk_dtype dt, int64_t *max_chunks, int64_t *max_lb) {
    const int64_t E = chunk_elems(n_total, dt);
    const int32_t batch = S > MAXSEG ? MAXSEG : (S < 1 ? 1 : S);
    *max_chunks = n_total / E + batch + 1;
    *max_lb = static_cast<int64_t>(batch) * list_blocks_cap(S);
}

// ---- stage timing (measurement hook)
constexpr int NSTAGE_C = 5, NSTAGE_D = 2;
const char *const kStageNames[NSTAGE_C + NSTAGE_D] = {"k_init", "k_hist1", "k_gather", "k_hist3",
                                                        "k_emit", "k_fill",  "k_scatter"};
bool g_measure = false;
bool g_events_made = false;
hipEvent_t g_ev_c[NSTAGE_C + 1], g_ev_d[NSTAGE_D + 1];
int g_rec_c = 0, g_rec_d = 0;  // events recorded by the latest timed call

inline void mark(hipEvent_t *ev, int *count, int slot, hipStream_t st) {
    if (!g_measure) return;
    if (hipEventRecord(ev[slot], st) == hipSuccess) *count = slot + 1;
}

template <int VEC> adatopk_status launch_batch(const Launch &a, int total_chunks, int total_lb, hipStream_t st) {
    g_rec_c = 0;
    mark(g_ev_c, &g_rec_c, 0, st);
    hipLaunchKernelGGL(k_init, dim3(a.S), dim3(BLOCK), 0, st, a);
    mark(g_ev_c, &g_rec_c, 1, st);
    if (total_chunks > 0) hipLaunchKernelGGL(k_hist1<VEC>, dim3(total_chunks), dim3(BLOCK), 0, st, a);
    mark(g_ev_c, &g_rec_c, 2, st);
    if (total_chunks > 0) hipLaunchKernelGGL(k_gather<VEC>, dim3(total_chunks), dim3(BLOCK), 0, st, a);
    mark(g_ev_c, &g_rec_c, 3, st);
    hipLaunchKernelGGL(k_hist3<VEC>, dim3(total_lb), dim3(BLOCK), 0, st, a);
    mark(g_ev_c, &g_rec_c, 4, st);
    hipLaunchKernelGGL(k_emit<VEC>, dim3(total_lb), dim3(BLOCK), 0, st, a);
    mark(g_ev_c, &g_rec_c, 5, st);
    return hipGetLastError() == hipSuccess ? ADATOPK_OK : ADATOPK_ERUNTIME;
}

adatopk_status compress_impl(const void *const *dense, const int64_t *n, const int64_t *k, int32_t S,
                             adatopk_dtype dt, int32_t *idx_out, void *val_out, const int64_t *out_offset,
                             float *err_out, void *workspace, size_t workspace_bytes, hipStream_t st) {
    if (!dtype_ok(dt) || S < 0) return ADATOPK_EINVAL;
    if (S == 0) return ADATOPK_OK;
    if (!dense || !n || !k || !out_offset) return ADATOPK_EINVAL;
    const int es = elem_size(dt);
    int64_t n_total = 0, k_total = 0;
    if (out_offset[0] != 0) return ADATOPK_EINVAL;
    for (int32_t s = 0; s < S; ++s) {
        if (n[s] < 0 || n[s] >= (static_cast<int64_t>(1) << 31) || k[s] < 0 || k[s] > n[s]) return ADATOPK_EINVAL;
        if (n[s] > 0 && (!dense[s] || reinterpret_cast<uintptr_t>(dense[s]) % es)) return ADATOPK_EINVAL;
        if (out_offset[s + 1] != out_offset[s] + k[s]) return ADATOPK_EINVAL;
        n_total += n[s];
        k_total += k[s];
    }
    if (k_total > 0 && (!idx_out || !val_out)) return ADATOPK_EINVAL;
    if (reinterpret_cast<uintptr_t>(idx_out) % 4 || reinterpret_cast<uintptr_t>(val_out) % es ||
        reinterpret_cast<uintptr_t>(err_out) % 4)
        return ADATOPK_EINVAL;
    const size_t need = adatopk_workspace_bytes(n_total, S, dt);
    if (!workspace || reinterpret_cast<uintptr_t>(workspace) % 256) return ADATOPK_EINVAL;
    if (workspace_bytes < need) return ADATOPK_EWORKSPACE;

    int64_t max_chunks, max_lb;
    bounds_for(n_total, S, dt, &max_chunks, &max_lb);
    const Carve cv = carve(max_chunks, max_lb, n_total, dt);
    char *ws = static_cast<char *>(workspace);
    const int64_t E = chunk_elems(n_total, dt);

    for (int32_t s0 = 0; s0 < S; s0 += MAXSEG) {
        Launch a{};
        a.S = (S - s0 < MAXSEG) ? S - s0 : MAXSEG;
        a.E = static_cast<int32_t>(E);
        a.state = reinterpret_cast<SegState *>(ws + cv.state);
        a.G1 = reinterpret_cast<uint32_t *>(ws + cv.G1);
        a.G2 = reinterpret_cast<uint32_t *>(ws + cv.G2);
        a.G3 = reinterpret_cast<uint32_t *>(ws + cv.G3);
        a.rows1 = reinterpret_cast<uint32_t *>(ws + cv.rows1);
        a.chunk_err = reinterpret_cast<double *>(ws + cv.chunk_err);
        a.rows3 = reinterpret_cast<uint32_t *>(ws + cv.rows3);
        a.ldef = reinterpret_cast<uint32_t *>(ws + cv.ldef);
        a.lerr = reinterpret_cast<double *>(ws + cv.lerr);
        a.L_idx = reinterpret_cast<int32_t *>(ws + cv.L_idx);
        a.L_val = ws + cv.L_val;
        a.idx_out = idx_out;
        a.val_out = val_out;
        a.err_out = err_out ? err_out + s0 : nullptr;
        int32_t chunks = 0, lbs = 0;
        int64_t l_base = 0;
        for (int32_t i = 0; i < a.S; ++i) {
            SegDesc &d = a.seg[i];
            const int32_t s = s0 + i;
            d.x = dense[s];
            d.out_off = out_offset[s];
            d.l_base = l_base;
            d.n = static_cast<int32_t>(n[s]);
            d.k = static_cast<int32_t>(k[s]);
            d.chunk_begin = chunks;
            d.nchunks = static_cast<int32_t>((n[s] + E - 1) / E);
            d.lb_begin = lbs;
            d.lb_count = list_blocks(n[s], S);
            d.aligned16 = (reinterpret_cast<uintptr_t>(dense[s]) % 16 == 0) ? 1u : 0u;
            chunks += d.nchunks;
            lbs += d.lb_count;
            l_base += n[s];
        }
        if (chunks > max_chunks || lbs > max_lb) return ADATOPK_ERUNTIME;  // planner invariant
        const adatopk_status rc = (dt == ADATOPK_F32) ? launch_batch<4>(a, chunks, lbs, st)
                                                      : launch_batch<8>(a, chunks, lbs, st);
        if (rc != ADATOPK_OK) return rc;
    }
    return ADATOPK_OK;
}

int grid_for(size_t work_items, int per_thread) {
    size_t b = (work_items + static_cast<size_t>(BLOCK) * per_thread - 1) / (static_cast<size_t>(BLOCK) * per_thread);
    if (b < 1) b = 1;
    if (b > 4096) b = 4096;
    return static_cast<int>(b);
}

adatopk_status fill_impl(void *dst, size_t bytes, hipStream_t st) {
    if (bytes == 0) return ADATOPK_OK;
    size_t head = (16 - reinterpret_cast<uintptr_t>(dst) % 16) % 16;
    if (head > bytes) head = bytes;
    const size_t body16 = (bytes - head) / 16;
    hipLaunchKernelGGL(k_fill, dim3(grid_for(body16, 4)), dim3(BLOCK), 0, st, static_cast<unsigned char *>(dst),
                       bytes, head, body16);
    return hipGetLastError() == hipSuccess ? ADATOPK_OK : ADATOPK_ERUNTIME;
}

}  // namespace

// ------------------------------------------------------------------ C ABI
extern "C" {

size_t adatopk_workspace_bytes(int64_t n_total, int32_t num_segments, adatopk_dtype dt) {
    if (n_total < 0 || num_segments < 1 || !dtype_ok(dt)) return 0;
    int64_t max_chunks, max_lb;
    bounds_for(n_total, num_segments, dt, &max_chunks, &max_lb);
    return carve(max_chunks, max_lb, n_total, dt).total;
}

adatopk_status adatopk_compress(const void *dense, int64_t n, adatopk_dtype dt, int64_t k, int32_t *idx_out,
                                void *val_out, float *err_norm_out, void *workspace, size_t workspace_bytes,
                                void *hip_stream) {
    const void *ptrs[1] = {dense};
    const int64_t off[2] = {0, k};
    return compress_impl(ptrs, &n, &k, 1, dt, idx_out, val_out, off, err_norm_out, workspace, workspace_bytes,
                         static_cast<hipStream_t>(hip_stream));
}

adatopk_status adatopk_compress_segmented(const void *const *dense, const int64_t *n, const int64_t *k, int32_t S,
                                          adatopk_dtype dt, int32_t *idx_out, void *val_out,
                                          const int64_t *out_offset, float *err_norm_out, void *workspace,
                                          size_t workspace_bytes, void *hip_stream) {
    return compress_impl(dense, n, k, S, dt, idx_out, val_out, out_offset, err_norm_out, workspace, workspace_bytes,
                         static_cast<hipStream_t>(hip_stream));
}

adatopk_status adatopk_decompress(const int32_t *idx, const void *val, int64_t k, adatopk_dtype dt, void *dense_out,
                                  int64_t n, void *hip_stream) {
    if (!dtype_ok(dt) || n < 0 || k < 0 || n >= (static_cast<int64_t>(1) << 31)) return ADATOPK_EINVAL;
    const int es = elem_size(dt);
    if (n > 0 && (!dense_out || reinterpret_cast<uintptr_t>(dense_out) % es)) return ADATOPK_EINVAL;
    if (k > 0 && (!idx || !val || reinterpret_cast<uintptr_t>(idx) % 4 || reinterpret_cast<uintptr_t>(val) % es))
        return ADATOPK_EINVAL;
    if (n == 0) return ADATOPK_OK;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    g_rec_d = 0;
    mark(g_ev_d, &g_rec_d, 0, st);
    const adatopk_status rc = fill_impl(dense_out, static_cast<size_t>(n) * es, st);
    if (rc != ADATOPK_OK) return rc;
    mark(g_ev_d, &g_rec_d, 1, st);
    if (k > 0) {
        const int grid = static_cast<int>((k + BLOCK - 1) / BLOCK);
        if (dt == ADATOPK_F32)
            hipLaunchKernelGGL(k_scatter<uint32_t>, dim3(grid), dim3(BLOCK), 0, st, idx,
                               static_cast<const uint32_t *>(val), k, static_cast<uint32_t *>(dense_out), n);
        else
            hipLaunchKernelGGL(k_scatter<uint16_t>, dim3(grid), dim3(BLOCK), 0, st, idx,
                               static_cast<const uint16_t *>(val), k, static_cast<uint16_t *>(dense_out), n);
    }
    mark(g_ev_d, &g_rec_d, 2, st);
    return hipGetLastError() == hipSuccess ? ADATOPK_OK : ADATOPK_ERUNTIME;
}

// ---- measurement hooks
adatopk_status adatopk_measure_enable(int32_t on) {
    if (on && !g_events_made) {
        for (int i = 0; i <= NSTAGE_C; ++i)
            if (hipEventCreate(&g_ev_c[i]) != hipSuccess) return ADATOPK_ERUNTIME;
        for (int i = 0; i <= NSTAGE_D; ++i)
            if (hipEventCreate(&g_ev_d[i]) != hipSuccess) return ADATOPK_ERUNTIME;
        g_events_made = true;
    }
    g_measure = on != 0;
    g_rec_c = g_rec_d = 0;
    return ADATOPK_OK;
}

int32_t adatopk_measure_stage_count(void) { return NSTAGE_C + NSTAGE_D; }

const char *adatopk_measure_stage_name(int32_t stage) {
    return (stage >= 0 && stage < NSTAGE_C + NSTAGE_D) ? kStageNames[stage] : "";
}

adatopk_status adatopk_measure_read(float *ms_out) {
    if (!ms_out || !g_events_made) return ADATOPK_EINVAL;
    for (int i = 0; i < NSTAGE_C + NSTAGE_D; ++i) ms_out[i] = -1.0f;
    if (g_rec_c > 0 && hipEventSynchronize(g_ev_c[g_rec_c - 1]) != hipSuccess) return ADATOPK_ERUNTIME;
    for (int i = 0; i + 1 < g_rec_c; ++i)
        if (hipEventElapsedTime(&ms_out[i], g_ev_c[i], g_ev_c[i + 1]) != hipSuccess) return ADATOPK_ERUNTIME;
    if (g_rec_d > 0 && hipEventSynchronize(g_ev_d[g_rec_d - 1]) != hipSuccess) return ADATOPK_ERUNTIME;
    for (int i = 0; i + 1 < g_rec_d; ++i)
        if (hipEventElapsedTime(&ms_out[NSTAGE_C + i], g_ev_d[i], g_ev_d[i + 1]) != hipSuccess)
            return ADATOPK_ERUNTIME;
    g_rec_c = g_rec_d = 0;
    return ADATOPK_OK;
}

adatopk_status adatopk_measure_copy(void *dst, const void *src, size_t bytes, void *hip_stream) {
    if (!dst || !src || bytes % 16 || reinterpret_cast<uintptr_t>(dst) % 16 || reinterpret_cast<uintptr_t>(src) % 16)
        return ADATOPK_EINVAL;
    if (bytes == 0) return ADATOPK_OK;
    hipLaunchKernelGGL(k_copy16, dim3(grid_for(bytes / 16, 4)), dim3(BLOCK), 0, static_cast<hipStream_t>(hip_stream),
                       static_cast<uint4 *>(dst), static_cast<const uint4 *>(src), bytes / 16);
    return hipGetLastError() == hipSuccess ? ADATOPK_OK : ADATOPK_ERUNTIME;
}

adatopk_status adatopk_measure_read_only(const void *src, size_t bytes, uint32_t *sink, void *hip_stream) {
    if (!src || !sink || bytes % 16 || reinterpret_cast<uintptr_t>(src) % 16) return ADATOPK_EINVAL;
    if (bytes == 0) return ADATOPK_OK;
    hipLaunchKernelGGL(k_read16, dim3(grid_for(bytes / 16, 4)), dim3(BLOCK), 0, static_cast<hipStream_t>(hip_stream),
                       static_cast<const uint4 *>(src), bytes / 16, sink);
    return hipGetLastError() == hipSuccess ? ADATOPK_OK : ADATOPK_ERUNTIME;
}

adatopk_status adatopk_measure_fill(void *dst, size_t bytes, void *hip_stream) {
    if (!dst || bytes % 16 || reinterpret_cast<uintptr_t>(dst) % 16) return ADATOPK_EINVAL;
    return fill_impl(dst, bytes, static_cast<hipStream_t>(hip_stream));
}

}  // extern "C"
