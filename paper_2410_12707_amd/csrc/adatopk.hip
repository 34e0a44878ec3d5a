// AdaTopK compress / decompress for MI355X (gfx950, wave64): kernels, launch planner and C ABI.
//
// Operation (paper Sec. 5.1, Top-K sparsification figure): keep the k entries of largest
// absolute value of a flat tensor as (int32 index, value) pairs; decompression writes them
// back into zeros.  Sec. 5.2 (Eq. "adacompress") gives every slow link its own ratio, so
// the launch is segmented: S tensors, each with its own k, one launch per pass for all.
//
// Method.  key(x) = bits(x) with the sign cleared (a 16-bit pattern, bf16 or fp16, is moved to
// the upper half, so all types share one 31-bit key).  The exact k-th largest key T is found
// with one read of the input when a sample of it predicts where T lies, and with two otherwise.
// A tensor is cut into chunks of whole tiles, one workgroup per chunk in the kernels that read it:
//   k_scan<spec>   (tensors of 2^20 elements and more, k up to 21 % of them)  Prologue, every
//             workgroup alike: a histogram of 8 to 32 thousand sampled keys gives two ranks that
//             bracket the k-th key by five standard deviations of the sampling noise; the key
//             window starts at the lower one and spans the bracket in 2048 bins.  Then the one
//             read of the input: every element with a key inside or above the window goes, in
//             index order, into the candidate list of its chunk (LDS stage, full-width stores)
//             and is counted in its window bin (one row of suffix sums per chunk); squares of the
//             others are summed in fp64 per chunk.  A chunk with more candidates than its list
//             holds (a quarter of its elements) is read from the input again by the later kernels
//   k_hist1   sums the chunks' candidate counts: the guess holds when at least k keys reached the
//             window and fewer than k lie above its bins.  Then it returns at once, and so does the
//             kernel after it.  Otherwise (and for tensors that never speculate) it is the first of
//             the two exact passes: per-chunk histogram of the top 11 key bits, rows of suffix sums
//   k_scan<exact>  prologue: column sums of those rows -> the bucket of the k-th key, which is the
//             window; then the same scan as above
//   k_refine  (fp32 only) prologue: column sums of the window rows -> window bin Bw of the k-th
//             key.  Over the chunk's candidates: histogram of the position inside bin Bw (at most
//             10 bits: the last digit) into G3, one row of suffix sums per list part
//   k_emit    prologue: G3 -> threshold key T and tie quota q (16-bit types: a window bin is one
//             pattern, so T comes from the window rows and k_refine is not launched); output
//             offsets from the rows of the earlier chunks.  Stable compaction into idx_out /
//             val_out (key > T, plus the first q keys equal to T).  The tensor's last workgroup
//             adds up the error norm from the partial sums the earlier kernels stored, in a fixed order
// Cross-block order comes only from counts that an EARLIER kernel stored and that every block
// of the next kernel scans for itself: no block waits for another block (no launch can hang),
// no block needs a release fence (on this chip an agent-scope fence writes back the L2 of its
// XCD, about 1.5 us per workgroup, serialised), and every result, the fp64 error sum included,
// is the same from run to run.
//
// Decompress: k_fill (16-byte zero stores) then k_scatter; for ascending indices k_merge does
// both in one kernel, every workgroup filling its own span and writing the entries that fall in it
// (k_merge_seg: the same for all tensors of a segmented batch in one launch); k_scatter_add adds
// the pairs into an existing tensor.
//
// Tensors of at most one register tile (8192 elements) skip all of the above: k_small selects
// and writes one tensor per workgroup in a single launch.
//
// Outputs can be laid out as one wire message (header, indices, values); indices are stored as
// int32 or, for the paper's own accounting (Sec. 5.2), int64.
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <hip/hip_fp16.h>

#include <stdint.h>
#include <stddef.h>
#include <string.h>

#include <atomic>

#include "adatopk.h"
#include "wire_layout.h"
#ifdef ADATOPK_MEASURE_BUILD
#include "adatopk_measure.h"
#endif

// Scratch of adatopk_compress_noalloc: the workspace of a compress call, resident in every GPU the
// library is loaded on for the life of the process.  In host code this name is a stand-in, not a
// device address: the address is asked for once per device (scratch_of_current_device) and only
// that pointer is handed to kernels.
#define ADATOPK_NOALLOC_SCRATCH_BYTES (static_cast<size_t>(64) << 20)
static __device__ __align__(256) unsigned char scratch[ADATOPK_NOALLOC_SCRATCH_BYTES];

namespace {

// Launch-shape constants.
constexpr int BLOCK = 512;            // threads per workgroup
constexpr int NW = BLOCK / 64;        // wavefronts per workgroup
constexpr int EPT = 16;               // input elements per thread per tile
constexpr int TILE = BLOCK * EPT;     // input elements per workgroup per tile, both dtypes
constexpr int LU = 4;                 // list elements per thread per tile in the list kernels
constexpr int BITS1 = 11;             // top digit of the key, counted by k_hist1
constexpr int NB1 = 1 << BITS1;
constexpr int SH1 = 31 - BITS1;       // key >> SH1 = top digit
constexpr int NC1 = 64;               // coarse boundaries of the top digit: every (NB1 / NC1)-th suffix sum
constexpr int FINE1 = NB1 / NC1;      // fine bins per coarse interval
constexpr int NBW = 2048;             // bins of the key window that the scan pass counts its candidates in
constexpr int NCW = 64;               // coarse boundaries of the window bins
constexpr int BITS3 = 10;             // the last digit: position of a key inside its window bin
constexpr int NB3 = 1 << BITS3;
constexpr int BITS2 = 31 - BITS1 - BITS3;  // the one-workgroup path selects on the fixed digits BITS1 / BITS2 / BITS3
constexpr int NB2 = 1 << BITS2;
constexpr int SH2 = BITS3;
constexpr int SAMPLE_ELEMS = 32768;   // elements of a tensor that the speculative pass looks at first
constexpr int SAMPLE_SH = 19;         // sample histogram: bin = key >> SAMPLE_SH ...
constexpr int NSB = 1 << (31 - SAMPLE_SH);  // ... 4096 bins, 16 to the binade (4.4 % in value)
constexpr int LIST_DIV = 4;           // a chunk's candidate list holds up to a quarter of the chunk
constexpr int MAXSUB = 8;             // parts that the list kernels cut a chunk's candidates into, at most ...
constexpr int MAXSUB_ONE = 4;         // ... and for a single tensor, whose chunks are a quarter as long as a large batch's
constexpr int SUB_ENTRIES = 8192;     // ... so that a part has about this many
constexpr int MAXSEG = 64;            // segments per launch (the table travels as kernel arguments)
constexpr int CTARGET = 512;          // chunks of a launch of several tensors, at most (two workgroups per compute unit)
// ... and of a single tensor: one workgroup per compute unit.  Half the rows for every prologue to
// sum; a batch of tensors with unequal keep counts wants the finer split, whose workgroups even out.
constexpr int CTARGET_ONE = 256;
constexpr int64_t SPEC_MIN_N = 1 << 20;    // tensors below this are not worth a speculative pass
constexpr double SPEC_MIN_EXPECTED = 32.0; // ... nor are keep counts that leave fewer than this many kept elements in the largest sample
constexpr double SPEC_GOOD_EXPECTED = 96.0; // a smaller sample will do when it still expects this many (fp32)
constexpr double SPEC_GOOD_EXPECTED_16 = 64.0; // 16-bit types: their sample costs twice the instructions per dword, and the wider window
                                              // of a smaller sample costs them nothing (a window bin is one pattern, no last digit to refine)
constexpr double SPEC_SIGMAS = 5.0;        // width of the sample's rank bracket in standard deviations, upper side
constexpr double SPEC_SIGMAS_LOW = 3.5;    // ... and lower side: every key down to there is a candidate, so this one costs
constexpr int64_t SPEC_MAX_KEEP_PERCENT = 21;  // beyond this the candidates (k and the bracket's margin) may not fit a quarter of a chunk
constexpr size_t MERGE_SPANS = 1024;       // output spans aimed at by the one-kernel decompress
constexpr int64_t MERGE_DENSE_RATIO = 32;  // k > n / 32 takes the LDS-built variant of the one-kernel decompress
constexpr size_t MERGE_MIN_SPAN = 16384;   // bytes; smaller outputs use fewer workgroups
constexpr size_t MERGE_MAX_SPAN = 98304;   // bytes; larger outputs use more workgroups
static_assert(LU * NW <= 64, "per-tile wave counts must fit one wavefront scan");
static_assert(NB1 % BLOCK == 0 && NBW % BLOCK == 0 && NB3 % BLOCK == 0 && NSB % BLOCK == 0, "bins split evenly over threads");
static_assert(CTARGET <= BLOCK, "k_emit scans the chunks of a segment with one thread each");
static_assert(BLOCK % 64 == 0, "whole wavefronts");
static_assert(TILE % (LIST_DIV * BLOCK * LU) == 0, "a chunk's list capacity is whole list tiles");

// The key window of a scan pass: keys below lo are dropped for sure, a key >= lo falls into window
// bin min((key - lo) >> shw, NBW - 1).  The last bin is open-ended.
struct SegState {  // one per segment; 64 bytes
    uint32_t loA, shwA;   // window of the speculative pass (written by its first chunk's workgroup)
    uint32_t loB, shwB;   // window of the exact pass (likewise)
    uint32_t Bw, c_gtw;   // window bin that holds the k-th key, #keys in the bins above it (written by k_refine)
    uint32_t spec_held;   // the speculative pass bracketed the k-th key (written by k_hist1, which always runs)
    uint32_t pad[9];
};
static_assert(sizeof(SegState) == 64, "state record size");

// The first eight words of a state record in two 16-byte loads (one memory round trip; field by field, the
// window's fields are asked for only after spec_held has arrived).
struct SegStateWords {
    uint32_t loA, shwA, loB, shwB, Bw, c_gtw, spec_held;
};
__device__ __forceinline__ SegStateWords read_state(const SegState *st) {
    const uint4 a = reinterpret_cast<const uint4 *>(st)[0], b = reinterpret_cast<const uint4 *>(st)[1];
    return SegStateWords{a.x, a.y, a.z, a.w, b.x, b.y, b.z};
}

constexpr uint32_t FLAG_ALIGNED4 = 1u;  // tensor base is 4-byte aligned (always for fp32): dword loads allowed
constexpr uint32_t FLAG_SPEC = 2u;      // the speculative pass runs for this tensor
struct SegDesc {
    const void *x;       // device pointer of the tensor
    int64_t out_off;     // first output slot of this segment; in wire mode the byte offset of its index section
    int32_t n, k;
    int32_t chunk_begin, nchunks;  // its chunks are workgroups [chunk_begin, chunk_begin + nchunks) of every compress kernel
    uint32_t flags;
    uint32_t r_lo, r_hi; // speculative pass: ranks in the sample (counted from the largest key) that bracket the k-th key
    uint32_t sample_batches;  // ... and the sample's size in batches of SAMPLE_BATCH dword loads per thread
};

struct Launch {
    SegDesc seg[MAXSEG];
    int32_t S;
    int32_t E;      // elements per chunk (multiple of the tile)
    uint32_t cap;   // list slots per chunk (E / LIST_DIV)
    uint32_t sub;   // workgroups per chunk in the list kernels (1 .. MAXSUB): long candidate lists are cut into parts
    uint32_t idx64;
    uint32_t wire;  // outputs are wire messages in one buffer (idx_out): values follow the padded index section
    SegState *state;
    uint32_t *G3;                 // [MAXSEG][NB3] global histogram of the last digit
    uint32_t *rows1, *coarse1;    // [chunks][NB1], [chunks][NC1]: suffix sums of the chunks' top-digit histograms (k_hist1)
    uint32_t *rowsW, *coarseW;    // [chunks][NBW], [chunks][NCW]: the same for the window bins of the candidates (k_scan)
    uint2 *cpairA;                // [chunks] speculative pass only: #candidates, #candidates in the open-ended last bin
    uint32_t *cnt;                // [chunks] #candidates of the chunk; more than cap: the list is incomplete
    double *chunk_err;            // [chunks] sum of squares of the chunk's elements below the window
    uint32_t *rows3;              // [chunks * sub][NB3] suffix sums of the last digit inside the k-th key's window bin
    uint32_t *ldef;               // [chunks * sub] #candidates in the window bins above that bin
    double *lerr;                 // [chunks * sub] squares of the candidates in the window bins below it
    int32_t *L_idx;               // [chunks][cap] candidate lists, one region per chunk
    void *L_val;
    void *idx_out;     // int32 entries, or int64 when idx64 is set (the paper's index width, Sec. 5.2)
    void *val_out;
    float *err_out;
};
static_assert(sizeof(Launch) <= 4096, "kernel arguments stay within 4 KB");

// Where a segment's k pairs go.  Plain mode: element out_off of the idx / val arrays.  Wire mode:
// byte out_off of the message buffer holds the indices, the values start at the next multiple of
// 16 bytes behind them.
struct OutPtrs {
    int32_t *i32;
    int64_t *i64;
    void *val;
};
__device__ __forceinline__ OutPtrs out_ptrs(void *idx_out, void *val_out, int64_t out_off, uint32_t k, bool idx64,
                                            bool wire, int elem_bytes) {
    OutPtrs o;
    if (wire) {
        char *base = static_cast<char *>(idx_out) + out_off;
        const size_t idx_bytes = (static_cast<size_t>(k) * (idx64 ? 8 : 4) + 15) / 16 * 16;
        o.i32 = reinterpret_cast<int32_t *>(base);
        o.i64 = reinterpret_cast<int64_t *>(base);
        o.val = base + idx_bytes;
    } else {
        o.i32 = static_cast<int32_t *>(idx_out) + out_off;
        o.i64 = static_cast<int64_t *>(idx_out) + out_off;
        o.val = static_cast<char *>(val_out) + out_off * elem_bytes;
    }
    return o;
}

// ------------------------------------------------------------------ element access
// VEC tags the dtype: 4 = fp32 (one element per dword), 8 = bf16 and 9 = fp16 (two per dword, low
// half first).  VEC / 4 is the number of elements in a dword; the two 16-bit types differ only in
// how a pattern widens to fp32 (for the error norm): both order by their low 15 bits.
constexpr int TAG_F32 = 4, TAG_BF16 = 8, TAG_F16 = 9;
template <int VEC> struct Raw;
template <> struct Raw<TAG_F32> { using type = uint32_t; };
template <> struct Raw<TAG_BF16> { using type = uint16_t; };
template <> struct Raw<TAG_F16> { using type = uint16_t; };

template <int VEC> __device__ __forceinline__ uint32_t key_of(uint32_t raw) {
    return VEC == TAG_F32 ? (raw & 0x7FFFFFFFu) : ((raw & 0x7FFFu) << 16);
}
template <int VEC> __device__ __forceinline__ float value_of(uint32_t raw) {
    if (VEC == TAG_F16) return __half2float(__ushort_as_half(static_cast<unsigned short>(raw)));  // exact
    return __uint_as_float(VEC == TAG_F32 ? raw : (raw << 16));
}
// Element h of a loaded dword, as the raw pattern of one element.
template <int VEC> __device__ __forceinline__ uint32_t elem_of(uint32_t dword, int h) {
    return VEC == TAG_F32 ? dword : ((dword >> (16 * h)) & 0xFFFFu);
}

typedef uint32_t dword4 __attribute__((ext_vector_type(4)));

// Streaming layout of the two full-input kernels.  A tile is TILE consecutive elements; wave w
// of the workgroup owns the w-th contiguous 1/NW of it and reads it as SLOTS dword loads of
// 64 consecutive dwords each (256 contiguous bytes per wave-level load).  Index order inside
// a wave is therefore: slot, then lane, then half-word - which makes the lane mask of a
// per-slot compare a bitmap in index order.
template <int VEC> struct Stream {
    static constexpr int EPD = VEC / 4;        // elements per dword
    static constexpr int SLOTS = EPT / EPD;    // dword loads per thread per tile
    // first element of (wave, slot, lane) in the tile that starts at element t0
    static __device__ __forceinline__ int64_t first_elem(int64_t t0, int slot) {
        const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
        return t0 + (static_cast<int64_t>(w * SLOTS + slot) * 64 + lane) * EPD;
    }
    // whole tile in range, base 4-byte aligned: dword loads, nontemporal.  The input is streamed
    // through twice and is as large as the caches or larger; loaded nontemporally it does not
    // displace what the call does reuse (the per-chunk rows, the candidate list) nor the output of
    // the previous call that is still draining to memory (measured: 83.7 -> 76.6 us per step on
    // the 100 MB tensor, 636 -> 554 us on the 805 MB batch).
    static __device__ __forceinline__ void load_fast(const void *x, int64_t t0, uint32_t (&dw)[SLOTS]) {
        const uint32_t *p = static_cast<const uint32_t *>(x) + first_elem(t0, 0) / EPD;
#pragma unroll
        for (int e = 0; e < SLOTS; ++e) dw[e] = __builtin_nontemporal_load(p + e * 64);
    }
    // The same tile with 16-byte loads, thread t taking the t-th, (BLOCK + t)-th ... 16 bytes: for a
    // kernel that does not care which lane holds which element (the histogram).  Base 16-byte aligned.
    static __device__ __forceinline__ void load_wide(const void *x, int64_t t0, uint32_t (&dw)[SLOTS]) {
        static_assert(SLOTS % 4 == 0, "whole 16-byte loads");
        const dword4 *p = reinterpret_cast<const dword4 *>(static_cast<const uint32_t *>(x) + t0 / EPD) + threadIdx.x;
#pragma unroll
        for (int j = 0; j < SLOTS / 4; ++j) {
            const dword4 v = __builtin_nontemporal_load(p + j * BLOCK);
            dw[4 * j] = v.x;
            dw[4 * j + 1] = v.y;
            dw[4 * j + 2] = v.z;
            dw[4 * j + 3] = v.w;
        }
    }
    // ragged tile or misaligned bf16 base: element-wise, guarded; valid[e] has bit h set when
    // element h of slot e is below `end`
    static __device__ __forceinline__ void load_slow(const void *x, int64_t t0, int64_t end, uint32_t (&dw)[SLOTS],
                                                     uint32_t (&valid)[SLOTS]) {
        using R = typename Raw<VEC>::type;
        const R *p = static_cast<const R *>(x);
#pragma unroll
        for (int e = 0; e < SLOTS; ++e) {
            const int64_t i0 = first_elem(t0, e);
            uint32_t d = 0, v = 0;
#pragma unroll
            for (int h = 0; h < EPD; ++h)
                if (i0 + h < end) {
                    d |= static_cast<uint32_t>(p[i0 + h]) << (16 * h);
                    v |= 1u << h;
                }
            dw[e] = d;
            valid[e] = v;
        }
    }
};

// ------------------------------------------------------------------ wave / block helpers
__device__ __forceinline__ uint32_t lanes_below(uint64_t mask) {
    return __builtin_amdgcn_mbcnt_hi(static_cast<uint32_t>(mask >> 32),
                                     __builtin_amdgcn_mbcnt_lo(static_cast<uint32_t>(mask), 0u));
}

// base + number of set bits of mask in lanes below this one (the add rides on the mbcnt pair)
__device__ __forceinline__ uint32_t lanes_below_plus(uint64_t mask, uint32_t base) {
    return __builtin_amdgcn_mbcnt_hi(static_cast<uint32_t>(mask >> 32),
                                     __builtin_amdgcn_mbcnt_lo(static_cast<uint32_t>(mask), base));
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

// Counts that lane 0 of every wavefront has put into cnt[0 .. NW) before a barrier: the sum over the
// wavefronts before this one and the sum over all.  Lanes 0 .. NW-1 load the counts in wavefront order
// and scan them with row shifts inside the vector unit (NW <= 16, one row); the two results are read out
// of the scanned lanes into scalar registers.  A dozen instructions, where selecting every count by
// "is that wavefront before mine" took about fifty in the streaming loop of k_gather.
template <int DPP_CTRL> __device__ __forceinline__ uint32_t row_shr_add(uint32_t v) {
    return v + static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(v), DPP_CTRL, 0xF, 0xF, true));
}
__device__ __forceinline__ void wave_counts(const uint32_t *cnt, uint32_t &before, uint32_t &total) {
    static_assert(NW <= 16, "the scan stays inside one row of 16 lanes");
    const uint32_t w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    uint32_t v = cnt[threadIdx.x & (NW - 1)];
    v = row_shr_add<0x111>(v);                // row_shr:1
    if (NW > 2) v = row_shr_add<0x112>(v);    // row_shr:2
    if (NW > 4) v = row_shr_add<0x114>(v);    // row_shr:4
    if (NW > 8) v = row_shr_add<0x118>(v);    // row_shr:8
    total = static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(v), NW - 1));
    const uint32_t prev = static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(v), w ? w - 1 : 0));
    before = w ? prev : 0u;
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

// One count per active lane into h[bin].  Lanes of a wavefront that hit the same LDS word are
// served one after the other; with most of the 64 lanes on one word (a constant or mostly-zero
// tensor, sorted data) a histogram pass gets several times slower.  So when at least half of the
// wavefront is active and at least a quarter of it shares the bin of the first active lane, those
// lanes are counted with a single add.  Only the lanes that execute the call take part in it.
__device__ __forceinline__ void hist_add(uint32_t *h, uint32_t bin, bool active) {
    const uint64_t act = __ballot(active);
    if (__popcll(act) >= 32) {  // wave-uniform
        const int leader = __ffsll(static_cast<unsigned long long>(act)) - 1;
        const uint32_t lbin = __builtin_amdgcn_readlane(bin, leader);
        const uint64_t same = __ballot(active && bin == lbin);
        if (__popcll(same) >= 16) {
            if (static_cast<int>(threadIdx.x & 63) == leader) atomicAdd(&h[lbin], static_cast<uint32_t>(__popcll(same)));
            active = active && bin != lbin;
        }
    }
    if (active) atomicAdd(&h[bin], 1u);
}

// Histogram counts of a wavefront that works through dense, ordered data (a chunk that is read
// again from the input because nearly all of it are candidates: a constant tensor, sorted values):
// the lanes then hit one bin after another, and hist_add's two ballots, leader search and four
// branches per element are the whole cost of the pass.  A run keeps the current bin and the counts
// owed to it in scalar registers; lanes on that bin cost one compare and one ballot, the LDS add
// happens when the bin changes and in flush().  Lanes on neither the old nor the new bin of a step
// add for themselves.  Every lane of the wavefront has to make every call (no divergent callers).
struct BinRun {
    uint32_t ref = 0xFFFFFFFFu;  // wave-uniform: the bin of the run (no bin is that large)
    uint32_t pend = 0;           // wave-uniform: counts not yet added to it
    // (h: the histogram in LDS, as a plain pointer or as one that names its address space)
    template <typename P> static __device__ __forceinline__ void bin_add(P h, uint32_t bin, uint32_t count) {
        __hip_atomic_fetch_add(&h[bin], count, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    template <typename P> __device__ __forceinline__ void flush(P h) {
        if (pend != 0 && (threadIdx.x & 63) == 0) bin_add(h, ref, pend);
        pend = 0;
    }
    template <typename P> __device__ __forceinline__ void add(P h, uint32_t bin, bool active) {
        const uint64_t act = __ballot(active);
        const uint64_t same = __ballot(active && bin == ref);
        pend += static_cast<uint32_t>(__popcll(same));
        if (same != act) {  // wave-uniform: a lane is on another bin, the run moves there
            flush(h);
            const int leader = __ffsll(static_cast<unsigned long long>(act & ~same)) - 1;
            ref = __builtin_amdgcn_readlane(bin, leader);
            const uint64_t moved = __ballot(active && bin == ref);
            pend = static_cast<uint32_t>(__popcll(moved));
            if (active && bin != ref && !((same >> (threadIdx.x & 63)) & 1ull)) bin_add(h, bin, 1u);
        }
    }
};

// Adds the non-zero bins of an LDS histogram into a global one.
template <int NB> __device__ __forceinline__ void flush_bins(const uint32_t *h, uint32_t *G) {
    for (int b = threadIdx.x; b < NB; b += BLOCK) {
        const uint32_t c = h[b];
        if (c) __hip_atomic_fetch_add(&G[b], c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}
// Segment that owns workgroup g: the last one whose first chunk is <= g.  One lane per table entry
// and one ballot instead of a loop of dependent scalar loads, which costs about 0.1 us per segment.
static_assert(MAXSEG <= 64, "one lane per segment");
__device__ __forceinline__ int find_segment(const Launch &a, int g) {
    if (a.S == 1) return 0;
    const int lane = threadIdx.x & 63;
    int begin = 0x7FFFFFFF;
    if (lane < a.S) begin = a.seg[lane].chunk_begin;
    const uint64_t owner_or_before = __ballot(g >= begin);  // begins never decrease and the first is 0
    return 63 - __builtin_clzll(owner_or_before | 1ull);
}

// An index the compiler knows nothing about.  For loads that are to be issued whatever a condition says
// (an element past the end reads a valid stand-in and the value is dropped afterwards): if the compiler can
// connect the stand-in with the condition it turns the load back into a guarded one, in a branch of its
// own, and loads in neighbouring branches were seen to wait for one another.
__device__ __forceinline__ uint32_t opaque(uint32_t i) {
    asm("" : "+v"(i));
    return i;
}
// All ones if keep, else zero, as a value the compiler cannot trace back to the condition: and-ing a loaded
// value with it drops the value without making the load depend on the condition.
__device__ __forceinline__ uint32_t keep_mask(bool keep) { return opaque(keep ? 0xFFFFFFFFu : 0u); }

// Bucket search on per-block rows of suffix sums.  rows[r][NB] holds, for block r, the number of
// its keys whose digit is >= d at entry d; coarse[r][NC] repeats every (NB / NC)-th entry
// contiguously.  The column sums over the nrows rows are the global suffix sums S[d], non-increasing
// in d, and the bucket is B = max d with S[d] >= krem.  Step A sums the NC coarse columns and finds
// the coarse interval, step B sums its NB / NC fine columns (and, aside, the part of those sums that
// belongs to rows < below_rows).  16-byte loads, 8 in flight per thread.  Every thread of the
// workgroup calls it and gets the same result; red is LDS scratch of NC + 2 * (NB / NC) words.
struct ColumnPick {
    uint32_t B;      // NB when krem == 0 (nothing to select)
    uint32_t above;  // S[B + 1]
    uint32_t total;  // S[B]
    uint32_t below;  // the part of S[B] that comes from rows < below_rows
};
// `after_first_loads` is called once, right after the first batch of step-A loads has been issued and
// before anything waits for it: loads that the caller issues there (a first input tile) are behind
// the step-A loads in the wavefront's in-order load counter, so step A does not wait for them, and
// they have the whole of step A to arrive before step B's loads queue up behind them.
struct NoPrefetch {
    __device__ __forceinline__ void operator()() const {}
};
template <int NB, int NC, int UA = 8, typename Prefetch = NoPrefetch>
__device__ __forceinline__ ColumnPick column_pick(const uint32_t *rows, const uint32_t *coarse, int nrows,
                                                  int below_rows, uint32_t krem, uint32_t *red,
                                                  Prefetch after_first_loads = Prefetch()) {
    constexpr int FINE = NB / NC;
    static_assert(NC <= 64 && FINE <= 64 && NC % 4 == 0 && FINE % 4 == 0 && BLOCK % (NC / 4) == 0 &&
                      BLOCK % (FINE / 4) == 0 && NC + 2 * FINE <= BLOCK,
                  "column_pick geometry");
    uint32_t *redA = red, *redB = red + NC, *redBelow = red + NC + FINE;
    ColumnPick r{static_cast<uint32_t>(NB), 0u, 0u, 0u};
    __syncthreads();
    if (threadIdx.x < NC + 2 * FINE) red[threadIdx.x] = 0;
    __syncthreads();
    const int lane = threadIdx.x & 63;
    {
        constexpr int Q = NC / 4, G = BLOCK / Q;
        const int q = threadIdx.x % Q;
        const uint4 *co = reinterpret_cast<const uint4 *>(coarse) + q;
        uint4 sum = make_uint4(0, 0, 0, 0);
        // UA rows per thread and batch: the caller picks it so that its usual row count is one batch
        bool first = true;
        for (int r0 = threadIdx.x / Q; r0 < nrows || first; r0 += G * UA) {
            uint4 v[UA];
#pragma unroll
            for (int u = 0; u < UA; ++u) {
                const int rr = r0 + u * G;
                v[u] = (rr < nrows) ? co[static_cast<size_t>(rr) * Q] : make_uint4(0, 0, 0, 0);
            }
            if (first) {
                __builtin_amdgcn_sched_barrier(0);
                after_first_loads();
                __builtin_amdgcn_sched_barrier(0);
                first = false;
            }
#pragma unroll
            for (int u = 0; u < UA; ++u) {
                sum.x += v[u].x; sum.y += v[u].y; sum.z += v[u].z; sum.w += v[u].w;
            }
        }
        atomicAdd(&redA[4 * q + 0], sum.x);
        atomicAdd(&redA[4 * q + 1], sum.y);
        atomicAdd(&redA[4 * q + 2], sum.z);
        atomicAdd(&redA[4 * q + 3], sum.w);
    }
    __syncthreads();
    const uint64_t okA = __ballot(lane < NC && redA[lane % NC] >= krem);  // bit j: S[j * FINE] >= krem; a prefix of ones
    if (krem != 0 && okA != 0) {                                            // uniform over the workgroup
        const int J = 63 - __builtin_clzll(okA);
        {
            constexpr int Q = FINE / 4, G = BLOCK / Q;
            const int q = threadIdx.x % Q;
            const uint4 *col = reinterpret_cast<const uint4 *>(rows + J * FINE) + q;
            uint4 all = make_uint4(0, 0, 0, 0), below = make_uint4(0, 0, 0, 0);
            for (int r0 = threadIdx.x / Q; r0 < nrows; r0 += G * 8) {
                uint4 v[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int rr = r0 + u * G;
                    v[u] = (rr < nrows) ? col[static_cast<size_t>(rr) * (NB / 4)] : make_uint4(0, 0, 0, 0);
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    all.x += v[u].x; all.y += v[u].y; all.z += v[u].z; all.w += v[u].w;
                    if (r0 + u * G < below_rows) {
                        below.x += v[u].x; below.y += v[u].y; below.z += v[u].z; below.w += v[u].w;
                    }
                }
            }
            atomicAdd(&redB[4 * q + 0], all.x);
            atomicAdd(&redB[4 * q + 1], all.y);
            atomicAdd(&redB[4 * q + 2], all.z);
            atomicAdd(&redB[4 * q + 3], all.w);
            if (below_rows > 0) {
                atomicAdd(&redBelow[4 * q + 0], below.x);
                atomicAdd(&redBelow[4 * q + 1], below.y);
                atomicAdd(&redBelow[4 * q + 2], below.z);
                atomicAdd(&redBelow[4 * q + 3], below.w);
            }
        }
        __syncthreads();
        const uint64_t okB = __ballot(lane < FINE && redB[lane % FINE] >= krem);
        const int I = 63 - __builtin_clzll(okB | 1ull);  // bit 0 is set anyway: S[J * FINE] >= krem
        r.B = J * FINE + I;
        r.above = (I + 1 < FINE) ? redB[I + 1] : ((J + 1 < NC) ? redA[J + 1] : 0u);
        r.total = redB[I];
        r.below = redBelow[I];
    }
    __syncthreads();
    return r;
}

// ------------------------------------------------------------------ which scan pass counts
// Sums of two counters over the workgroup.  sm holds 2 * NW words.
__device__ __forceinline__ void block_sum2_u32(uint32_t &a, uint32_t &b, uint32_t *sm) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        a += __shfl_down(a, d);
        b += __shfl_down(b, d);
    }
    __syncthreads();
    if (lane == 0) {
        sm[w] = a;
        sm[NW + w] = b;
    }
    __syncthreads();
    uint32_t sa = 0, sb = 0;
#pragma unroll
    for (int i = 0; i < NW; ++i) {
        sa += sm[i];
        sb += sm[NW + i];
    }
    a = sa;
    b = sb;
}

// Did the speculative pass of this tensor bracket the k-th key?  Its window was a guess from a
// sample; the guess holds when at least k keys reached the window and fewer than k of them lie in
// its open-ended last bin.  Every workgroup of k_hist1, the kernel behind that pass, asks this for
// itself from the per-chunk counts that the pass stored (and that nothing overwrites), and leaves
// the answer in the tensor's state for the kernels that follow.  Every thread calls; the result is
// the same in all of them.
__device__ __forceinline__ bool spec_holds(const Launch &a, const SegDesc &sg, uint32_t *sm) {
    if (!(sg.flags & FLAG_SPEC)) return false;
    uint32_t reached = 0, open_ended = 0;
    for (int cc = threadIdx.x; cc < sg.nchunks; cc += BLOCK) {
        const uint2 p = a.cpairA[sg.chunk_begin + cc];
        reached += p.x;
        open_ended += p.y;
    }
    block_sum2_u32(reached, open_ended, sm);
    const uint32_t k = static_cast<uint32_t>(sg.k);
    return reached >= k && open_ended < k;
}

// Window bin of a key at or above the window's lowest key.
__device__ __forceinline__ uint32_t window_bin(uint32_t key, uint32_t lo, uint32_t shw) {
    const uint32_t b = (key - lo) >> shw;
    return b < NBW - 1 ? b : NBW - 1;
}

// ------------------------------------------------------------------ k_hist1
// LDS histogram of the top digit of one tile.
template <int VEC, bool FAST>
__device__ __forceinline__ void hist1_tile(const uint32_t (&dw)[Stream<VEC>::SLOTS],
                                           const uint32_t (&valid)[Stream<VEC>::SLOTS], uint32_t *h) {
    constexpr int EPD = Stream<VEC>::EPD;
    // Probe: does half of the wavefront share the top digit of lane 0's first element?  Then the tile
    // is counted with that digit's lanes taken together, slot by slot (one add per slot for them);
    // otherwise every lane adds for itself, which is the faster way when digits are spread.
    const uint32_t d0 = key_of<VEC>(elem_of<VEC>(dw[0], 0)) >> SH1;
    const uint32_t hot = __builtin_amdgcn_readfirstlane(d0);
    const bool skewed = FAST && __popcll(__ballot(d0 == hot)) >= 32;  // wave-uniform
    if (skewed) {
        uint32_t hot_count = 0;
#pragma unroll
        for (int e = 0; e < Stream<VEC>::SLOTS; ++e)
#pragma unroll
            for (int hh = 0; hh < EPD; ++hh) {
                const uint32_t d = key_of<VEC>(elem_of<VEC>(dw[e], hh)) >> SH1;
                hot_count += static_cast<uint32_t>(__popcll(__ballot(d == hot)));
                if (d != hot) atomicAdd(&h[d], 1u);
            }
        if ((threadIdx.x & 63) == 0) atomicAdd(&h[hot], hot_count);
        return;
    }
#pragma unroll
    for (int e = 0; e < Stream<VEC>::SLOTS; ++e)
#pragma unroll
        for (int hh = 0; hh < EPD; ++hh)
            if (FAST || ((valid[e] >> hh) & 1u))
                atomicAdd(&h[key_of<VEC>(elem_of<VEC>(dw[e], hh)) >> SH1], 1u);
}

// The full tiles of a chunk: `rem` tiles from element t0 on, which is advanced past them.
// Two register buffers used in turn: the next tile's loads are in flight while this one is
// counted.  The loop body loads unconditionally and moves no registers (the last one or two
// tiles are peeled): a load under a condition, or a copy of the new buffer into the old one,
// makes the compiler wait for the new tile before the old one is processed.
template <int VEC, bool WIDE>
__device__ __forceinline__ void hist1_full_tiles(const void *x, int64_t &t0, int64_t rem, uint32_t *h) {
    using St = Stream<VEC>;
    uint32_t cur[St::SLOTS], nxt[St::SLOTS], valid[St::SLOTS];
    auto load = [&](int64_t at, uint32_t(&dw)[St::SLOTS]) {
        if (WIDE)
            St::load_wide(x, at, dw);
        else
            St::load_fast(x, at, dw);
    };
    if (rem <= 0) return;
    load(t0, cur);
    while (rem > 2) {
        load(t0 + TILE, nxt);
        __builtin_amdgcn_sched_barrier(0);
        hist1_tile<VEC, true>(cur, valid, h);
        load(t0 + 2 * static_cast<int64_t>(TILE), cur);
        __builtin_amdgcn_sched_barrier(0);
        hist1_tile<VEC, true>(nxt, valid, h);
        t0 += 2 * static_cast<int64_t>(TILE);
        rem -= 2;
    }
    if (rem == 2) {
        load(t0 + TILE, nxt);
        __builtin_amdgcn_sched_barrier(0);
        hist1_tile<VEC, true>(cur, valid, h);
        hist1_tile<VEC, true>(nxt, valid, h);
        t0 += 2 * static_cast<int64_t>(TILE);
    } else {
        hist1_tile<VEC, true>(cur, valid, h);
        t0 += TILE;
    }
}

template <int VEC> __global__ __launch_bounds__(BLOCK) void k_hist1(Launch a) {
    using St = Stream<VEC>;
    __shared__ uint32_t h[NB1];
    __shared__ uint32_t sm[2 * NW];

    const int g = blockIdx.x;
    const int s = find_segment(a, g);
    const SegDesc &sg = a.seg[s];
    const int c = g - sg.chunk_begin;
    const int64_t beg = static_cast<int64_t>(c) * a.E;
    const int64_t end = (beg + a.E < sg.n) ? beg + a.E : sg.n;
    const bool held = spec_holds(a, sg, sm);
    if (c == 0 && threadIdx.x == 0) a.state[s].spec_held = held ? 1u : 0u;
    if (held) return;  // the speculative pass bracketed the k-th key: no exact pass is needed

    for (int b = threadIdx.x; b < NB1; b += BLOCK) h[b] = 0;
    __syncthreads();

    uint32_t cur[St::SLOTS], valid[St::SLOTS];
    int64_t t0 = beg;
    const int64_t full = (sg.flags & FLAG_ALIGNED4) ? (end - beg) / TILE : 0;
    // 16-byte loads when the tensor's base allows them (chunks start at multiples of the tile)
    if ((reinterpret_cast<uintptr_t>(sg.x) & 15) == 0)
        hist1_full_tiles<VEC, true>(sg.x, t0, full, h);
    else
        hist1_full_tiles<VEC, false>(sg.x, t0, full, h);
    for (; t0 < end; t0 += TILE) {
        St::load_slow(sg.x, t0, end, cur, valid);
        hist1_tile<VEC, false>(cur, valid, h);
    }
    __syncthreads();

    // The chunk's row of suffix sums, and every FINE1-th entry of it once more, contiguously: the
    // next kernel finds the bucket of the k-th key from the column sums of these rows alone.
    block_suffix_inplace<NB1>(h, sm);
    uint32_t *row = a.rows1 + static_cast<size_t>(g) * NB1;
    for (int b = threadIdx.x; b < NB1; b += BLOCK) row[b] = h[b];
    if (threadIdx.x < NC1) a.coarse1[static_cast<size_t>(g) * NC1 + threadIdx.x] = h[threadIdx.x * FINE1];
    if (c == 0)  // first chunk of the tensor: clear what k_refine accumulates into
        for (int b = threadIdx.x; b < NB3; b += BLOCK) a.G3[s * NB3 + b] = 0;
}

// ------------------------------------------------------------------ k_scan
// The pass that reads the whole input and keeps the candidates: every element whose key is at least
// the window's lowest key `lo` goes, in index order, into the candidate list of its chunk and is
// counted in its window bin; the squares of all other elements are summed in fp64.
//
// One tile.  Common path per element: clear the sign, compare with lo (the compare's lane mask is
// the keep bitmap of the slot), add the square of a dropped element in fp64.  Candidates are rare
// (about k/n and a margin).  After the waves have exchanged their counts, every kept
// (index, value) pair is written to its list position inside an LDS stage that holds STAGE_CAP
// consecutive list slots of the chunk; the stage goes out to memory with full-width stores only
// when it would overflow and at the end of the chunk, so the streaming loop itself issues loads
// only (loads and stores share one in-order counter: a store inside the loop would make every wait
// for the next tile's loads drain it).  List slots beyond the chunk's capacity are counted, not
// stored: such a chunk is read from the input again by the kernels that follow.  A tile that alone
// holds more than STAGE_CAP pairs (a quarter of its elements: a constant tensor, many ties, the kept
// end of sorted data) does not go through the stage; in the scan of a single tensor it gives the
// chunk's list up at once, so that nothing more is stored for a chunk that will be read again
// (storing such tiles until the list was full cost a constant tensor 50 MB of writes that nobody
// read); in the scan of a batch it stores directly while the list has room.
constexpr int STAGE_CAP = 2048;

// Writes list slots [from, to) of the chunk from the stage to memory and counts their window bins.
// stage[0] is list slot `from`.
template <int VEC>
__device__ __forceinline__ void flush_stage(const uint2 *stage, uint32_t from, uint32_t to, uint32_t cap, uint32_t lo,
                                            uint32_t shw, uint32_t *hw, int32_t *Li, typename Raw<VEC>::type *Lv) {
    for (uint32_t i = from + threadIdx.x; i < to; i += BLOCK) {
        const uint2 pr = stage[i - from];
        if (i < cap) {
            Li[i] = static_cast<int32_t>(pr.x);
            Lv[i] = static_cast<typename Raw<VEC>::type>(pr.y);
        }
        hist_add(hw, window_bin(key_of<VEC>(pr.y), lo, shw), true);
    }
}

template <int VEC, bool FAST, bool RUNS>
__device__ __forceinline__ void scan_tile(const uint32_t (&dw)[Stream<VEC>::SLOTS],
                                          const uint32_t (&valid)[Stream<VEC>::SLOTS], int64_t t0, uint32_t lo,
                                          uint32_t shw, uint32_t *hw, uint32_t *wcnt, uint2 *stage, uint32_t &running,
                                          uint32_t &flushed, uint32_t &cap, int32_t *Li,
                                          typename Raw<VEC>::type *Lv, double &acc) {  // cap: 0 once the list is given up
    using St = Stream<VEC>;
    using R = typename Raw<VEC>::type;
    constexpr int EPD = St::EPD, SLOTS = St::SLOTS;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    uint64_t m[SLOTS][EPD];
    bool keep[SLOTS][EPD];  // lives as the compare's lane mask, i.e. the same registers as m
    uint32_t wc = 0;
    if (VEC != TAG_F32 && FAST) {
        // Two 16-bit elements per dword, handled as a pair: one AND clears both signs, each half is
        // compared with the window's lowest pattern (lo is a multiple of 2^16 for these types).  The
        // squares of the dropped ones: fp16 values are added in fp32 over the tile's 16 elements of the
        // lane before the sum is widened (a square of an fp16 value is exact in fp32, 22 significant
        // bits and well inside its range, and 16 additions in fp32 leave the sum within 1e-6 of exact,
        // far inside the error norm's tolerance); bf16 values have fp32's exponent range, their squares
        // do not, so they are widened first as fp32 values are.
        const uint32_t thr16 = lo >> 16;
        float part = 0.0f;
#pragma unroll
        for (int e = 0; e < SLOTS; ++e) {
            const uint32_t k2 = dw[e] & 0x7FFF7FFFu;
            const uint32_t k_lo = k2 & 0xFFFFu, k_hi = k2 >> 16;
            keep[e][0] = k_lo >= thr16;
            keep[e][EPD - 1] = k_hi >= thr16;
            m[e][0] = __ballot(keep[e][0]);
            m[e][EPD - 1] = __ballot(keep[e][EPD - 1]);
            wc += __popcll(m[e][0]) + __popcll(m[e][EPD - 1]);
            float x_lo, x_hi;  // magnitudes: the signs are gone, the squares do not care
            if (VEC == TAG_F16) {
                x_lo = __half2float(__ushort_as_half(static_cast<unsigned short>(k_lo)));
                x_hi = __half2float(__ushort_as_half(static_cast<unsigned short>(k_hi)));
            } else {
                x_lo = __uint_as_float(k2 << 16);
                x_hi = __uint_as_float(k2 & 0xFFFF0000u);
            }
            x_lo = keep[e][0] ? 0.0f : x_lo;
            x_hi = keep[e][EPD - 1] ? 0.0f : x_hi;
            if (VEC == TAG_F16) {
                part = fmaf(x_lo, x_lo, part);
                part = fmaf(x_hi, x_hi, part);
            } else {
                asm("" : "+v"(x_lo));  // keeps the selects on the 32-bit values (see below)
                asm("" : "+v"(x_hi));
                const double d_lo = static_cast<double>(x_lo), d_hi = static_cast<double>(x_hi);
                acc = fma(d_lo, d_lo, acc);
                acc = fma(d_hi, d_hi, acc);
            }
        }
        acc += static_cast<double>(part);
    } else {
#pragma unroll
        for (int e = 0; e < SLOTS; ++e)
#pragma unroll
            for (int hh = 0; hh < EPD; ++hh) {
                const uint32_t raw = elem_of<VEC>(dw[e], hh);
                const bool ok = FAST || ((valid[e] >> hh) & 1u);
                keep[e][hh] = ok && key_of<VEC>(raw) >= lo;
                m[e][hh] = __ballot(keep[e][hh]);
                wc += __popcll(m[e][hh]);
                float xs = (ok && !keep[e][hh]) ? value_of<VEC>(raw) : 0.0f;
                // The empty statement pins the select to the 32-bit value: left alone, the compiler widens
                // first and then selects both halves of the double (one more instruction per element in a
                // loop whose time follows its instruction count: 24.0 -> 22.7 us on the 100 MB tensor).
                asm("" : "+v"(xs));
                const double xd = static_cast<double>(xs);
                acc = fma(xd, xd, acc);
            }
    }
    if (lane == 0) wcnt[w] = wc;
    __syncthreads();
    uint32_t before, tot;  // wave-uniform, in scalar registers: the branches below are scalar
    wave_counts(wcnt, before, tot);
    if (tot == 0) return;  // uniform over the workgroup
    if (running + tot - flushed > STAGE_CAP) {  // uniform: make room
        flush_stage<VEC>(stage, flushed, running, cap, lo, shw, hw, Li, Lv);
        __syncthreads();
        flushed = running;
    }
    const bool direct = tot > STAGE_CAP;  // uniform: this tile alone does not fit in the stage
    uint32_t slot_base = running + before;  // list slot of the wave's first kept element of this tile
    const uint32_t i_lane = static_cast<uint32_t>(St::first_elem(t0, 0));
    if (!direct) {
        uint2 *dst = stage - flushed;
#pragma unroll
        for (int e = 0; e < SLOTS; ++e) {
            uint64_t any = 0;
#pragma unroll
            for (int hh = 0; hh < EPD; ++hh) any |= m[e][hh];
            if (any == 0) continue;  // wave-uniform
            uint32_t pos = slot_base;
#pragma unroll
            for (int hh = 0; hh < EPD; ++hh) pos = lanes_below_plus(m[e][hh], pos);
            if constexpr (EPD == 2) {
                // (a lane's two halves are neighbours in the list: one address, the second eight bytes on if the first is kept)
                char *p = reinterpret_cast<char *>(dst + pos);
                const uint32_t i0 = i_lane + e * 64 * EPD;
                if (keep[e][0]) *reinterpret_cast<uint2 *>(p) = make_uint2(i0, elem_of<VEC>(dw[e], 0));
                p += keep[e][0] ? sizeof(uint2) : 0;
                if (keep[e][1]) *reinterpret_cast<uint2 *>(p) = make_uint2(i0 + 1, elem_of<VEC>(dw[e], 1));
                slot_base += __popcll(m[e][0]) + __popcll(m[e][1]);
            } else {
#pragma unroll
                for (int hh = 0; hh < EPD; ++hh) {
                    if (keep[e][hh]) dst[pos] = make_uint2(i_lane + e * 64 * EPD + hh, elem_of<VEC>(dw[e], hh));
                    pos += keep[e][hh] ? 1u : 0u;
                    slot_base += __popcll(m[e][hh]);
                }
            }
        }
    } else if (RUNS) {
        // A dense tile in the variant with one workgroup per compute unit, whose register budget has
        // room for it: the window bins by runs.  Nothing is stored, the list is given up.
        cap = 0;
        // A wavefront whose whole share of the tile is kept and sits in one bin (a constant tensor) adds once.
        const uint32_t bin0 = __builtin_amdgcn_readfirstlane(window_bin(key_of<VEC>(elem_of<VEC>(dw[0], 0)), lo, shw));
        uint32_t other = 0;
#pragma unroll
        for (int e = 0; e < SLOTS; ++e)
#pragma unroll
            for (int hh = 0; hh < EPD; ++hh) other |= window_bin(key_of<VEC>(elem_of<VEC>(dw[e], hh)), lo, shw) ^ bin0;
        if (wc == 64u * SLOTS * EPD && __ballot(other != 0) == 0) {  // wave-uniform
            if (lane == 0) atomicAdd(&hw[bin0], wc);
        } else {
            BinRun run;
#pragma unroll
            for (int e = 0; e < SLOTS; ++e)
#pragma unroll
                for (int hh = 0; hh < EPD; ++hh)
                    run.add(hw, window_bin(key_of<VEC>(elem_of<VEC>(dw[e], hh)), lo, shw), keep[e][hh]);
            run.flush(hw);
        }
    } else {
        // (the variant with two workgroups per compute unit has no register to spare for a list that
        // ends early: it stores while the list has room)
#pragma unroll
        for (int e = 0; e < SLOTS; ++e) {
            uint32_t pos = slot_base;
#pragma unroll
            for (int hh = 0; hh < EPD; ++hh) pos = lanes_below_plus(m[e][hh], pos);
#pragma unroll
            for (int hh = 0; hh < EPD; ++hh) {
                if (keep[e][hh]) {
                    const uint32_t raw = elem_of<VEC>(dw[e], hh);
                    if (pos < cap) {
                        Li[pos] = static_cast<int32_t>(i_lane + e * 64 * EPD + hh);
                        Lv[pos] = static_cast<R>(raw);
                    }
                    hist_add(hw, window_bin(key_of<VEC>(raw), lo, shw), true);
                    ++pos;
                }
                slot_base += __popcll(m[e][hh]);
            }
        }
    }
    running += tot;
    if (direct) flushed = running;  // nothing of this tile is staged
}

// The speculative pass's window, from a sample.  Every workgroup of the tensor reads the same
// SAMPLE_ELEMS elements (runs of 1 KB spread evenly over the tensor; after the first
// workgroup they come from the cache), counts their keys in a histogram of NSB bins and takes from
// it the keys at two ranks that the host derived from k: r_lo, a few standard deviations of the
// sampling noise below where the k-th key is expected in the sample (the window's lowest key: the
// lower edge of that rank's bin), and r_hi as far above it (the upper edge of its bin: the window's
// bins span up to there, as finely as NBW bins and a last digit of BITS3 bits allow).  A rank
// beyond the sample's size puts the lower end at key 0; rank 0 leaves the upper end open.  All
// integer work on the same data: every workgroup gets the same window.
//
// The histogram lives in LDS with one unused word after every 32 (a thread then walks its NSB / BLOCK
// consecutive bins without the 16-fold bank conflict of an unpadded stride).  The whole prologue is
// bound by instruction issue (two wavefronts per SIMD), so the work per sampled element is kept to a
// handful of instructions: one compare against a floor below which nothing needs counting, one add.
// The bins holding the two ranks are found while the suffix sums are formed in registers.
constexpr int NSB_PADDED = NSB + NSB / 32;
constexpr int SCAN_SMEM_WORDS = 2 * STAGE_CAP + NBW;  // k_scan's stage and window histogram; its prologue's scratch fits inside
constexpr uint32_t SAMPLE_SKEW = 32;   // runs: the sample's runs are shifted by up to this many run lengths
constexpr int SAMPLE_BATCH = 16;  // dword loads per thread and batch; the host picks 1, 2 or 4 batches (fp32: 8192 elements each)
__device__ __forceinline__ uint32_t padded(uint32_t bin) { return bin + (bin >> 5); }
template <int VEC, typename Prefetch>
__device__ __forceinline__ void sample_window(const SegDesc &sg, uint32_t *hs, uint32_t *sm, uint32_t *s_pick,
                                              Prefetch after_loads, uint32_t &lo, uint32_t &shw) {
    constexpr int EPD = VEC / 4;
    constexpr int MAXB = SAMPLE_ELEMS / BLOCK / EPD / SAMPLE_BATCH;  // batches at the full sample size
    constexpr int PER = NSB / BLOCK;                                 // bins per thread in the search
    static_assert(MAXB == 4 || MAXB == 2, "sample batches");
    const int lane = threadIdx.x & 63;
    const uint32_t w = static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x >> 6)));  // in a scalar register
    const int nbatch = static_cast<int>(sg.sample_batches);           // uniform; 1 .. MAXB
    // 16-byte loads: a run is 64 lanes x 16 bytes = 1 KB; nbatch * (SAMPLE_BATCH / 4) * NW runs, a power of two
    constexpr int QUADS = SAMPLE_BATCH / 4;
    const int run_shift = __builtin_ctz(QUADS * NW) + (nbatch >= 4 ? 2 : (nbatch >= 2 ? 1 : 0));
    const uint64_t nruns = (static_cast<uint64_t>(sg.n) / EPD) / 256;  // far more than are sampled: the host checks the size
    const dword4 *x = static_cast<const dword4 *>(sg.x) + lane;
    uint32_t v[MAXB][SAMPLE_BATCH];
#pragma unroll
    for (int b = 0; b < MAXB; ++b)
        if (b < nbatch) {
#pragma unroll
            for (int j = 0; j < QUADS; ++j) {
                // evenly spaced, plus a small run-dependent offset: an even spacing alone can put every
                // run on the same memory channel
                const uint32_t r = static_cast<uint32_t>(b * QUADS + j) * NW + w;
                const uint64_t run = ((static_cast<uint64_t>(r) * (nruns - SAMPLE_SKEW)) >> run_shift) + (r * 37u) % SAMPLE_SKEW;
                const dword4 q = x[run * 64];
                v[b][4 * j] = q.x;
                v[b][4 * j + 1] = q.y;
                v[b][4 * j + 2] = q.z;
                v[b][4 * j + 3] = q.w;
            }
        }
    __builtin_amdgcn_sched_barrier(0);
    after_loads();
    __builtin_amdgcn_sched_barrier(0);
    for (int b = threadIdx.x; b < NSB_PADDED; b += BLOCK) hs[b] = 0;
    if (threadIdx.x == 0) {
        s_pick[0] = NSB;  // what stays when no bin holds the rank
        s_pick[1] = NSB;
    }
    // Only the largest few per cent of the sample decide the two ranks.  Every thread's largest key
    // is at least `floor` = the smallest of the threads' largest keys, so at least BLOCK sampled keys
    // are >= floor: when the lower rank is within BLOCK, keys below floor need not be counted at all.
    // Bin 0 (zeros and the smallest denormals) is never counted: a rank that falls into it is not
    // found, which puts the window's lower end at key 0 just the same, and a tensor that is mostly
    // zeros does not pile its lanes onto one word.
    uint32_t mine = 0, least = 0xFFFFFFFFu;
#pragma unroll
    for (int b = 0; b < MAXB; ++b)
        if (b < nbatch) {
#pragma unroll
            for (int j = 0; j < SAMPLE_BATCH; ++j)
#pragma unroll
                for (int hh = 0; hh < EPD; ++hh) {
                    const uint32_t key = key_of<VEC>(elem_of<VEC>(v[b][j], hh));
                    mine = key > mine ? key : mine;
                    least = key < least ? key : least;
                }
        }
    uint32_t floor_key = mine;
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        const uint32_t o = __shfl_xor(floor_key, d);
        floor_key = o < floor_key ? o : floor_key;
    }
    if (lane == 0) sm[w] = floor_key;
    __syncthreads();
#pragma unroll
    for (int i = 0; i < NW; ++i) floor_key = sm[i] < floor_key ? sm[i] : floor_key;
    if (sg.r_lo > BLOCK) floor_key = 0;
    uint32_t floor_bin = floor_key >> SAMPLE_SH;
    floor_bin = floor_bin < 1 ? 1 : floor_bin;
    // A thread whose sampled keys all lie in one bin (a constant tensor) adds them with one add:
    // element by element the whole sample would go to one LDS word, one key after the other.
    const uint32_t top_bin = mine >> SAMPLE_SH;
    const bool one_bin = (least >> SAMPLE_SH) == top_bin;
    if (one_bin) {
        if (top_bin >= floor_bin) atomicAdd(&hs[padded(top_bin)], static_cast<uint32_t>(nbatch * SAMPLE_BATCH * EPD));
    } else {
#pragma unroll
        for (int b = 0; b < MAXB; ++b)
            if (b < nbatch) {
#pragma unroll
                for (int j = 0; j < SAMPLE_BATCH; ++j)
#pragma unroll
                    for (int hh = 0; hh < EPD; ++hh) {
                        const uint32_t bin = key_of<VEC>(elem_of<VEC>(v[b][j], hh)) >> SAMPLE_SH;
                        if (bin >= floor_bin) atomicAdd(&hs[padded(bin)], 1u);
                    }
            }
    }
    __syncthreads();
    // thread t owns bins [t * PER, (t + 1) * PER); higher bins hold larger keys
    uint32_t cnt[PER], own = 0;
#pragma unroll
    for (int j = 0; j < PER; ++j) {
        cnt[j] = hs[padded(threadIdx.x * PER + j)];
        own += cnt[j];
    }
    uint32_t total;
    const uint32_t inc = block_incl_scan(own, sm, &total);
    uint32_t above = total - inc;  // sampled (and counted) keys in the bins of the threads after this one
    const uint32_t r_lo = sg.r_lo, r_hi = sg.r_hi;
#pragma unroll
    for (int j = PER - 1; j >= 0; --j) {
        const uint32_t with = above + cnt[j];  // suffix sum at this bin
        if (above < r_lo && with >= r_lo) s_pick[0] = threadIdx.x * PER + j;
        if (r_hi != 0 && above < r_hi && with >= r_hi) s_pick[1] = threadIdx.x * PER + j;
        above = with;
    }
    __syncthreads();
    const uint32_t b_lo = s_pick[0], b_hi = s_pick[1];
    __syncthreads();
    lo = b_lo < NSB ? b_lo << SAMPLE_SH : 0u;
    const uint32_t hi = b_hi < NSB ? (b_hi + 1u) << SAMPLE_SH : 0x80000000u;  // first key above the bracket
    // fp32: bins as fine as the bracket and a last digit of BITS3 bits allow.  16-bit types: a bin is one
    // pattern (their keys have 16 zero bits below it), 2047 patterns upwards of lo, no last digit.
    const uint64_t width = hi > lo ? hi - lo : 1u;
    shw = VEC == TAG_F32 ? 0u : 16u;
    while (VEC == TAG_F32 && shw < static_cast<uint32_t>(BITS3) && (static_cast<uint64_t>(NBW - 1) << shw) < width) ++shw;
}

// DEPTH = register buffers of one tile each that the streaming loop rotates through, i.e. DEPTH - 1
// tiles of loads in flight while one is processed.  The loop waits for memory, not for instructions
// (one workgroup per compute unit with one tile ahead keeps 32 KB per compute unit in flight, which at
// the latency of a load under this traffic sustains about 4.8 TB/s), so a single tensor, whose launch has
// one workgroup per compute unit and twice the registers to spend, runs two tiles ahead.  A batch of
// tensors is launched with two workgroups per compute unit (four wavefronts per SIMD), which needs the
// kernel to stay within 128 vector registers: one tile ahead.
template <int VEC, bool SPEC, int DEPTH>
__global__ __launch_bounds__(BLOCK, DEPTH == 2 ? 4 : 2) void k_scan(Launch a) {
    static_assert(DEPTH == 2 || DEPTH == 3, "one or two tiles ahead");
    using R = typename Raw<VEC>::type;
    using St = Stream<VEC>;
    // 24 KB used in turn as: the sample histogram or the bucket search's scratch (prologue), then the
    // stage (STAGE_CAP pairs) followed by the window histogram
    __shared__ __attribute__((aligned(16))) uint32_t smem[SCAN_SMEM_WORDS];
    __shared__ uint32_t wcnt[2][NW];
    __shared__ uint32_t sm[2 * NW];
    __shared__ double smd[NW];
    __shared__ uint32_t s_pick[4];
    static_assert(NSB_PADDED <= SCAN_SMEM_WORDS && NC1 + 2 * FINE1 <= SCAN_SMEM_WORDS, "shared scratch fits");

    const int g = blockIdx.x;
    const int s = find_segment(a, g);
    const SegDesc &sg = a.seg[s];
    const int c = g - sg.chunk_begin;
    const int64_t beg = static_cast<int64_t>(c) * a.E;
    const int64_t end = (beg + a.E < sg.n) ? beg + a.E : sg.n;
    if (SPEC) {
        if (!(sg.flags & FLAG_SPEC)) return;  // this tensor goes straight to the exact passes
    } else {
        if (a.state[s].spec_held) return;     // the speculative pass did the work already
    }

    // The first tile does not depend on the prologue: its loads are put in flight inside it, behind
    // the prologue's first loads.
    uint32_t cur[St::SLOTS], nxt[St::SLOTS], far[St::SLOTS], valid[St::SLOTS];  // far: DEPTH 3 only
    const int64_t ntiles = (sg.flags & FLAG_ALIGNED4) ? (end - beg) / TILE : 0;
    auto first_tile = [&]() {
        if (ntiles > 0) St::load_fast(sg.x, beg, cur);
    };

    uint32_t lo, shw;
    if (SPEC) {
        sample_window<VEC>(sg, smem, sm, s_pick, first_tile, lo, shw);
        if (c == 0) {  // the accumulators of the kernels that follow
            for (int b = threadIdx.x; b < NB3; b += BLOCK) a.G3[s * NB3 + b] = 0;
            if (threadIdx.x == 0) {
                a.state[s].loA = lo;
                a.state[s].shwA = shw;
            }
        }
    } else {
        // The same in every workgroup of the tensor: bucket B1 of the k-th key from the rows of k_hist1
        // is the window, its 2^20 keys in the first 1024 bins.
        const ColumnPick p1 = column_pick<NB1, NC1, 16>(a.rows1 + static_cast<size_t>(sg.chunk_begin) * NB1,
                                                        a.coarse1 + static_cast<size_t>(sg.chunk_begin) * NC1, sg.nchunks,
                                                        0, static_cast<uint32_t>(sg.k), smem, first_tile);
        lo = p1.B << SH1;  // 2^31 when nothing is kept (k = 0): no key reaches it
        shw = VEC == TAG_F32 ? SH1 - BITS3 : 16;  // fp32: the bucket's 2^20 keys in 1024 bins; 16-bit: its 16 patterns in 16
        if (c == 0 && threadIdx.x == 0) {
            a.state[s].loB = lo;
            a.state[s].shwB = shw;
        }
    }
    uint32_t cap = a.cap;  // 0 once a dense tile has made the scan give the chunk's list up
    int32_t *Li = a.L_idx + static_cast<size_t>(g) * cap;
    R *Lv = static_cast<R *>(a.L_val) + static_cast<size_t>(g) * cap;

    uint2 *stage = reinterpret_cast<uint2 *>(smem);
    uint32_t *hw = smem + 2 * STAGE_CAP;
    __syncthreads();
    for (int b = threadIdx.x; b < NBW; b += BLOCK) hw[b] = 0;
    __syncthreads();

    double acc = 0.0;
    uint32_t running = 0, flushed = 0;
    int wb = 0;
    // Full tiles, the register buffers used in turn, unconditional loads in the loop, peeled tail (see
    // hist1_full_tiles).
    int64_t t0 = beg;
    int64_t rem = ntiles;
    auto tile = [&](const uint32_t(&dw)[St::SLOTS]) {
        scan_tile<VEC, true, DEPTH == 3>(dw, valid, t0, lo, shw, hw, wcnt[wb], stage, running, flushed, cap, Li, Lv, acc);
        t0 += TILE;
        wb ^= 1;
    };
    if (DEPTH == 3) {
        // cur holds the tile at t0; nxt the one behind it; far the one behind that
        if (rem >= 2) St::load_fast(sg.x, t0 + TILE, nxt);
        while (rem >= 5) {
            St::load_fast(sg.x, t0 + 2 * static_cast<int64_t>(TILE), far);
            __builtin_amdgcn_sched_barrier(0);
            tile(cur);
            St::load_fast(sg.x, t0 + 2 * static_cast<int64_t>(TILE), cur);
            __builtin_amdgcn_sched_barrier(0);
            tile(nxt);
            St::load_fast(sg.x, t0 + 2 * static_cast<int64_t>(TILE), nxt);
            __builtin_amdgcn_sched_barrier(0);
            tile(far);
            rem -= 3;
        }
        if (rem >= 1) {  // one to four tiles left: cur is loaded, nxt is if there are two
            if (rem >= 3) St::load_fast(sg.x, t0 + 2 * static_cast<int64_t>(TILE), far);
            __builtin_amdgcn_sched_barrier(0);
            tile(cur);
            if (rem >= 2) {
                if (rem >= 4) St::load_fast(sg.x, t0 + 2 * static_cast<int64_t>(TILE), cur);
                __builtin_amdgcn_sched_barrier(0);
                tile(nxt);
                if (rem >= 3) tile(far);
                if (rem >= 4) tile(cur);
            }
        }
    } else if (rem > 0) {
        while (rem > 2) {
            St::load_fast(sg.x, t0 + TILE, nxt);
            __builtin_amdgcn_sched_barrier(0);
            tile(cur);
            St::load_fast(sg.x, t0 + TILE, cur);
            __builtin_amdgcn_sched_barrier(0);
            tile(nxt);
            rem -= 2;
        }
        if (rem == 2) {
            St::load_fast(sg.x, t0 + TILE, nxt);
            __builtin_amdgcn_sched_barrier(0);
            tile(cur);
            tile(nxt);
        } else {
            tile(cur);
        }
    }
    for (; t0 < end; t0 += TILE, wb ^= 1) {
        St::load_slow(sg.x, t0, end, cur, valid);
        scan_tile<VEC, false, DEPTH == 3>(cur, valid, t0, lo, shw, hw, wcnt[wb], stage, running, flushed, cap, Li, Lv, acc);
    }
    __syncthreads();
    flush_stage<VEC>(stage, flushed, running, cap, lo, shw, hw, Li, Lv);

    const double bsum = block_sum_f64(acc, smd);
    if (threadIdx.x == 0) {
        a.chunk_err[g] = bsum;
        // more than the list holds = "read this chunk from the input", also for a list that was given up
        a.cnt[g] = (cap == 0 && running <= a.cap) ? a.cap + 1 : running;
    }
    __syncthreads();
    if (SPEC && threadIdx.x == 0) a.cpairA[g] = make_uint2(running, hw[NBW - 1]);
    // window-bin counts of this chunk's candidates, as a row of suffix sums (no global atomics)
    block_suffix_inplace<NBW>(hw, sm);
    uint32_t *row = a.rowsW + static_cast<size_t>(g) * NBW;
    for (int b = threadIdx.x; b < NBW; b += BLOCK) row[b] = hw[b];
    if (threadIdx.x < NCW) a.coarseW[static_cast<size_t>(g) * NCW + threadIdx.x] = hw[threadIdx.x * (NBW / NCW)];
}

// ------------------------------------------------------------------ list kernels
// Both work chunk by chunk on the candidates that the scan pass kept: from the chunk's list, or,
// when the chunk had more candidates than its list holds, from the chunk's part of the input
// itself (every element at or above the window's lowest key, in index order: the same sequence).
template <int VEC> struct ChunkSource {
    using R = typename Raw<VEC>::type;
    const int32_t *Li;   // the part's first list entry
    const R *Lv;
    const R *x;          // the part's first input element
    uint32_t base;       // its index in the tensor
    uint32_t len;        // entries of the part: list entries, or input elements
    uint32_t lo;
    bool from_input;
    // entry i of the part: its raw pattern, and whether it is a candidate at all
    // (Loads without a condition: an entry past the end reads the last one, or the first slot of an empty list,
    // and is masked out.  Guarded, the four loads of a tile, or the eight of k_emit's, sit in branches of their
    // own and were seen to wait for one another: a memory round trip per load instead of one for all.)
    __device__ __forceinline__ uint32_t raw(uint32_t i) const {
        const R *p = (from_input && len != 0) ? x : Lv;  // (an empty part of the input may start at the tensor's end)
        const uint32_t v = static_cast<uint32_t>(p[opaque(i < len ? i : (len ? len - 1 : 0))]);
        return v & keep_mask(i < len);
    }
    // the same for an entry known to exist (whole tiles of a long part): no stand-in, no mask
    __device__ __forceinline__ uint32_t raw_inside(uint32_t i) const { return static_cast<uint32_t>((from_input ? x : Lv)[i]); }
    __device__ __forceinline__ int32_t index_inside(uint32_t i) const { return from_input ? static_cast<int32_t>(base + i) : Li[i]; }
    __device__ __forceinline__ bool is_candidate(uint32_t i, uint32_t r) const {
        return i < len && (!from_input || key_of<VEC>(r) >= lo);
    }
    __device__ __forceinline__ int32_t index(uint32_t i) const {
        const uint32_t v = static_cast<uint32_t>(Li[opaque(from_input ? 0u : (i < len ? i : (len ? len - 1 : 0)))]);
        return static_cast<int32_t>((v & keep_mask(!from_input && i < len)) | ((base + i) & keep_mask(from_input)));
    }
};
// Entries of part `part` of `sub` of chunk g's candidates (list entries, or the chunk's elements when
// its list overflowed): the same cut as chunk_source below.  A short list leaves its later parts empty;
// the list kernels return at once for those and skip what they would have stored.
__device__ __forceinline__ uint32_t part_entries(const Launch &a, const SegDesc &sg, int g, uint32_t count, uint32_t part,
                                                 uint32_t sub) {  // count = a.cnt[g], loaded by the caller
    constexpr uint32_t LT = BLOCK * LU;
    const int c = g - sg.chunk_begin;
    const int64_t beg = static_cast<int64_t>(c) * a.E;
    const int64_t end = (beg + a.E < sg.n) ? beg + a.E : sg.n;
    const uint32_t entries = count > a.cap ? static_cast<uint32_t>(end - beg) : count;
    if (sub == 1) return entries;
    uint32_t per = (entries + sub - 1) / sub;
    per = (per + LT - 1) / LT * LT;
    const uint64_t first = static_cast<uint64_t>(per) * part;
    if (first >= entries) return 0u;
    return (first + per < entries) ? per : entries - static_cast<uint32_t>(first);
}

// Part `part` of `sub` of chunk g's candidates: the entries are cut into `sub` runs of whole list
// tiles; the later parts of a short list are empty.
template <int VEC>
__device__ __forceinline__ ChunkSource<VEC> chunk_source(const Launch &a, const SegDesc &sg, int g, uint32_t part,
                                                         uint32_t sub, uint32_t lo) {
    using R = typename Raw<VEC>::type;
    constexpr uint32_t LT = BLOCK * LU;
    ChunkSource<VEC> src;
    const int c = g - sg.chunk_begin;
    const int64_t beg = static_cast<int64_t>(c) * a.E;
    const int64_t end = (beg + a.E < sg.n) ? beg + a.E : sg.n;
    const uint32_t count = a.cnt[g];
    src.from_input = count > a.cap;
    const uint32_t entries = src.from_input ? static_cast<uint32_t>(end - beg) : count;
    uint32_t per = (entries + sub - 1) / sub;
    per = (per + LT - 1) / LT * LT;
    const uint64_t first = static_cast<uint64_t>(per) * part;
    const uint32_t off = first < entries ? static_cast<uint32_t>(first) : entries;
    src.len = (first + per < entries) ? per : entries - off;
    // (an empty part, or one that is read from the input, points at the start of the chunk's list: the loads
    // that ChunkSource issues without a condition then stay inside the chunk's own region)
    const uint32_t list_off = (src.from_input || src.len == 0) ? 0u : off;
    src.Li = a.L_idx + static_cast<size_t>(g) * a.cap + list_off;
    src.Lv = static_cast<const R *>(a.L_val) + static_cast<size_t>(g) * a.cap + list_off;
    src.x = static_cast<const R *>(sg.x) + beg + off;
    src.base = static_cast<uint32_t>(beg) + off;
    src.lo = lo;
    return src;
}

// A part that is read from the input is long (a quarter of the chunk's elements were candidates, or
// more), and a loop that loads LU entries per thread and then works on them moves 8 KB per
// workgroup and memory round trip: 1.8 TB/s over the whole chip when every chunk is dense (a
// constant tensor), and far less when only a few are (sorted data: the chunks at one end).  With one
// workgroup per compute unit nothing else hides the round trips.  The list kernels therefore come
// in two forms.  WIDE, for a launch with one workgroup per chunk and at most one per compute unit
// (a single tensor, lists of one part): a part from the input is read as tiles of U 16-byte loads
// per thread (thread t takes the t-th, (BLOCK + t)-th ... 16 bytes of the tile) with the next tiles'
// loads in flight; what is left after the last whole tile goes through the entry loop.  Needs the
// part to start on a 16-byte boundary (chunks are whole tiles, so this is the alignment of the
// tensor's base).  Plain, for every other launch: several workgroups per compute unit hide the
// round trips, and registers (occupancy) are worth more than wide tiles; entry loop only.
constexpr int WIDE_U = 4;
template <int VEC> struct Wide {
    static constexpr int EPV = 16 / static_cast<int>(sizeof(typename Raw<VEC>::type));  // elements per load
    static constexpr uint32_t ELEMS = BLOCK * WIDE_U * EPV;                              // elements per tile
    // whole tiles of the part, 0 when it is not read this way
    static __device__ __forceinline__ uint32_t tiles(const ChunkSource<VEC> &src) {
        const bool ok = src.from_input && (reinterpret_cast<uintptr_t>(src.x) & 15u) == 0;
        return ok ? src.len / ELEMS : 0u;
    }
    // element e (0 .. EPV) of a load, as the raw pattern of one element
    static __device__ __forceinline__ uint32_t elem(const dword4 &v, int e) {
        const int epd = EPV / 4;
        const uint32_t d = e / epd == 0 ? v.x : (e / epd == 1 ? v.y : (e / epd == 2 ? v.z : v.w));
        return elem_of<VEC>(d, e % epd);
    }
};
// That is k_refine's form, which only counts (WIDE_U loads per thread and tile, two tiles ahead).
// k_emit also places what it keeps, and 16-byte loads would leave a wavefront's store with four
// bytes every sixteen, in sixteen cache lines: its wide tiles (DENSE_SLOTS elements per thread) use
// the streaming layout of the scan instead: a wavefront owns a contiguous eighth of the tile and
// reads it 64 consecutive elements at a time, so consecutive lanes place consecutive elements, and
// only the wavefronts' totals are exchanged per tile; two tiles ahead, so that a tile's loads are
// issued before the stores of the tile two before it (one counter, in order: a wait for loads lets
// everything issued before them drain).  No alignment needed.
constexpr int DENSE_SLOTS = 16;
constexpr uint32_t DENSE_ELEMS = BLOCK * DENSE_SLOTS;

// f(tile, registers of the tile) for tiles [0, t_end) in order, with two tiles of loads in flight behind
// the one worked on: three register buffers of N loads used in turn, the loop body written out per buffer
// so that none is ever copied (a copy would wait for its loads); load(tile, buffer) fills one.  b0 holds
// tile 0 already.  Same shape as the streaming loop of the scan.  For a loop that also stores: the loads
// of a tile are issued before the stores of the tile two before it, so the wait for them does not have to
// let those stores drain first.
template <typename E, int N, typename L, typename F>
__device__ __forceinline__ void tiles_three(uint32_t t_end, E (&b0)[N], L &&load, F &&f) {
    E b1[N], b2[N];
    uint32_t t = 0, rem = t_end;
    if (rem == 0) return;
    if (rem >= 2) load(1, b1);
    while (rem >= 5) {
        load(t + 2, b2);
        __builtin_amdgcn_sched_barrier(0);
        f(t++, b0);
        load(t + 2, b0);
        __builtin_amdgcn_sched_barrier(0);
        f(t++, b1);
        load(t + 2, b1);
        __builtin_amdgcn_sched_barrier(0);
        f(t++, b2);
        rem -= 3;
    }
    if (rem >= 3) load(t + 2, b2);
    __builtin_amdgcn_sched_barrier(0);
    f(t++, b0);
    if (rem >= 2) {
        if (rem >= 4) load(t + 2, b0);
        __builtin_amdgcn_sched_barrier(0);
        f(t++, b1);
        if (rem >= 3) f(t++, b2);
        if (rem >= 4) f(t++, b0);
    }
}

// A pointer argument of a function that is not inlined is generic, and loads through it are flat
// loads: the hardware may serve them from LDS or from memory, out of order, so a wait for one tile
// is a wait for every load in flight, and the tiles ahead are not ahead at all (measured: the dense
// tiles of k_emit 2.4 us per call slower).  The two out-of-line passes below say where their memory
// is: they convert their pointer arguments to these types before they use them.
template <typename T> using GlobalPtr = T __attribute__((address_space(1))) *;
template <typename T> using LdsPtr = T __attribute__((address_space(3))) *;
template <typename T> __device__ __forceinline__ GlobalPtr<T> in_global(T *p) { return (GlobalPtr<T>)p; }
template <typename T> __device__ __forceinline__ LdsPtr<T> in_lds(T *p) { return (LdsPtr<T>)p; }

// k_refine's counts over the wide tiles of a part read from the input.  Out of line: inlined, its seven
// copies of the tile body sit in the middle of the kernel and the path of an ordinary part (a list of a
// few hundred entries, microseconds in all) pays for them in instruction fetch and register allocation.
struct DenseCounts {
    uint32_t def;  // candidates above bin Bw
    double acc;    // squares of the candidates below bin Bw
};
template <int VEC>
__device__ __attribute__((noinline)) DenseCounts refine_wide_tiles(const ChunkSource<VEC> src, uint32_t wide_tiles, uint32_t lo,
                                                                   uint32_t shw, uint32_t Bw, uint32_t *h3_arg) {
    using WR = Wide<VEC>;
    const GlobalPtr<const dword4> x = in_global(reinterpret_cast<const dword4 *>(src.x)) + threadIdx.x;
    const LdsPtr<uint32_t> h3 = in_lds(h3_arg);
    auto load = [&](uint32_t tile, dword4(&v)[WIDE_U]) {  // thread t: the t-th, (BLOCK + t)-th ... 16 bytes of the tile
#pragma unroll
        for (int u = 0; u < WIDE_U; ++u) v[u] = __builtin_nontemporal_load(x + static_cast<size_t>(tile) * (BLOCK * WIDE_U) + u * BLOCK);
    };
    const uint32_t shl = VEC == TAG_F32 ? 0u : 16u;
    const uint32_t in_bin = (1u << shw) - 1u;
    DenseCounts out = {0u, 0.0};
    dword4 cur[WIDE_U];
    load(0, cur);
    BinRun run;
    tiles_three(wide_tiles, cur, load, [&](uint32_t, const dword4(&v)[WIDE_U]) {
        // a wavefront whose whole share of the tile is one key (a constant tensor) counts it once
        const uint32_t raw0 = __builtin_amdgcn_readfirstlane(WR::elem(v[0], 0));
        uint32_t other = 0;
#pragma unroll
        for (int u = 0; u < WIDE_U; ++u)
#pragma unroll
            for (int e = 0; e < WR::EPV; ++e) other |= WR::elem(v[u], e) ^ raw0;
        if (__ballot(other != 0) == 0) {  // wave-uniform
            constexpr uint32_t PER_LANE = WIDE_U * WR::EPV;
            const uint32_t key = key_of<VEC>(raw0);
            const uint32_t bin = window_bin(key, lo, shw);
            if (key >= lo) {
                if (bin > Bw) out.def += PER_LANE;
                if (bin == Bw && (threadIdx.x & 63) == 0) BinRun::bin_add(h3, ((key - lo) & in_bin) >> shl, 64u * PER_LANE);
                if (bin < Bw) {
                    const double xd = static_cast<double>(value_of<VEC>(raw0));
                    out.acc = fma(static_cast<double>(PER_LANE) * xd, xd, out.acc);
                }
            }
            return;
        }
        // Sorted data: a wavefront whose smallest key lies in a bin above Bw only counts (the kept end),
        // one whose keys are all candidates in bins below Bw only sums squares (the dropped end).
        uint32_t least = 0xFFFFFFFFu, most = 0;
#pragma unroll
        for (int u = 0; u < WIDE_U; ++u)
#pragma unroll
            for (int e = 0; e < WR::EPV; ++e) {
                const uint32_t key = key_of<VEC>(WR::elem(v[u], e));
                least = key < least ? key : least;
                most = key > most ? key : most;
            }
        if (__ballot(!(least >= lo && window_bin(least, lo, shw) > Bw)) == 0) {  // wave-uniform
            out.def += WIDE_U * WR::EPV;
            return;
        }
        if (__ballot(!(least >= lo && window_bin(most, lo, shw) < Bw)) == 0) {  // wave-uniform
#pragma unroll
            for (int u = 0; u < WIDE_U; ++u)
#pragma unroll
                for (int e = 0; e < WR::EPV; ++e) {
                    const double xd = static_cast<double>(value_of<VEC>(WR::elem(v[u], e)));
                    out.acc = fma(xd, xd, out.acc);
                }
            return;
        }
        bool in_Bw = false;
#pragma unroll
        for (int u = 0; u < WIDE_U; ++u)
#pragma unroll
            for (int e = 0; e < WR::EPV; ++e) {
                const uint32_t raw = WR::elem(v[u], e);
                const uint32_t key = key_of<VEC>(raw);
                const bool cand = key >= lo;
                const uint32_t bin = window_bin(key, lo, shw);
                out.def += (cand && bin > Bw) ? 1u : 0u;
                in_Bw |= cand && bin == Bw;
                const double xd = (cand && bin < Bw) ? static_cast<double>(value_of<VEC>(raw)) : 0.0;
                out.acc = fma(xd, xd, out.acc);
            }
        // the last digit is counted only where the wavefront has a key in bin Bw at all (sorted data: one tile)
        if (__ballot(in_Bw) == 0) return;  // wave-uniform
#pragma unroll
        for (int u = 0; u < WIDE_U; ++u)
#pragma unroll
            for (int e = 0; e < WR::EPV; ++e) {
                const uint32_t key = key_of<VEC>(WR::elem(v[u], e));
                run.add(h3, ((key - lo) & in_bin) >> shl, key >= lo && window_bin(key, lo, shw) == Bw);
            }
    });
    run.flush(h3);
    return out;
}

// k_refine.  Prologue (every workgroup of the tensor, redundantly): the column sums of the chunks'
// window rows give the window bin Bw that holds the k-th key.  Then, over the chunk's candidates:
// the last digit (the position inside bin Bw) of those in Bw is counted, globally (G3) and as a row
// of suffix sums per chunk; candidates in higher bins are counted (kept whatever the last digit
// is), the squares of those in lower bins are summed (dropped whatever it is).
template <int VEC, bool WIDE> __global__ __launch_bounds__(BLOCK) void k_refine(Launch a) {
    __shared__ uint32_t h[NB3 > NCW + 2 * (NBW / NCW) ? NB3 : NCW + 2 * (NBW / NCW)];
    __shared__ uint32_t sm[2 * NW];
    __shared__ double smd[NW];

    const int g = blockIdx.x / a.sub;  // chunk
    const uint32_t part = blockIdx.x % a.sub;
    const int s = find_segment(a, g);
    const SegDesc &sg = a.seg[s];
    const int c = g - sg.chunk_begin;
    const SegStateWords stw = read_state(&a.state[s]);
    const bool spec = stw.spec_held != 0;
    const uint32_t lo = spec ? stw.loA : stw.loB;
    const uint32_t shw = spec ? stw.shwA : stw.shwB;
    const uint32_t shl = VEC == TAG_F32 ? 0u : 16u;
    const ChunkSource<VEC> src = chunk_source<VEC>(a, sg, g, part, a.sub, lo);
    if (src.len == 0 && !(c == 0 && part == 0)) return;  // an empty part (the tensor's first part still reports Bw)

    // The first LU entries of every thread do not depend on the prologue: their loads are in flight
    // while it runs (a typical chunk has no more than these), issued behind its first loads.
    uint32_t first[LU];
    auto first_entries = [&]() {
#pragma unroll
        for (int j = 0; j < LU; ++j) first[j] = src.raw(j * BLOCK + threadIdx.x);
    };
    const ColumnPick pw = column_pick<NBW, NCW>(a.rowsW + static_cast<size_t>(sg.chunk_begin) * NBW,
                                                a.coarseW + static_cast<size_t>(sg.chunk_begin) * NCW, sg.nchunks, 0,
                                                static_cast<uint32_t>(sg.k), h, first_entries);
    const uint32_t Bw = pw.B;  // NBW when nothing is kept
    if (c == 0 && part == 0 && threadIdx.x == 0) {
        a.state[s].Bw = Bw;
        a.state[s].c_gtw = pw.above;
    }

    uint32_t *h3 = h;
    for (int b = threadIdx.x; b < NB3; b += BLOCK) h3[b] = 0;
    __syncthreads();
    const uint32_t in_bin = (1u << shw) - 1u;
    uint32_t def = 0;  // candidates above bin Bw
    double acc = 0.0;  // squares of the candidates below bin Bw
    auto count_entry = [&](uint32_t i, uint32_t raw) {
        const bool cand = src.is_candidate(i, raw);
        const uint32_t key = key_of<VEC>(raw);
        const uint32_t bin = window_bin(key, lo, shw);
        def += (cand && bin > Bw) ? 1u : 0u;
        hist_add(h3, ((key - lo) & in_bin) >> shl, cand && bin == Bw);
        const double xd = (cand && bin < Bw) ? static_cast<double>(value_of<VEC>(raw)) : 0.0;
        acc = fma(xd, xd, acc);
    };
    uint32_t i_next = LU * BLOCK;  // where the entry loop goes on
    const uint32_t wide_tiles = WIDE ? Wide<VEC>::tiles(src) : 0u;  // uniform over the workgroup
    if (WIDE && __builtin_expect(wide_tiles != 0, 0)) {
        const DenseCounts dc = refine_wide_tiles<VEC>(src, wide_tiles, lo, shw, Bw, h3);
        def = dc.def;
        acc = dc.acc;
        i_next = wide_tiles * Wide<VEC>::ELEMS;
    } else {
#pragma unroll
        for (int j = 0; j < LU; ++j) count_entry(j * BLOCK + threadIdx.x, first[j]);
    }
    // longer parts (large k, many ties), the end of a part read from the input: LU entries per thread at a time
    for (uint32_t i0 = i_next; i0 < src.len; i0 += LU * BLOCK) {
        uint32_t more[LU];
        if (i0 + LU * BLOCK <= src.len) {  // uniform: a whole tile
#pragma unroll
            for (int j = 0; j < LU; ++j) more[j] = src.raw_inside(i0 + j * BLOCK + threadIdx.x);
        } else {
#pragma unroll
            for (int j = 0; j < LU; ++j) more[j] = src.raw(i0 + j * BLOCK + threadIdx.x);
        }
#pragma unroll
        for (int j = 0; j < LU; ++j) count_entry(i0 + j * BLOCK + threadIdx.x, more[j]);
    }
    const double bsum = block_sum_f64(acc, smd);
    if (threadIdx.x == 0) a.lerr[blockIdx.x] = bsum;
    __syncthreads();
    flush_bins<NB3>(h3, a.G3 + s * NB3);
    __syncthreads();
    block_suffix_inplace<NB3>(h3, sm);
    uint32_t *row = a.rows3 + static_cast<size_t>(blockIdx.x) * NB3;
    for (int b = threadIdx.x; b < NB3; b += BLOCK) row[b] = h3[b];
    uint32_t deftot;
    block_incl_scan(def, sm, &deftot);
    if (threadIdx.x == 0) a.ldef[blockIdx.x] = deftot;
}

// k_emit's placing over the whole dense tiles of a part read from the input; returns the counts of
// keys above T and equal to T after them.  Out of line for the same reason as refine_wide_tiles.
// Per slot the lane masks of "above T" and "equal to T" give a lane its two counts inside the
// wavefront's run (two 16-bit counts in one word); the wavefronts exchange their totals once per tile
// (totals: 2 * NW words of LDS, two buffers used in turn).
template <int VEC>
__device__ __attribute__((noinline)) uint2 emit_dense_tiles(const ChunkSource<VEC> src, uint32_t dense_tiles, uint32_t T, uint32_t q,
                                                            uint32_t kout, uint32_t run_gt, uint32_t run_eq, bool no_gt,
                                                            int32_t *oi_arg, int64_t *oi64_arg, typename Raw<VEC>::type *ov_arg, bool wide,
                                                            uint32_t *totals_arg) {
    using R = typename Raw<VEC>::type;
    const GlobalPtr<const R> x = in_global(src.x);
    const GlobalPtr<int32_t> oi = in_global(oi_arg);
    const GlobalPtr<int64_t> oi64 = in_global(oi64_arg);
    const GlobalPtr<R> ov = in_global(ov_arg);
    const LdsPtr<uint32_t> totals = in_lds(totals_arg);
    static_assert(DENSE_ELEMS < 65536, "two 16-bit counts travel in one word");
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    // element (slot j, this lane) of dense tile t of the part: wavefront w owns the w-th eighth of the tile
    auto dense_entry = [&](uint32_t t, int j) { return t * DENSE_ELEMS + (static_cast<uint32_t>(w) * DENSE_SLOTS + j) * 64 + lane; };
    auto dense_load = [&](uint32_t t, uint32_t(&r)[DENSE_SLOTS]) {
        const GlobalPtr<const R> p = x + dense_entry(t, 0);
#pragma unroll
        for (int j = 0; j < DENSE_SLOTS; ++j) r[j] = __builtin_nontemporal_load(p + j * 64);
    };
    uint32_t cur[DENSE_SLOTS];
    dense_load(0, cur);
    int buf = 0;
    tiles_three(dense_tiles, cur, dense_load, [&](uint32_t t, const uint32_t(&r)[DENSE_SLOTS]) {
        if (no_gt && run_eq >= q) return;  // uniform: nothing above T in the part and the quota of ties used up
        // The wavefront's totals first; a lane's own counts inside the wavefront's run only where a tile
        // is kept in part (further down): a tile kept whole or dropped whole does not need them.
        uint32_t wave_run = 0;  // wave-uniform
#pragma unroll
        for (int j = 0; j < DENSE_SLOTS; ++j) {
            const uint32_t key = key_of<VEC>(r[j]);
            wave_run += static_cast<uint32_t>(__popcll(__ballot(key > T))) + (static_cast<uint32_t>(__popcll(__ballot(key == T))) << 16);
        }
        const LdsPtr<uint32_t> tot = totals + buf * NW;
        if (lane == 0) tot[w] = wave_run;
        __syncthreads();
        uint32_t lower, tile_total;  // wave-uniform
        wave_counts((const uint32_t *)tot, lower, tile_total);
        buf ^= 1;
        const uint32_t tile_gt = tile_total & 0xFFFFu, tile_eq = tile_total >> 16;
        const uint32_t first_pos = run_gt + run_eq;  // of the tile's first kept element while the quota lasts
        if (tile_gt + tile_eq == DENSE_ELEMS && run_eq + tile_eq <= q && first_pos + DENSE_ELEMS <= kout) {
            // Every element of the tile is kept (uniform): the tile goes out as it came in, which is
            // what a constant tensor or the dense end of sorted data consists of.  The placing below
            // costs some sixty instructions per element, and with one workgroup on the compute unit
            // their issue is what the tile waits for.
            const uint32_t in_tile = dense_entry(0, 0);
            const int32_t index0 = static_cast<int32_t>(src.base + dense_entry(t, 0));
            if (wide) {
#pragma unroll
                for (int j = 0; j < DENSE_SLOTS; ++j) oi64[first_pos + in_tile + j * 64] = index0 + j * 64;
            } else {
#pragma unroll
                for (int j = 0; j < DENSE_SLOTS; ++j) oi[first_pos + in_tile + j * 64] = index0 + j * 64;
            }
#pragma unroll
            for (int j = 0; j < DENSE_SLOTS; ++j) ov[first_pos + in_tile + j * 64] = static_cast<R>(r[j]);
        } else if (tile_total != 0) {  // uniform over the workgroup
            uint32_t slots_before = lower;  // wave-uniform: (above T, equal to T) of the tile before slot j of this wavefront
#pragma unroll
            for (int j = 0; j < DENSE_SLOTS; ++j) {
                const uint32_t key = key_of<VEC>(r[j]);
                const uint64_t bg = __ballot(key > T), be = __ballot(key == T);
                const uint32_t mine = slots_before + lanes_below(bg) + (lanes_below(be) << 16);
                slots_before += static_cast<uint32_t>(__popcll(bg)) + (static_cast<uint32_t>(__popcll(be)) << 16);
                const uint32_t gt_before = run_gt + (mine & 0xFFFFu), eq_before = run_eq + (mine >> 16);
                if (key > T || (key == T && eq_before < q)) {
                    const uint32_t pos = gt_before + (eq_before < q ? eq_before : q);
                    if (pos < kout) {
                        const int32_t index = static_cast<int32_t>(src.base + dense_entry(t, j));
                        if (wide) oi64[pos] = index;
                        else oi[pos] = index;
                        ov[pos] = static_cast<R>(r[j]);
                    }
                }
            }
        }
        run_gt += tile_gt;
        run_eq += tile_eq;
    });
    return make_uint2(run_gt, run_eq);
}

// k_emit.  Prologue: G3 -> the last digit B3 of the k-th key, hence the threshold key T and the tie
// quota q; output offsets of the chunk from the rows of the earlier chunks.  Stable compaction of
// the chunk's candidates into idx_out / val_out (key > T, plus the first q keys equal to T).  The
// tensor's last chunk also adds up the error norm from the partial sums stored by the earlier
// kernels, in a fixed order.
template <int VEC, bool WIDE> __global__ __launch_bounds__(BLOCK) void k_emit(Launch a) {
    using R = typename Raw<VEC>::type;
    // fp32: the last digit's histogram; 16-bit types: the global suffix sums of the window bins up to Bw
    __shared__ uint32_t h[VEC == TAG_F32 ? NB3 : NBW + 1];
    __shared__ uint32_t wcnt[2][2][LU * NW];
    __shared__ uint32_t sm[2 * NW];
    __shared__ double smd[NW];
    __shared__ uint32_t s_pick[2];
    __shared__ uint32_t s_off[4];

    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const uint32_t sub = VEC == TAG_F32 ? a.sub : 1u;  // 16-bit types: one workgroup per chunk (their counts are per chunk)
    const int g = blockIdx.x / sub;  // chunk
    const uint32_t part = blockIdx.x % sub;
    const int s = find_segment(a, g);
    const SegDesc &sg = a.seg[s];
    const int c = g - sg.chunk_begin;
    const SegStateWords stw = read_state(&a.state[s]);
    // thread t: the candidate count of the tensor's chunk t, for the offsets and the error sum further down
    // (asked for here, with the state record: one memory round trip less in front of the rows' loads)
    const uint32_t count_t = static_cast<int>(threadIdx.x) < sg.nchunks ? a.cnt[sg.chunk_begin + threadIdx.x] : 0u;
    const bool spec = stw.spec_held != 0;
    const uint32_t lo = spec ? stw.loA : stw.loB;
    const uint32_t shw = spec ? stw.shwA : stw.shwB;
    const uint32_t kout = static_cast<uint32_t>(sg.k);
    const ChunkSource<VEC> src = chunk_source<VEC>(a, sg, g, part, sub, lo);
    // the tensor's last chunk is the short one, and the last part of a chunk the shortest
    const bool sums_error = c == sg.nchunks - 1 && part == sub - 1 && a.err_out != nullptr;
    // 16-bit types: thread t of that workgroup asks for chunk t's sum of squares below the window now, so that it
    // arrives behind the prologue instead of costing the error sum a memory round trip of its own at the end
    double below_t = 0.0;
    if (VEC != TAG_F32 && sums_error && static_cast<int>(threadIdx.x) < sg.nchunks) below_t = a.chunk_err[sg.chunk_begin + threadIdx.x];

    uint32_t raw[LU];
    int32_t id[LU];
    auto load_tile = [&](uint32_t t0) {
        if (t0 + LU * BLOCK <= src.len) {  // uniform: a whole tile
#pragma unroll
            for (int j = 0; j < LU; ++j) {
                const uint32_t i = t0 + j * BLOCK + threadIdx.x;
                raw[j] = src.raw_inside(i);
                id[j] = src.index_inside(i);
            }
        } else {
#pragma unroll
            for (int j = 0; j < LU; ++j) {
                const uint32_t i = t0 + j * BLOCK + threadIdx.x;
                raw[j] = src.raw(i);
                id[j] = src.index(i);
            }
        }
    };
    auto first_tile = [&]() { load_tile(0); };

    // Prologue -> threshold key T, tie quota q, and per chunk the number of keys above T and equal to
    // T among its candidates (gt_of / eq_of below).  The chunk's first tile is loaded behind the
    // prologue's first loads (the wavefront's load counter is in order).
    uint32_t T, q;
    bool any_kept;
    const uint32_t *cnt_rows;  // per-chunk rows of suffix sums in which T's counts are entries t_bin and t_bin + 1
    uint32_t row_len, t_bin, t_bins;
    const uint32_t *extra_gt;  // per-chunk count that is above T whatever the row says (fp32: the higher window bins)
    if (VEC == TAG_F32) {
        // last digit (k_refine's G3) -> T.  All candidates of one last-digit bin share one key.
        const uint32_t Bw = stw.Bw, c_gtw = stw.c_gtw;
        uint32_t my_bins[NB3 / BLOCK];  // raw counts of the last-digit bins this thread owns
#pragma unroll
        for (int j = 0; j < NB3 / BLOCK; ++j) my_bins[j] = a.G3[s * NB3 + threadIdx.x * (NB3 / BLOCK) + j];
        __builtin_amdgcn_sched_barrier(0);
        first_tile();
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int j = 0; j < NB3 / BLOCK; ++j) h[threadIdx.x * (NB3 / BLOCK) + j] = my_bins[j];
        __syncthreads();
        block_suffix_inplace<NB3>(h, sm);
        block_pick_bucket<NB3>(h, kout - c_gtw, s_pick);
        __syncthreads();
        const uint32_t B3 = s_pick[0], above3 = s_pick[1];
        __syncthreads();
        any_kept = Bw < NBW && B3 < NB3;
        const uint32_t bin_key = lo + (Bw << shw);  // lowest key of window bin Bw
        T = any_kept ? bin_key + B3 : 0xFFFFFFFFu;
        q = kout - (c_gtw + above3);
        cnt_rows = a.rows3;
        row_len = NB3;
        t_bin = B3;
        t_bins = NB3;
        extra_gt = a.ldef;

        // Error norm of the tensor, by one workgroup.  Everything it needs was stored by earlier kernels:
        // per-chunk sums of squares below the window (k_scan), per-chunk sums of squares of the candidates
        // below bin Bw (k_refine), and the counts of the candidates in bin Bw by last digit: the dropped
        // ones of a bin add count * value^2.  Fixed summation order.
        if (sums_error) {
            double sum = 0.0;
            static_assert(CTARGET <= BLOCK, "thread t has chunk t");
            if (static_cast<int>(threadIdx.x) < sg.nchunks) {
                const int cc = threadIdx.x;
                sum += a.chunk_err[sg.chunk_begin + cc];
                for (uint32_t pp = 0; pp < sub; ++pp)
                    if (part_entries(a, sg, sg.chunk_begin + cc, count_t, pp, sub) != 0)  // an empty part stored nothing
                        sum += a.lerr[static_cast<size_t>(sg.chunk_begin + cc) * sub + pp];
            }
#pragma unroll
            for (int j = 0; j < NB3 / BLOCK; ++j) {
                const uint32_t b = threadIdx.x * (NB3 / BLOCK) + j;
                uint32_t dropped = 0;
                if (b < B3 || B3 >= NB3) dropped = my_bins[j];
                else if (b == B3) dropped = my_bins[j] - q;
                if (dropped) {
                    const double v = static_cast<double>(value_of<VEC>(bin_key + b));
                    sum = fma(static_cast<double>(dropped) * v, v, sum);
                }
            }
            const double tot = block_sum_f64(sum, smd);
            if (threadIdx.x == 0) a.err_out[s] = static_cast<float>(sqrt(tot));
        }
    } else {
        // 16-bit types: a window bin is one pattern (the window's shift is the 16 zero bits below the
        // pattern), so the bin of the k-th key is the threshold itself and no last digit exists:
        // k_refine is not launched.  The column sums of the chunks' window rows give the bin.
        const ColumnPick pw = column_pick<NBW, NCW>(a.rowsW + static_cast<size_t>(sg.chunk_begin) * NBW,
                                                    a.coarseW + static_cast<size_t>(sg.chunk_begin) * NCW, sg.nchunks,
                                                    0, kout, h, first_tile);
        const uint32_t Bw = pw.B;
        any_kept = Bw < NBW;
        T = any_kept ? lo + (Bw << shw) : 0xFFFFFFFFu;
        q = kout - pw.above;
        cnt_rows = a.rowsW;
        row_len = NBW;
        t_bin = Bw;
        t_bins = NBW;
        extra_gt = nullptr;

        // Error norm: the squares below the window (k_scan) and, for every window bin below Bw and for
        // the dropped part of bin Bw, count * value^2.  The counts are differences of the global suffix
        // sums S[0 .. Bw + 1], which this one workgroup adds up from the chunks' rows: 64 columns at a
        // time, eight row groups side by side.
        if (sums_error) {
            // nothing kept means k = 0, for which the window starts above every key: no candidates at all
            const uint32_t ncols = any_kept ? Bw + 2 : 0u;  // S[Bw + 1] is the last one needed (0 past the last bin)
            // With the k-th key in the window's first 31 bins (the usual case for bf16, whose window starts
            // a few patterns below it) the sums S[0 .. Bw + 1] are among those column_pick has just left in h
            // (behind its NCW coarse sums: the fine sums of the first NBW / NCW bins): nothing to add up.
            const bool have_sums = any_kept && Bw + 1 < NBW / NCW;  // uniform
            const uint32_t *S = have_sums ? h + NCW : h;
            if (!have_sums) {
                for (uint32_t b = threadIdx.x; b < NBW + 1; b += BLOCK) h[b] = 0;
                __syncthreads();
            }
            const uint32_t col = threadIdx.x & 63, rg = threadIdx.x >> 6;
            for (uint32_t c0 = 0; !have_sums && c0 < ncols && c0 < NBW; c0 += 64) {
                const uint32_t b = c0 + col;
                if (b < ncols && b < NBW) {
                    const uint32_t *p = a.rowsW + static_cast<size_t>(sg.chunk_begin) * NBW + b;
                    uint32_t sum = 0;
                    for (int r0 = rg; r0 < sg.nchunks; r0 += NW * 8) {
                        uint32_t v[8];
#pragma unroll
                        for (int u = 0; u < 8; ++u) {  // (loads without a condition, see ChunkSource)
                            const int rr = r0 + u * NW;
                            const uint32_t t = p[static_cast<size_t>(opaque(static_cast<uint32_t>(rr < sg.nchunks ? rr : sg.nchunks - 1))) * NBW];
                            v[u] = t & keep_mask(rr < sg.nchunks);
                        }
#pragma unroll
                        for (int u = 0; u < 8; ++u) sum += v[u];
                    }
                    atomicAdd(&h[b], sum);
                }
            }
            __syncthreads();
            static_assert(CTARGET <= BLOCK, "thread t has chunk t");
            double sum = below_t;
            for (uint32_t b = threadIdx.x; any_kept && b <= Bw; b += BLOCK) {
                uint32_t dropped = S[b] - S[b + 1];
                if (b == Bw) dropped -= q;
                if (dropped) {  // the open-ended last bin is never below Bw: a dropped bin is one pattern
                    const double v = static_cast<double>(value_of<VEC>((lo + (b << shw)) >> 16));
                    sum = fma(static_cast<double>(dropped) * v, v, sum);
                }
            }
            const double tot = block_sum_f64(sum, smd);
            if (threadIdx.x == 0) a.err_out[s] = static_cast<float>(sqrt(tot));
            __syncthreads();
        }
    }

    // Output offsets of this part = sums over the earlier chunks, and over the earlier parts of this
    // chunk, of (#keys above T, #keys equal to T).  Thread t takes chunk t.
    {
        uint32_t gt = 0, eq = 0, gt_mine = 0, eq_mine = 0;  // totals of chunk t; what its parts before `part` hold
        uint32_t gt_own = 0, eq_own = 0;                    // what part `part` itself holds
        if (static_cast<int>(threadIdx.x) < sg.nchunks && any_kept) {
            for (uint32_t pp = 0; pp < sub; ++pp) {
                if (part_entries(a, sg, sg.chunk_begin + threadIdx.x, count_t, pp, sub) == 0) continue;  // nothing stored for it, nothing in it
                const size_t e = static_cast<size_t>(sg.chunk_begin + threadIdx.x) * sub + pp;
                const uint32_t *r = cnt_rows + e * row_len;
                const uint32_t above = (t_bin + 1 < t_bins) ? r[t_bin + 1] : 0u;
                const uint32_t g1 = (extra_gt != nullptr ? extra_gt[e] : 0u) + above, e1 = r[t_bin] - above;
                if (pp < part) {
                    gt_mine += g1;
                    eq_mine += e1;
                }
                if (pp == part) {
                    gt_own = g1;
                    eq_own = e1;
                }
                gt += g1;
                eq += e1;
            }
        }
        uint32_t tot;
        const uint32_t inc_gt = block_incl_scan(gt, sm, &tot);
        const uint32_t inc_eq = block_incl_scan(eq, sm, &tot);
        if (static_cast<int>(threadIdx.x) == c) {
            s_off[0] = inc_gt - gt + gt_mine;
            s_off[1] = inc_eq - eq + eq_mine;
            s_off[2] = gt_own;
            s_off[3] = eq_own;
        }
        __syncthreads();
    }
    // Nothing of this part is kept (no key above T in it, and its keys equal to T, if any, come after the
    // quota is used up): sorted or constant tensors leave most parts like this.
    if (src.len == 0 || (s_off[2] == 0 && (s_off[3] == 0 || s_off[1] >= q))) return;
    uint32_t run_gt = s_off[0], run_eq = s_off[1];

    const bool wide = a.idx64 != 0;
    const OutPtrs op = out_ptrs(a.idx_out, a.val_out, sg.out_off, kout, wide, a.wire != 0, sizeof(R));
    int32_t *oi = op.i32;
    int64_t *oi64 = op.i64;
    R *ov = static_cast<R *>(op.val);

    int buf = 0;
    // A part read from the input: its whole dense tiles first (out of line, see emit_dense_tiles).
    const uint32_t dense_tiles = (WIDE && src.from_input) ? src.len / DENSE_ELEMS : 0u;  // uniform over the workgroup
    if (WIDE && __builtin_expect(dense_tiles != 0, 0)) {
        const uint2 run = emit_dense_tiles<VEC>(src, dense_tiles, T, q, kout, run_gt, run_eq, s_off[2] == 0, oi, oi64, ov, wide,
                                                &wcnt[0][0][0]);
        run_gt = run.x;
        run_eq = run.y;
        __syncthreads();  // the count array changes hands
    }
    for (uint32_t t0 = dense_tiles * DENSE_ELEMS; t0 < src.len; t0 += BLOCK * LU, buf ^= 1) {
        if (t0 != 0) load_tile(t0);
        uint32_t pre_gt[LU], pre_eq[LU], cls[LU];  // cls: 0 not kept for sure, 1 equal to T, 2 above T
#pragma unroll
        for (int j = 0; j < LU; ++j) {
            const uint32_t i = t0 + j * BLOCK + threadIdx.x;
            const bool valid = i < src.len;
            const uint32_t key = key_of<VEC>(raw[j]);
            const bool gt = valid && key > T, eq = valid && key == T;
            cls[j] = gt ? 2u : (eq ? 1u : 0u);
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
            if (cls[j] == 2u || (cls[j] == 1u && eq_before < q)) {
                const uint32_t pos = gt_before + (eq_before < q ? eq_before : q);
                if (pos < kout) {
                    if (wide) oi64[pos] = id[j];
                    else oi[pos] = id[j];
                    ov[pos] = static_cast<R>(raw[j]);
                }
            }
        }
        run_gt += tg;
        run_eq += te;
    }
}

// ------------------------------------------------------------------ k = n
// A tensor of which everything is kept (the rule of Sec. 5.2 gives a fast link the ratio 1, "no
// compression") has nothing to select: its pairs are (i, x[i]) for every i and its error norm is 0.
// One launch for all such tensors of a batch: the segment table's chunks are tiles here, one
// workgroup per tile, 16 elements per thread, consecutive lanes on consecutive elements.
template <int VEC> __global__ __launch_bounds__(BLOCK) void k_keep_all(Launch a) {
    using R = typename Raw<VEC>::type;
    const int g = blockIdx.x;
    const int s = find_segment(a, g);
    const SegDesc &sg = a.seg[s];
    const int c = g - sg.chunk_begin;
    const uint32_t beg = static_cast<uint32_t>(c) * TILE;
    const uint32_t n = static_cast<uint32_t>(sg.n);
    const uint32_t end = beg + TILE < n ? beg + TILE : n;
    const bool wide = a.idx64 != 0;
    const OutPtrs op = out_ptrs(a.idx_out, a.val_out, sg.out_off, n, wide, a.wire != 0, sizeof(R));
    const R *x = static_cast<const R *>(sg.x);
    R *ov = static_cast<R *>(op.val);
    if (c == 0 && threadIdx.x == 0 && a.err_out != nullptr) a.err_out[s] = 0.0f;
    if (wide) {
        for (uint32_t i = beg + threadIdx.x; i < end; i += BLOCK) op.i64[i] = static_cast<int64_t>(i);
    } else {
        for (uint32_t i = beg + threadIdx.x; i < end; i += BLOCK) op.i32[i] = static_cast<int32_t>(i);
    }
    for (uint32_t i = beg + threadIdx.x; i < end; i += BLOCK) ov[i] = x[i];
}

// ------------------------------------------------------------------ small tensors: one launch
// Many small messages (a few thousand elements each) are bound by launch latency in the
// four-kernel path: about 5 us per kernel whatever the size.  Here one workgroup does the whole
// selection of one tensor that fits its registers: one read, three histogram rounds (the same
// 11/10/10-bit digits, LDS histograms, the same bucket search) that fix the threshold key T and
// the tie quota q, then one ordered round that writes the kept pairs in ascending index order and
// sums the squares of the dropped ones.  Same results as the big path.  One compute unit works
// through about 3 elements per ns in the ordered round, so tensors beyond one register tile stay
// with the four-kernel path, which spreads them over many compute units.
constexpr int SMALL_EPT = 128 / NW;            // elements per thread (16 with 512 threads)
constexpr int SMALL_N = BLOCK * SMALL_EPT;     // largest tensor this path takes
constexpr int SMALL_MAXSEG = 128;              // tensors per launch (the table travels as kernel arguments)
struct SmallDesc {
    const void *x;
    int64_t out_off;
    int32_t n, k;
};
struct SmallLaunch {
    SmallDesc seg[SMALL_MAXSEG];
    void *idx_out;
    void *val_out;
    float *err_out;
    uint32_t idx64;
    uint32_t wire;
};
static_assert(sizeof(SmallLaunch) <= 3584, "kernel arguments stay below 4 KB");
static_assert(SMALL_EPT * NW <= 128, "the (slot, wave) counts are scanned two per lane");
static_assert(SMALL_N < 65536, "two 16-bit counts travel in one word");

// One histogram round over the tensor in registers: counts digit (key >> shift) & (NB - 1) of the
// keys whose bits above the digit equal `prefix` (every key when use_prefix is false), then picks
// the bucket holding the krem-th largest.  Returns the bucket (NB when krem == 0) and the count
// above it.  Slot e of thread t is element e * BLOCK + t; slots past the end are skipped by a
// uniform branch.
template <int VEC, int NB>
__device__ __forceinline__ void small_round(const uint32_t (&raw)[SMALL_EPT], int n, int shift, int prefix_shift,
                                            uint32_t prefix, bool use_prefix, uint32_t krem, uint32_t *h, uint32_t *sm,
                                            uint32_t *s_pick, uint32_t &B, uint32_t &above) {
    for (int b = threadIdx.x; b < NB; b += BLOCK) h[b] = 0;
    __syncthreads();
    // probe on the first slot: do half of the wavefront's lanes count, and into one bin?  Then the
    // round adds through hist_add (equal keys would serialise on one LDS word), else every lane for itself
    bool skewed;
    {
        const uint32_t key = key_of<VEC>(raw[0]);
        const bool in = static_cast<int>(threadIdx.x) < n && (!use_prefix || (key >> prefix_shift) == prefix);
        const uint32_t bin = (key >> shift) & (NB - 1);
        const uint64_t act = __ballot(in);
        const uint32_t lbin = __builtin_amdgcn_readlane(bin, act ? __ffsll(static_cast<unsigned long long>(act)) - 1 : 0);
        skewed = __popcll(__ballot(in && bin == lbin)) >= 32;  // wave-uniform
    }
#pragma unroll
    for (int e = 0; e < SMALL_EPT; ++e) {
        if (e * BLOCK < n) {  // uniform
            const int i = e * BLOCK + static_cast<int>(threadIdx.x);
            const uint32_t key = key_of<VEC>(raw[e]);
            const bool in = i < n && (!use_prefix || (key >> prefix_shift) == prefix);
            const uint32_t bin = (key >> shift) & (NB - 1);
            if (skewed) hist_add(h, bin, in);
            else if (in) atomicAdd(&h[bin], 1u);
        }
    }
    __syncthreads();
    block_suffix_inplace<NB>(h, sm);
    block_pick_bucket<NB>(h, krem, s_pick);
    __syncthreads();
    B = s_pick[0];
    above = s_pick[1];
    __syncthreads();
}

template <int VEC> __global__ __launch_bounds__(BLOCK) void k_small(const SmallLaunch a) {
    using R = typename Raw<VEC>::type;
    __shared__ uint32_t h[NB1];
    __shared__ uint32_t sm[NW];
    __shared__ double smd[NW];
    __shared__ uint32_t s_pick[2];
    __shared__ uint32_t wcnt[SMALL_EPT * NW];  // (#above T) | (#equal to T) << 16 of every (slot, wave)

    const SmallDesc &sg = a.seg[blockIdx.x];
    const int n = sg.n;
    const uint32_t kout = static_cast<uint32_t>(sg.k);
    const R *x = static_cast<const R *>(sg.x);
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;

    // the whole tensor in one round of loads without conditions (see ChunkSource): an element past the end
    // reads the last one and is masked out
    uint32_t raw[SMALL_EPT];
#pragma unroll
    for (int e = 0; e < SMALL_EPT; ++e) raw[e] = 0;
    if (n > 0) {  // uniform
#pragma unroll
        for (int e = 0; e < SMALL_EPT; ++e) {
            const int i = e * BLOCK + static_cast<int>(threadIdx.x);
            raw[e] = static_cast<uint32_t>(x[opaque(static_cast<uint32_t>(i < n ? i : n - 1))]) & keep_mask(i < n);
        }
    }

    // threshold key T, number of keys above it, tie quota q
    uint32_t T = 0xFFFFFFFFu, c_gt = 0;
    if (kout != 0) {
        uint32_t B1, a1, B2, a2, B3, a3;
        small_round<VEC, NB1>(raw, n, SH1, 0, 0u, false, kout, h, sm, s_pick, B1, a1);
        small_round<VEC, NB2>(raw, n, SH2, SH1, B1, true, kout - a1, h, sm, s_pick, B2, a2);
        const uint32_t P = (B1 << BITS2) | B2;
        small_round<VEC, NB3>(raw, n, 0, SH2, P, true, kout - a1 - a2, h, sm, s_pick, B3, a3);
        T = (P << BITS3) | B3;
        c_gt = a1 + a2 + a3;
    }
    const uint32_t q = kout - c_gt;

    // Ordered round.  Index order is (slot, wave, lane): per slot the rank of every lane among the
    // wave's keys above / equal to T (two 16-bit fields of one register; the lane masks themselves
    // are not kept), the counts to LDS (lane e writes slot e's), one barrier, then every wavefront
    // scans the SMALL_EPT * NW counts in index order, two entries per lane.
    uint32_t rk[SMALL_EPT];
    uint32_t mine = 0;
#pragma unroll
    for (int e = 0; e < SMALL_EPT; ++e) {
        rk[e] = 0;
        uint32_t c = 0;
        if (e * BLOCK < n) {  // uniform
            const int i = e * BLOCK + static_cast<int>(threadIdx.x);
            const uint32_t key = key_of<VEC>(raw[e]);
            const uint64_t bg = __ballot(i < n && key > T);
            const uint64_t be = __ballot(i < n && key == T);
            rk[e] = lanes_below(bg) | (lanes_below(be) << 16);
            c = static_cast<uint32_t>(__popcll(bg)) | (static_cast<uint32_t>(__popcll(be)) << 16);
        }
        mine = (lane == e) ? c : mine;
    }
    if (lane < SMALL_EPT) wcnt[lane * NW + w] = mine;
    __syncthreads();
    const uint32_t c0 = (2 * lane < SMALL_EPT * NW) ? wcnt[2 * lane] : 0u;
    const uint32_t c1 = (2 * lane + 1 < SMALL_EPT * NW) ? wcnt[2 * lane + 1] : 0u;
    const uint32_t inc = wave_incl_scan(c0 + c1);
    const uint32_t ex0 = inc - c0 - c1, ex1 = inc - c1;  // counts before entry 2 * lane and before 2 * lane + 1

    const bool wide = a.idx64 != 0;
    const OutPtrs op = out_ptrs(a.idx_out, a.val_out, sg.out_off, kout, wide, a.wire != 0, sizeof(R));
    int32_t *oi = op.i32;
    int64_t *oi64 = op.i64;
    R *ov = static_cast<R *>(op.val);
    double acc = 0.0;
#pragma unroll
    for (int e = 0; e < SMALL_EPT; ++e) {
        if (e * BLOCK < n) {  // uniform
            const int i = e * BLOCK + static_cast<int>(threadIdx.x);
            const int entry = e * NW + w;
            const uint32_t before = __shfl((entry & 1) ? ex1 : ex0, entry >> 1);  // one entry for the whole wave
            const uint32_t key = key_of<VEC>(raw[e]);
            const bool valid = i < n;
            const uint32_t gt_before = (before & 0xFFFFu) + (rk[e] & 0xFFFFu);
            const uint32_t eq_before = (before >> 16) + (rk[e] >> 16);
            const bool keep = valid && (key > T || (key == T && eq_before < q));
            if (keep) {
                const uint32_t pos = gt_before + (eq_before < q ? eq_before : q);
                if (pos < kout) {
                    if (wide) oi64[pos] = i;
                    else oi[pos] = i;
                    ov[pos] = static_cast<R>(raw[e]);
                }
            }
            const double v = static_cast<double>((valid && !keep) ? value_of<VEC>(raw[e]) : 0.0f);
            acc = fma(v, v, acc);
        }
    }
    if (a.err_out != nullptr) {
        const double tot = block_sum_f64(acc, smd);
        if (threadIdx.x == 0) a.err_out[blockIdx.x] = static_cast<float>(sqrt(tot));
    }
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

template <typename R, typename I>
__global__ __launch_bounds__(BLOCK) void k_scatter(const I *idx, const R *val, int64_t k, R *y, int64_t n) {
    const int64_t j = static_cast<int64_t>(blockIdx.x) * BLOCK + threadIdx.x;
    if (j >= k) return;
    const int64_t i = idx[j];
    if (i >= 0 && i < n) y[i] = val[j];
}

// Round an fp32 value to the 16-bit type of the tag, to nearest, ties to even.
template <int VEC> __device__ __forceinline__ uint32_t narrow_rne(float f) {
    if (VEC == TAG_F16) return __half_as_ushort(__float2half_rn(f));
    const uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (u >> 16) | 0x40u;  // NaN stays NaN
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;  // bf16: add half an ulp of the kept part, less one when it is even
}

// Accumulating decompress: y[idx[j]] += val[j], one entry per thread.  16-bit types: both operands
// widened to fp32, added, rounded to nearest even; fp32 is wide enough (24 >= 2 * 11 + 2 bits) for
// this to be the correctly rounded sum of the two 16-bit values.  Entries of one call must have
// distinct indices: the read-modify-write is not atomic.
template <int VEC, typename I>
__global__ __launch_bounds__(BLOCK) void k_scatter_add(const I *idx, const typename Raw<VEC>::type *val, int64_t k,
                                                       typename Raw<VEC>::type *y, int64_t n) {
    using R = typename Raw<VEC>::type;
    const int64_t j = static_cast<int64_t>(blockIdx.x) * BLOCK + threadIdx.x;
    if (j >= k) return;
    const int64_t i = idx[j];
    if (i < 0 || i >= n) return;
    const float sum = value_of<VEC>(y[i]) + value_of<VEC>(val[j]);
    y[i] = VEC == TAG_F32 ? static_cast<R>(__float_as_uint(sum)) : static_cast<R>(narrow_rne<VEC>(sum));
}

// 16-byte store of the dense output.  `stream` = the output of the call is large against the
// last-level cache (256 MB): a nontemporal store then keeps the output from flushing the cache, and
// the write kernel and the reads of the next call both run faster (805 MB in 24 tensors: decompress
// 210 -> 179 us, the next call's first read pass 217 -> 178 us; single tensors of 150 to 400 MB: the
// compress + decompress step 4 to 6 % faster).  An output of 100 MB is better left to the cache
// (decompress 16 us with plain stores, 25 us with nontemporal ones).
__device__ __forceinline__ void store16(uint4 *dst, uint4 v, bool stream) {
    if (stream) __builtin_nontemporal_store(dword4{v.x, v.y, v.z, v.w}, reinterpret_cast<dword4 *>(dst));
    else *dst = v;
}
constexpr size_t STREAM_STORE_BYTES = static_cast<size_t>(128) << 20;

// Lower bound by one wavefront: the first j in [0, k) with idx[j] >= value (k if none), for
// ascending idx.  The 64 lanes probe evenly spaced entries; the number of probes below `value`
// narrows [lo, hi] 64-fold per round (4 rounds for k = 250 000).  Wave-synchronous: no barrier,
// so the other wavefronts of the workgroup can do something else meanwhile.  With idx not
// ascending the result is some position in [0, k]: memory-safe, meaningless.
template <typename I>
__device__ __forceinline__ uint32_t wave_lower_bound(const I *idx, uint32_t k, int64_t value) {
    const uint32_t lane = threadIdx.x & 63;
    uint32_t lo = 0, hi = k;  // invariant: idx[j] < value for j < lo, idx[hi] >= value or hi == k
    while (lo < hi) {         // lo, hi are wave-uniform; the width shrinks to below width / 64 every round
        const uint32_t width = hi - lo;
        const uint32_t step = (width + 63) / 64;
        const uint64_t p = static_cast<uint64_t>(lo) + static_cast<uint64_t>(lane) * step;
        const bool below = p < hi && static_cast<int64_t>(idx[p]) < value;
        const uint32_t c = static_cast<uint32_t>(__popcll(__ballot(below)));  // probes 0 .. c-1 are below value
        const uint32_t nprobe = (width + step - 1) / step;
        const uint32_t old_lo = lo;
        lo = c ? old_lo + (c - 1) * step + 1 : old_lo;
        hi = c ? (c < nprobe ? old_lo + c * step : hi) : old_lo;
    }
    return lo;
}

// Decompress for ascending indices in one kernel.  The output is cut into byte spans: workgroup b
// owns bytes [B_b, B_b+1) with B_0 = 0, B_b = head + b * span (16-byte aligned addresses) and
// B_last = total.  Two of its wavefronts first search idx for the entries of the span while the
// others already zero-fill it with 16-byte stores; after a barrier the entries are written.
// Every output byte is written by one workgroup only; an entry whose index lies outside the span
// that the search assigned it to (possible only when idx is not ascending) is skipped.
template <typename R, typename I>
__device__ __forceinline__ void merge_span(const I *idx, const R *val, uint32_t k, unsigned char *y, size_t total,
                                           size_t head, size_t span, uint32_t blk, uint32_t nblk, bool stream,
                                           uint32_t *s_range) {
    const size_t byte_a = blk == 0 ? 0 : head + static_cast<size_t>(blk) * span;
    const size_t byte_b = blk + 1 == nblk ? total : head + static_cast<size_t>(blk + 1) * span;
    const int64_t ea = static_cast<int64_t>(byte_a / sizeof(R)), eb = static_cast<int64_t>(byte_b / sizeof(R));
    const int w = threadIdx.x >> 6;
    if (w < 2) {
        const uint32_t pos = wave_lower_bound(idx, k, w == 0 ? ea : eb);
        if ((threadIdx.x & 63) == 0) s_range[w] = pos;
    }
    const size_t va = blk == 0 ? (head < byte_b ? head : byte_b) : byte_a;  // aligned start
    const size_t nvec = (byte_b - va) / 16;
    uint4 *body = reinterpret_cast<uint4 *>(y + va);
    const uint4 z = make_uint4(0, 0, 0, 0);
    for (size_t i = threadIdx.x; i < nvec; i += BLOCK) store16(&body[i], z, stream);
    for (size_t i = byte_a + threadIdx.x; i < va; i += BLOCK) y[i] = 0;
    for (size_t i = va + nvec * 16 + threadIdx.x; i < byte_b; i += BLOCK) y[i] = 0;
    __syncthreads();  // also orders this workgroup's zero stores before its value stores
    R *out = reinterpret_cast<R *>(y);
    const uint32_t ja = s_range[0], jb = s_range[1];
    if (jb - ja > 4 * BLOCK) {  // uniform over the workgroup
        // A span that holds many entries although the tensor holds few (indices bunched together: a constant
        // tensor keeps its first k elements, sorted data one end): twelve entries per thread at a time, with
        // loads that do not depend on a condition (an entry past the end is read as the last one and not
        // used), so that all of them are in flight together; guarded loads are issued one after the other,
        // each waiting for the one before, and such a span took twice the whole kernel's usual time.
        constexpr int AT_ONCE = 12;
        const uint32_t last = jb - 1;
        for (uint32_t j0 = ja + threadIdx.x; j0 < jb; j0 += AT_ONCE * BLOCK) {
            int64_t i[AT_ONCE];
            R v[AT_ONCE];
#pragma unroll
            for (int u = 0; u < AT_ONCE; ++u) {
                const uint32_t j = j0 + u * BLOCK;
                const uint32_t jc = j < last ? j : last;
                i[u] = static_cast<int64_t>(idx[jc]);
                v[u] = val[jc];
            }
#pragma unroll
            for (int u = 0; u < AT_ONCE; ++u)
                if (j0 + u * BLOCK < jb && i[u] >= ea && i[u] < eb) out[i[u]] = v[u];
        }
        return;
    }
    // the usual span: at most four entries per thread (one, mostly)
    for (uint32_t j0 = ja + threadIdx.x; j0 < jb; j0 += 4 * BLOCK) {
        int64_t i[4];
        R v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint32_t j = j0 + u * BLOCK;
            i[u] = j < jb ? static_cast<int64_t>(idx[j]) : -1;  // -1 lies in no span
            v[u] = j < jb ? val[j] : R(0);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (i[u] >= ea && i[u] < eb) out[i[u]] = v[u];
    }
}
// The same for many entries per line (k / n of a few per cent and more), where k_merge's value
// stores would rewrite most output lines a second time: same spans, same search, but the span is
// built piece by piece in LDS (zeros, then the entries that fall into the piece) and every
// piece is written out once with 16-byte stores, so no output line is written twice.  Entries are
// ascending, so every thread walks its own (strided) subsequence of them forwards.  An entry
// whose index lies outside the piece that the walk assigned it to (possible only when idx is not
// ascending) is skipped: every store stays inside the span.
constexpr int MERGE_PIECE = 32768;  // bytes of LDS per piece
template <typename R, typename I>
__device__ __forceinline__ void merge_span_lds(const I *idx, const R *val, uint32_t k, unsigned char *y, size_t total,
                                               size_t head, size_t span, uint32_t blk, uint32_t nblk, bool stream,
                                               unsigned char *piece, uint32_t *s_range) {
    const size_t byte_a = blk == 0 ? 0 : head + static_cast<size_t>(blk) * span;
    const size_t byte_b = blk + 1 == nblk ? total : head + static_cast<size_t>(blk + 1) * span;
    const int w = threadIdx.x >> 6;
    if (w < 2) {
        const int64_t bound = static_cast<int64_t>((w == 0 ? byte_a : byte_b) / sizeof(R));
        const uint32_t pos = wave_lower_bound(idx, k, bound);
        if ((threadIdx.x & 63) == 0) s_range[w] = pos;
    }
    // unaligned head of the whole tensor (workgroup 0 only, < 16 bytes): entries there are written
    // after the zeros by the same thread order below, so handle it as part of the first piece
    const size_t va = blk == 0 ? (head < byte_b ? head : byte_b) : byte_a;  // 16-byte aligned start
    __syncthreads();
    uint32_t j = s_range[0] + threadIdx.x;  // this thread's next entry
    const uint32_t jb = s_range[1];
    R *out = reinterpret_cast<R *>(y);
    if (va > byte_a) {  // workgroup 0: the few bytes before the first aligned address, straight to memory
        for (size_t i = byte_a + threadIdx.x; i < va; i += BLOCK) y[i] = 0;
        __syncthreads();
        const int64_t e1 = static_cast<int64_t>(va / sizeof(R));
        for (uint32_t jj = s_range[0] + threadIdx.x; jj < jb; jj += BLOCK) {
            const int64_t i = idx[jj];
            if (i >= e1) break;
            if (i >= 0) out[i] = val[jj];
        }
    }
    for (size_t p0 = va; p0 < byte_b; p0 += MERGE_PIECE) {
        const size_t p1 = (p0 + MERGE_PIECE < byte_b) ? p0 + MERGE_PIECE : byte_b;
        const int64_t e0 = static_cast<int64_t>(p0 / sizeof(R)), e1 = static_cast<int64_t>(p1 / sizeof(R));
        uint4 *pz = reinterpret_cast<uint4 *>(piece);
        for (int i = threadIdx.x; i < MERGE_PIECE / 16; i += BLOCK) pz[i] = make_uint4(0, 0, 0, 0);
        __syncthreads();
        R *pl = reinterpret_cast<R *>(piece);
        while (j < jb) {
            const int64_t i = idx[j];
            if (i >= e1) break;
            if (i >= e0) pl[i - e0] = val[j];
            j += BLOCK;
        }
        __syncthreads();
        const size_t nvec = (p1 - p0) / 16;
        uint4 *dst = reinterpret_cast<uint4 *>(y + p0);
        for (size_t i = threadIdx.x; i < nvec; i += BLOCK) store16(&dst[i], pz[i], stream);
        for (size_t i = p0 + nvec * 16 + threadIdx.x; i < p1; i += BLOCK) y[i] = piece[i - p0];  // ragged end of the tensor
        __syncthreads();
    }
}

template <typename R, typename I>
__global__ __launch_bounds__(BLOCK) void k_merge(const I *idx, const R *val, uint32_t k, unsigned char *y,
                                                 size_t total, size_t head, size_t span, uint32_t stream) {
    __shared__ uint32_t s_range[2];
    merge_span<R, I>(idx, val, k, y, total, head, span, blockIdx.x, gridDim.x, stream != 0, s_range);
}

template <typename R, typename I>
__global__ __launch_bounds__(BLOCK) void k_merge_lds(const I *idx, const R *val, uint32_t k, unsigned char *y,
                                                     size_t total, size_t head, size_t span, uint32_t stream) {
    __shared__ __attribute__((aligned(16))) unsigned char piece[MERGE_PIECE];
    __shared__ uint32_t s_range[2];
    merge_span_lds<R, I>(idx, val, k, y, total, head, span, blockIdx.x, gridDim.x, stream != 0, piece, s_range);
}

// Decompress of several tensors in one launch: the spans of all tensors form one grid, a table in
// the kernel arguments says which workgroups belong to which tensor, and every workgroup runs the
// one-tensor code above on its span (the sparse or the LDS-built variant, per tensor).
constexpr int MERGE_MAXSEG = 96;
struct MergeSeg {   // 40 bytes
    unsigned char *y;
    int64_t pair_off;      // first pair of this tensor in idx / val
    int64_t n;             // elements
    uint32_t k;
    uint32_t first_block;  // its spans are workgroups [first_block, first_block of the next tensor)
    uint32_t dense;        // k > n / MERGE_DENSE_RATIO: build the lines in LDS
    uint32_t pad;
};
struct MergeLaunch {
    MergeSeg seg[MERGE_MAXSEG];
    const int32_t *idx;
    const void *val;
    size_t span;           // bytes of output per workgroup, the same for every tensor of the call
    uint32_t blocks;       // workgroups of the launch
    int32_t S;
    uint32_t stream;       // the call's output is larger than the last-level cache: nontemporal stores
};
static_assert(sizeof(MergeLaunch) <= 4096, "kernel arguments stay within 4 KB");
static_assert(MERGE_MAXSEG <= 128, "two table entries per lane");

template <typename R> __global__ __launch_bounds__(BLOCK) void k_merge_seg(const MergeLaunch a) {
    __shared__ __attribute__((aligned(16))) unsigned char piece[MERGE_PIECE];
    __shared__ uint32_t s_range[2];
    // owner of this workgroup: the last tensor whose first workgroup is <= blockIdx.x (first workgroups
    // never decrease and the first is 0); lane l looks at table entries l and l + 64
    const int lane = threadIdx.x & 63;
    uint32_t first_lo = 0xFFFFFFFFu, first_hi = 0xFFFFFFFFu;
    if (lane < a.S) first_lo = a.seg[lane].first_block;
    if (lane + 64 < a.S) first_hi = a.seg[lane + 64].first_block;
    const uint64_t lo = __ballot(blockIdx.x >= first_lo), hi = __ballot(blockIdx.x >= first_hi);
    const int s = hi ? 127 - __builtin_clzll(hi) : 63 - __builtin_clzll(lo | 1ull);
    const MergeSeg &sg = a.seg[s];
    const uint32_t next_first = (s + 1 < a.S) ? a.seg[s + 1].first_block : a.blocks;
    const uint32_t blk = blockIdx.x - sg.first_block, nblk = next_first - sg.first_block;
    const size_t total = static_cast<size_t>(sg.n) * sizeof(R);
    size_t head = (16 - reinterpret_cast<uintptr_t>(sg.y) % 16) % 16;
    if (head > total) head = total;
    const int32_t *idx = a.idx + sg.pair_off;
    const R *val = static_cast<const R *>(a.val) + sg.pair_off;
    const bool stream = a.stream != 0;
    if (sg.dense) merge_span_lds<R, int32_t>(idx, val, sg.k, sg.y, total, head, a.span, blk, nblk, stream, piece, s_range);
    else merge_span<R, int32_t>(idx, val, sg.k, sg.y, total, head, a.span, blk, nblk, stream, s_range);
}

#ifdef ADATOPK_MEASURE_BUILD
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

#endif

// ------------------------------------------------------------------ host side: plan and launch
using adatopk_internal::align_up;
using adatopk_internal::dtype_ok;
using adatopk_internal::elem_size;
using adatopk_internal::wire_val_offset;

// Elements per chunk for a launch of S_batch tensors holding n_batch elements: a multiple of the
// tile such that the chunks of all tensors together (every tensor's last chunk may be partial, an
// empty tensor still gets one) number at most `target`: n_batch / E + S_batch <= target.
int64_t chunk_elems(int64_t n_batch, int32_t S_batch, int64_t target) {
    const int64_t tile = TILE;
    const int64_t full = target - S_batch;  // S_batch <= MAXSEG < target
    int64_t e = (n_batch + full - 1) / full;
    if (e < tile) e = tile;
    return (e + tile - 1) / tile * tile;
}
inline int64_t chunk_target(int32_t S_batch) { return S_batch == 1 ? CTARGET_ONE : CTARGET; }

struct Carve {
    size_t state, G3, rows1, coarse1, rowsW, coarseW, cpairA, cnt, chunk_err, rows3, ldef, lerr, wire_err, L_idx, L_val,
        total;
};

// Workspace layout for up to max_chunks chunks and list_slots candidate-list slots.
Carve carve(int64_t max_chunks, int64_t list_slots, int32_t S, adatopk_dtype dt) {
    const int64_t max_parts = max_chunks * (S == 1 ? MAXSUB_ONE : MAXSUB);
    Carve c;
    size_t p = 0;
    auto take = [&](size_t bytes) {
        const size_t at = p;
        p = align_up(p + bytes, 256);
        return at;
    };
    c.state = take(sizeof(SegState) * MAXSEG);
    c.G3 = take(sizeof(uint32_t) * NB3 * MAXSEG);
    c.rows1 = take(sizeof(uint32_t) * NB1 * max_chunks);
    c.coarse1 = take(sizeof(uint32_t) * NC1 * max_chunks);
    c.rowsW = take(sizeof(uint32_t) * NBW * max_chunks);
    c.coarseW = take(sizeof(uint32_t) * NCW * max_chunks);
    c.cpairA = take(sizeof(uint2) * max_chunks);
    c.cnt = take(sizeof(uint32_t) * max_chunks);
    c.chunk_err = take(sizeof(double) * max_chunks);
    c.rows3 = take(sizeof(uint32_t) * NB3 * max_parts);
    c.ldef = take(sizeof(uint32_t) * max_parts);
    c.lerr = take(sizeof(double) * max_parts);
    c.wire_err = take(sizeof(float) * static_cast<size_t>(S < 1 ? 1 : S));  // error norms on their way into message headers
    c.L_idx = take(sizeof(int32_t) * static_cast<size_t>(list_slots));
    c.L_val = take(static_cast<size_t>(elem_size(dt)) * static_cast<size_t>(list_slots));
    c.total = p;
    return c;
}

// Upper bounds on the chunks and the list slots of any one launch of a call over n_total elements
// in S tensors: a launch holds at most MAXSEG tensors and at most chunk_target() chunks of
// chunk_elems() elements, and no launch holds more elements than the whole call.
void bounds_for(int64_t n_total, int32_t S, int64_t *max_chunks, int64_t *list_slots) {
    const int32_t batch = S > MAXSEG ? MAXSEG : (S < 1 ? 1 : S);
    const int64_t target = chunk_target(batch);
    *max_chunks = target;
    *list_slots = target * (chunk_elems(n_total, batch, target) / LIST_DIV);
}

// Every kernel launch of the library goes through launch().  The stage names the kernel for the
// measuring build of this file (ADATOPK_MEASURE_BUILD, a library of its own next to the product
// library), which gives every launch start / stop events carrying the timestamps of the dispatch
// itself, as a profiler sees it; the product build launches plainly and keeps no state.
enum Stage {
    ST_SPEC, ST_HIST1, ST_SCAN, ST_REFINE, ST_EMIT, ST_FILL, ST_SCATTER, ST_MERGE, ST_HEADER, ST_SMALL, ST_ALL, NSTAGE
};
#ifdef ADATOPK_MEASURE_BUILD
const char *const kStageNames[NSTAGE] = {"k_scan_spec", "k_hist1", "k_scan", "k_refine", "k_emit",
                                         "k_fill", "k_scatter", "k_merge", "k_wire_header", "k_small", "k_keep_all"};
bool g_measure = false;
bool g_events_made = false;
hipEvent_t g_start[NSTAGE], g_stop[NSTAGE];
bool g_ran[NSTAGE];  // launched, with events, since the last read
#endif

template <typename K, typename... Args>
inline void launch(int stage, K kernel, dim3 grid, hipStream_t st, Args... args) {
#ifdef ADATOPK_MEASURE_BUILD
    if (g_measure) {
        hipExtLaunchKernelGGL(kernel, grid, dim3(BLOCK), 0, st, g_start[stage], g_stop[stage], 0, args...);
        g_ran[stage] = true;
        return;
    }
#endif
    (void)stage;
    hipLaunchKernelGGL(kernel, grid, dim3(BLOCK), 0, st, args...);
}

// The kernels of one launch.  With `speculate` the first full read of the input is the speculative
// scan; the two exact passes behind it return at once for every tensor whose speculation held and
// do the work for the others, so what reaches k_refine is complete either way.
template <int VEC> adatopk_status launch_batch(const Launch &a, int total_chunks, bool speculate, hipStream_t st) {
    const dim3 grid(total_chunks);
    const bool one_per_cu = total_chunks <= CTARGET_ONE;  // the scan can afford the deeper pipeline
    if (speculate) {
        if (one_per_cu) launch(ST_SPEC, k_scan<VEC, true, 3>, grid, st, a);
        else launch(ST_SPEC, k_scan<VEC, true, 2>, grid, st, a);
    }
    launch(ST_HIST1, k_hist1<VEC>, grid, st, a);
    if (one_per_cu) launch(ST_SCAN, k_scan<VEC, false, 3>, grid, st, a);
    else launch(ST_SCAN, k_scan<VEC, false, 2>, grid, st, a);
    const dim3 parts(total_chunks * (VEC == TAG_F32 ? a.sub : 1u));
    if (one_per_cu && parts.x == grid.x) {  // one workgroup per chunk, at most one per compute unit: see Wide
        if constexpr (VEC == TAG_F32) launch(ST_REFINE, k_refine<VEC, true>, parts, st, a);  // the 16-bit types have no last digit to refine
        launch(ST_EMIT, k_emit<VEC, true>, parts, st, a);
    } else {
        if constexpr (VEC == TAG_F32) launch(ST_REFINE, k_refine<VEC, false>, parts, st, a);
        launch(ST_EMIT, k_emit<VEC, false>, parts, st, a);
    }
    return hipGetLastError() == hipSuccess ? ADATOPK_OK : ADATOPK_ERUNTIME;
}

// Where a compress call writes.  Plain: idx_out / val_out arrays, tensor s at element offset[s]
// (offset = exclusive scan of k, S + 1 entries).  Wire: one message buffer (idx_out), tensor s's
// message at byte offset[s] (S entries): its index section behind the header, its values behind the
// padded indices, and the error norms in the workspace (err_out is ignored) for the header kernel
// to pick up.
struct OutSpec {
    void *idx_out;
    int idx_bytes;
    void *val_out;
    const int64_t *offset;
    bool wire;
};

// Size of the sample and the ranks in it that bracket the k-th key of a tensor of n elements, or
// false when the speculative pass is not worth it for this tensor (small tensors; keep counts so
// small that even the largest sample says little about the k-th key; keep counts so large that the
// candidates would not fit the chunks' lists anyway).  Of ns sampled elements, mu = k * ns / n are
// expected among the k largest, with a standard deviation of at most sqrt(mu); the bracket is
// SPEC_SIGMAS of them towards the larger keys and SPEC_SIGMAS_LOW towards the smaller ones (a
// bracket that misses costs the two exact passes, about one call in four thousand at 3.5; every
// key down to the lower end is a candidate in every call: 3.5 instead of 5 takes 3 us off a tensor
// of 25 M elements at k = 10 %).  The sample is the smallest of a quarter, half or all of
// SAMPLE_ELEMS that expects SPEC_GOOD_EXPECTED kept elements, and the largest otherwise.
bool speculation_ranks(int64_t n, int64_t k, adatopk_dtype dt, bool aligned16, uint32_t *r_lo, uint32_t *r_hi,
                       uint32_t *batches) {
    if (!aligned16 || n < SPEC_MIN_N || k <= 0 || k > n / 100 * SPEC_MAX_KEEP_PERCENT) return false;
    const int epd = 4 / elem_size(dt);
    const int max_batches = SAMPLE_ELEMS / BLOCK / epd / SAMPLE_BATCH;
    double mu = 0.0;
    int nb = max_batches;
    for (int b = 1; b <= max_batches; b *= 2) {
        mu = static_cast<double>(k) * (static_cast<double>(b) * SAMPLE_BATCH * BLOCK * epd) / static_cast<double>(n);
        nb = b;
        if (mu >= (epd == 2 ? SPEC_GOOD_EXPECTED_16 : SPEC_GOOD_EXPECTED)) break;
    }
    if (mu < SPEC_MIN_EXPECTED) return false;
    const double margin = SPEC_SIGMAS * sqrt(mu) + 2.0;
    const double lo = ceil(mu + SPEC_SIGMAS_LOW * sqrt(mu) + 2.0), hi = floor(mu - margin);
    *r_lo = lo > 4.0e9 ? 0xFFFFFFFFu : static_cast<uint32_t>(lo);
    *r_hi = hi < 1.0 ? 0u : static_cast<uint32_t>(hi);
    *batches = static_cast<uint32_t>(nb);
    return true;
}

adatopk_status compress_impl(const void *const *dense, const int64_t *n, const int64_t *k, int32_t S,
                             adatopk_dtype dt, const OutSpec &out, float *err_out, void *workspace,
                             size_t workspace_bytes, hipStream_t st) {
    if (!dtype_ok(dt) || S < 0) return ADATOPK_EINVAL;
    if (S == 0) return ADATOPK_OK;
    if (!dense || !n || !k || !out.offset) return ADATOPK_EINVAL;
    const int es = elem_size(dt);
    const int idx_bytes = out.idx_bytes;
    void *const idx_out = out.idx_out;
    void *const val_out = out.val_out;
    const int64_t *const out_offset = out.offset;
    int64_t n_total = 0, k_total = 0;
    if (!out.wire && out_offset[0] != 0) return ADATOPK_EINVAL;
    for (int32_t s = 0; s < S; ++s) {
        if (n[s] < 0 || n[s] >= (static_cast<int64_t>(1) << 31) || k[s] < 0 || k[s] > n[s]) return ADATOPK_EINVAL;
        if (n[s] > 0 && (!dense[s] || reinterpret_cast<uintptr_t>(dense[s]) % es)) return ADATOPK_EINVAL;
        if (!out.wire && out_offset[s + 1] != out_offset[s] + k[s]) return ADATOPK_EINVAL;
        if (out.wire && (out_offset[s] < 0 || out_offset[s] % 16)) return ADATOPK_EINVAL;
        n_total += n[s];
        k_total += k[s];
    }
    if (k_total > 0 && (!idx_out || (!out.wire && !val_out))) return ADATOPK_EINVAL;
    if (reinterpret_cast<uintptr_t>(idx_out) % (out.wire ? 16 : idx_bytes) || reinterpret_cast<uintptr_t>(val_out) % es ||
        reinterpret_cast<uintptr_t>(err_out) % 4)
        return ADATOPK_EINVAL;
    const size_t need = adatopk_workspace_bytes(n_total, S, dt);
    if (!workspace || reinterpret_cast<uintptr_t>(workspace) % 256) return ADATOPK_EINVAL;
    if (workspace_bytes < need) return ADATOPK_EWORKSPACE;
    int64_t max_chunks, list_slots;
    bounds_for(n_total, S, &max_chunks, &list_slots);
    const Carve cv = carve(max_chunks, list_slots, S, dt);
    char *ws = static_cast<char *>(workspace);
    if (out.wire) err_out = reinterpret_cast<float *>(ws + cv.wire_err);
    const int64_t header = out.wire ? static_cast<int64_t>(sizeof(adatopk_wire_header)) : 0;

    // Only small tensors: one launch, one workgroup per tensor, no workspace traffic.
    bool all_small = true;
    for (int32_t s = 0; s < S; ++s) all_small = all_small && n[s] <= SMALL_N;
    if (all_small) {
        for (int32_t s0 = 0; s0 < S; s0 += SMALL_MAXSEG) {
            SmallLaunch sl{};
            const int32_t cnt = (S - s0 < SMALL_MAXSEG) ? S - s0 : SMALL_MAXSEG;
            for (int32_t i = 0; i < cnt; ++i) {
                sl.seg[i].x = dense[s0 + i];
                sl.seg[i].out_off = out_offset[s0 + i] + header;
                sl.seg[i].n = static_cast<int32_t>(n[s0 + i]);
                sl.seg[i].k = static_cast<int32_t>(k[s0 + i]);
            }
            sl.idx_out = idx_out;
            sl.idx64 = idx_bytes == 8 ? 1u : 0u;
            sl.wire = out.wire ? 1u : 0u;
            sl.val_out = val_out;
            sl.err_out = err_out ? err_out + s0 : nullptr;
            if (dt == ADATOPK_F32) launch(ST_SMALL, k_small<TAG_F32>, dim3(cnt), st, sl);
            else if (dt == ADATOPK_BF16) launch(ST_SMALL, k_small<TAG_BF16>, dim3(cnt), st, sl);
            else launch(ST_SMALL, k_small<TAG_F16>, dim3(cnt), st, sl);
            if (hipGetLastError() != hipSuccess) return ADATOPK_ERUNTIME;
        }
        return ADATOPK_OK;
    }

    for (int32_t s0 = 0; s0 < S; s0 += MAXSEG) {
        Launch a{};
        a.S = (S - s0 < MAXSEG) ? S - s0 : MAXSEG;
        // Chunk size of this launch: at most chunk_target() chunks in all, so that all workgroups are
        // resident at once (a few chunks beyond that would run as a second, nearly empty round).
        // Tensors kept whole (k = n) take no part in the selection: they go through it as empty tensors
        // (one empty chunk each) and get their pairs from k_keep_all below.
        auto kept_whole = [&](int32_t s) { return n[s] > 0 && k[s] == n[s]; };
        auto n_select = [&](int32_t s) { return kept_whole(s) ? static_cast<int64_t>(0) : n[s]; };
        int64_t n_batch = 0;
        int32_t whole = 0;
        for (int32_t i = 0; i < a.S; ++i) {
            n_batch += n_select(s0 + i);
            whole += kept_whole(s0 + i) ? 1 : 0;
        }
        const int64_t target = chunk_target(a.S);
        const int64_t E_fits = chunk_elems(n_batch, a.S, target);  // fits whatever the tensors' lengths are
        int64_t E = (n_batch + target - 1) / target;
        E = E < TILE ? TILE : (E + TILE - 1) / TILE * TILE;
        auto chunks_at = [&](int64_t e) {
            int64_t count = 0;
            for (int32_t i = 0; i < a.S; ++i) count += n_select(s0 + i) > 0 ? (n_select(s0 + i) + e - 1) / e : 1;
            return count;
        };
        while (E < E_fits && chunks_at(E) > target) E += TILE;
        a.E = static_cast<int32_t>(E);
        a.cap = static_cast<uint32_t>(E / LIST_DIV);
        a.state = reinterpret_cast<SegState *>(ws + cv.state);
        a.G3 = reinterpret_cast<uint32_t *>(ws + cv.G3);
        a.rows1 = reinterpret_cast<uint32_t *>(ws + cv.rows1);
        a.coarse1 = reinterpret_cast<uint32_t *>(ws + cv.coarse1);
        a.rowsW = reinterpret_cast<uint32_t *>(ws + cv.rowsW);
        a.coarseW = reinterpret_cast<uint32_t *>(ws + cv.coarseW);
        a.cpairA = reinterpret_cast<uint2 *>(ws + cv.cpairA);
        a.cnt = reinterpret_cast<uint32_t *>(ws + cv.cnt);
        a.chunk_err = reinterpret_cast<double *>(ws + cv.chunk_err);
        a.rows3 = reinterpret_cast<uint32_t *>(ws + cv.rows3);
        a.ldef = reinterpret_cast<uint32_t *>(ws + cv.ldef);
        a.lerr = reinterpret_cast<double *>(ws + cv.lerr);
        a.L_idx = reinterpret_cast<int32_t *>(ws + cv.L_idx);
        a.L_val = ws + cv.L_val;
        a.idx_out = idx_out;
        a.idx64 = idx_bytes == 8 ? 1u : 0u;
        a.wire = out.wire ? 1u : 0u;
        a.val_out = val_out;
        a.err_out = err_out ? err_out + s0 : nullptr;
        int32_t chunks = 0;
        bool speculate = false;
        double densest = 0.0;  // largest keep fraction of the launch
        for (int32_t i = 0; i < a.S; ++i) {
            SegDesc &d = a.seg[i];
            const int32_t s = s0 + i;
            d.x = dense[s];
            d.out_off = out_offset[s] + header;
            const int64_t ns = n_select(s), ks = kept_whole(s) ? 0 : k[s];
            d.n = static_cast<int32_t>(ns);
            d.k = static_cast<int32_t>(ks);
            d.chunk_begin = chunks;
            d.nchunks = ns > 0 ? static_cast<int32_t>((ns + E - 1) / E) : 1;  // an empty tensor keeps one (empty) chunk
            const bool aligned4 = reinterpret_cast<uintptr_t>(dense[s]) % 4 == 0;
            d.flags = aligned4 ? FLAG_ALIGNED4 : 0u;
            const bool aligned16 = reinterpret_cast<uintptr_t>(dense[s]) % 16 == 0;  // the sample is read with 16-byte loads
            if (speculation_ranks(ns, ks, dt, aligned16, &d.r_lo, &d.r_hi, &d.sample_batches)) {
                d.flags |= FLAG_SPEC;
                speculate = true;
            }
            chunks += d.nchunks;
            if (ns > 0 && static_cast<double>(ks) / static_cast<double>(ns) > densest)
                densest = static_cast<double>(ks) / static_cast<double>(ns);
        }
        // parts per chunk for the list kernels: a chunk's candidates are about a third more than its kept
        // elements; a part gets about SUB_ENTRIES of them
        {
            const double per_chunk = 1.35 * densest * static_cast<double>(E);
            int sub = static_cast<int>(per_chunk / SUB_ENTRIES) + 1;
            const int most = S == 1 ? MAXSUB_ONE : MAXSUB;  // what the workspace of this call was laid out for
            a.sub = static_cast<uint32_t>(sub > most ? most : sub);
        }
        if (chunks > max_chunks || static_cast<int64_t>(chunks) * a.cap > list_slots) return ADATOPK_ERUNTIME;  // planner invariant
        if (whole < a.S) {  // something to select
            const adatopk_status rc = (dt == ADATOPK_F32)    ? launch_batch<TAG_F32>(a, chunks, speculate, st)
                                      : (dt == ADATOPK_BF16) ? launch_batch<TAG_BF16>(a, chunks, speculate, st)
                                                             : launch_batch<TAG_F16>(a, chunks, speculate, st);
            if (rc != ADATOPK_OK) return rc;
        }
        if (whole > 0) {
            // the same table with the kept-whole tensors at their true length, tile by tile, and the others empty
            Launch w = a;
            int32_t tiles = 0;
            for (int32_t i = 0; i < a.S; ++i) {
                SegDesc &d = w.seg[i];
                const int32_t s = s0 + i;
                d.n = kept_whole(s) ? static_cast<int32_t>(n[s]) : 0;
                d.k = d.n;
                d.chunk_begin = tiles;
                d.nchunks = static_cast<int32_t>((static_cast<int64_t>(d.n) + TILE - 1) / TILE);
                tiles += d.nchunks;
            }
            if (dt == ADATOPK_F32) launch(ST_ALL, k_keep_all<TAG_F32>, dim3(tiles), st, w);
            else if (dt == ADATOPK_BF16) launch(ST_ALL, k_keep_all<TAG_BF16>, dim3(tiles), st, w);
            else launch(ST_ALL, k_keep_all<TAG_F16>, dim3(tiles), st, w);
            if (hipGetLastError() != hipSuccess) return ADATOPK_ERUNTIME;
        }
    }
    return ADATOPK_OK;
}

int grid_for(size_t work_items, int per_thread) {
    size_t b = (work_items + static_cast<size_t>(BLOCK) * per_thread - 1) / (static_cast<size_t>(BLOCK) * per_thread);
    if (b < 1) b = 1;
    if (b > 4096) b = 4096;
    return static_cast<int>(b);
}

adatopk_status fill_impl(void *dst, size_t bytes, hipStream_t st) {  // the k_fill launch of decompress
    if (bytes == 0) return ADATOPK_OK;
    size_t head = (16 - reinterpret_cast<uintptr_t>(dst) % 16) % 16;
    if (head > bytes) head = bytes;
    const size_t body16 = (bytes - head) / 16;
    launch(ST_FILL, k_fill, dim3(grid_for(body16, 4)), st, static_cast<unsigned char *>(dst), bytes, head, body16);
    return hipGetLastError() == hipSuccess ? ADATOPK_OK : ADATOPK_ERUNTIME;
}

// Bytes of output per workgroup of the one-kernel decompress: about MERGE_SPANS workgroups, but
// spans neither so small that the search dominates nor so large that big outputs get too few
// workgroups (a multiple of 16).
inline size_t merge_span_bytes(size_t bytes) {
    size_t span = (bytes / MERGE_SPANS + 15) / 16 * 16;
    if (span < MERGE_MIN_SPAN) span = MERGE_MIN_SPAN;
    if (span > MERGE_MAX_SPAN) span = MERGE_MAX_SPAN;
    return span;
}

// ---- decompress, for either index width
adatopk_status check_pairs(const void *idx, int ib, const void *val, int64_t k, adatopk_dtype dt, const void *dense,
                           int64_t n) {
    if (!dtype_ok(dt) || n < 0 || k < 0 || k > n || n >= (static_cast<int64_t>(1) << 31)) return ADATOPK_EINVAL;
    const int es = elem_size(dt);
    if (n > 0 && (!dense || reinterpret_cast<uintptr_t>(dense) % es)) return ADATOPK_EINVAL;
    if (k > 0 && (!idx || !val || reinterpret_cast<uintptr_t>(idx) % ib || reinterpret_cast<uintptr_t>(val) % es))
        return ADATOPK_EINVAL;
    return ADATOPK_OK;
}

template <typename I>
void launch_scatter(const I *idx, const void *val, int64_t k, adatopk_dtype dt, void *y, int64_t n, hipStream_t st) {
    const dim3 grid(static_cast<unsigned>((k + BLOCK - 1) / BLOCK));
    if (dt == ADATOPK_F32)
        launch(ST_SCATTER, k_scatter<uint32_t, I>, grid, st, idx, static_cast<const uint32_t *>(val), k,
               static_cast<uint32_t *>(y), n);
    else
        launch(ST_SCATTER, k_scatter<uint16_t, I>, grid, st, idx, static_cast<const uint16_t *>(val), k,
               static_cast<uint16_t *>(y), n);
}

adatopk_status decompress_impl(const void *idx, int ib, const void *val, int64_t k, adatopk_dtype dt, void *dense_out,
                               int64_t n, hipStream_t st) {
    const adatopk_status ok = check_pairs(idx, ib, val, k, dt, dense_out, n);
    if (ok != ADATOPK_OK) return ok;
    if (n == 0) return ADATOPK_OK;
    const adatopk_status rc = fill_impl(dense_out, static_cast<size_t>(n) * elem_size(dt), st);
    if (rc != ADATOPK_OK) return rc;
    if (k > 0) {
        if (ib == 4) launch_scatter(static_cast<const int32_t *>(idx), val, k, dt, dense_out, n, st);
        else launch_scatter(static_cast<const int64_t *>(idx), val, k, dt, dense_out, n, st);
    }
    return hipGetLastError() == hipSuccess ? ADATOPK_OK : ADATOPK_ERUNTIME;
}

template <typename I>
void launch_scatter_add(const I *idx, const void *val, int64_t k, adatopk_dtype dt, void *y, int64_t n, hipStream_t st) {
    const dim3 grid(static_cast<unsigned>((k + BLOCK - 1) / BLOCK));
    if (dt == ADATOPK_F32)
        launch(ST_SCATTER, k_scatter_add<TAG_F32, I>, grid, st, idx, static_cast<const uint32_t *>(val), k,
               static_cast<uint32_t *>(y), n);
    else if (dt == ADATOPK_BF16)
        launch(ST_SCATTER, k_scatter_add<TAG_BF16, I>, grid, st, idx, static_cast<const uint16_t *>(val), k,
               static_cast<uint16_t *>(y), n);
    else
        launch(ST_SCATTER, k_scatter_add<TAG_F16, I>, grid, st, idx, static_cast<const uint16_t *>(val), k,
               static_cast<uint16_t *>(y), n);
}

adatopk_status accumulate_impl(const void *idx, int ib, const void *val, int64_t k, adatopk_dtype dt, void *dense_inout,
                               int64_t n, hipStream_t st) {
    const adatopk_status ok = check_pairs(idx, ib, val, k, dt, dense_inout, n);
    if (ok != ADATOPK_OK) return ok;
    if (n == 0 || k == 0) return ADATOPK_OK;
    if (ib == 4) launch_scatter_add(static_cast<const int32_t *>(idx), val, k, dt, dense_inout, n, st);
    else launch_scatter_add(static_cast<const int64_t *>(idx), val, k, dt, dense_inout, n, st);
    return hipGetLastError() == hipSuccess ? ADATOPK_OK : ADATOPK_ERUNTIME;
}

template <typename R, typename I>
void launch_merge(bool dense, unsigned grid, hipStream_t st, const I *idx, const R *val, uint32_t k, unsigned char *y,
                  size_t total, size_t head, size_t span) {
    const uint32_t stream = total > STREAM_STORE_BYTES ? 1u : 0u;
    if (dense) launch(ST_MERGE, k_merge_lds<R, I>, dim3(grid), st, idx, val, k, y, total, head, span, stream);
    else launch(ST_MERGE, k_merge<R, I>, dim3(grid), st, idx, val, k, y, total, head, span, stream);
}

adatopk_status decompress_sorted_impl(const void *idx, int ib, const void *val, int64_t k, adatopk_dtype dt,
                                      void *dense_out, int64_t n, hipStream_t st) {
    const adatopk_status ok = check_pairs(idx, ib, val, k, dt, dense_out, n);
    if (ok != ADATOPK_OK) return ok;
    if (n == 0) return ADATOPK_OK;
    const int es = elem_size(dt);
    const size_t total = static_cast<size_t>(n) * es;
    size_t head = (16 - reinterpret_cast<uintptr_t>(dense_out) % 16) % 16;
    if (head > total) head = total;
    const size_t body = total - head;
    const size_t span = merge_span_bytes(body);
    const unsigned grid = static_cast<unsigned>(body / span + 1);  // the last workgroup takes the remainder
    const bool dense = k > n / MERGE_DENSE_RATIO;  // more than one entry per few lines: build the lines in LDS
    const uint32_t ku = static_cast<uint32_t>(k);
    unsigned char *yb = static_cast<unsigned char *>(dense_out);
    if (es == 4) {
        const uint32_t *v = static_cast<const uint32_t *>(val);
        if (ib == 4) launch_merge(dense, grid, st, static_cast<const int32_t *>(idx), v, ku, yb, total, head, span);
        else launch_merge(dense, grid, st, static_cast<const int64_t *>(idx), v, ku, yb, total, head, span);
    } else {
        const uint16_t *v = static_cast<const uint16_t *>(val);
        if (ib == 4) launch_merge(dense, grid, st, static_cast<const int32_t *>(idx), v, ku, yb, total, head, span);
        else launch_merge(dense, grid, st, static_cast<const int64_t *>(idx), v, ku, yb, total, head, span);
    }
    return hipGetLastError() == hipSuccess ? ADATOPK_OK : ADATOPK_ERUNTIME;
}

// ---- decompress of several tensors (ascending indices per tensor) in as few launches as the table allows
adatopk_status decompress_segmented_impl(const int32_t *idx, const void *val, const int64_t *out_offset, int32_t S,
                                         adatopk_dtype dt, void *const *dense_out, const int64_t *n, hipStream_t st) {
    if (!dtype_ok(dt) || S < 0) return ADATOPK_EINVAL;
    if (S == 0) return ADATOPK_OK;
    if (!out_offset || !dense_out || !n || out_offset[0] != 0) return ADATOPK_EINVAL;
    const int es = elem_size(dt);
    size_t bytes_all = 0;
    for (int32_t s = 0; s < S; ++s) {
        const int64_t k = out_offset[s + 1] - out_offset[s];
        if (n[s] < 0 || n[s] >= (static_cast<int64_t>(1) << 31) || k < 0 || k > n[s]) return ADATOPK_EINVAL;
        if (n[s] > 0 && (!dense_out[s] || reinterpret_cast<uintptr_t>(dense_out[s]) % es)) return ADATOPK_EINVAL;
        bytes_all += static_cast<size_t>(n[s]) * es;
    }
    if (out_offset[S] > 0 && (!idx || !val || reinterpret_cast<uintptr_t>(idx) % 4 || reinterpret_cast<uintptr_t>(val) % es))
        return ADATOPK_EINVAL;
    const size_t span = merge_span_bytes(bytes_all);  // one span size for the call
    for (int32_t s0 = 0; s0 < S; s0 += MERGE_MAXSEG) {
        MergeLaunch a{};
        a.S = (S - s0 < MERGE_MAXSEG) ? S - s0 : MERGE_MAXSEG;
        a.idx = idx;
        a.val = val;
        a.span = span;
        a.stream = bytes_all > STREAM_STORE_BYTES ? 1u : 0u;
        uint64_t blocks = 0;
        for (int32_t i = 0; i < a.S; ++i) {
            const int32_t s = s0 + i;
            MergeSeg &g = a.seg[i];
            const int64_t k = out_offset[s + 1] - out_offset[s];
            g.y = static_cast<unsigned char *>(dense_out[s]);
            g.pair_off = out_offset[s];
            g.n = n[s];
            g.k = static_cast<uint32_t>(k);
            g.first_block = static_cast<uint32_t>(blocks);
            g.dense = k > n[s] / MERGE_DENSE_RATIO ? 1u : 0u;
            if (n[s] > 0) {  // same span count as the kernel derives: (bytes behind the unaligned head) / span + 1
                const size_t total = static_cast<size_t>(n[s]) * es;
                size_t head = (16 - reinterpret_cast<uintptr_t>(dense_out[s]) % 16) % 16;
                if (head > total) head = total;
                blocks += (total - head) / span + 1;
            }
        }
        a.blocks = static_cast<uint32_t>(blocks);
        if (blocks == 0) continue;
        if (blocks > 0x7FFFFFFFull) return ADATOPK_EINVAL;
        const dim3 grid(static_cast<unsigned>(blocks));
        if (es == 4) launch(ST_MERGE, k_merge_seg<uint32_t>, grid, st, a);
        else launch(ST_MERGE, k_merge_seg<uint16_t>, grid, st, a);
        if (hipGetLastError() != hipSuccess) return ADATOPK_ERUNTIME;
    }
    return ADATOPK_OK;
}

// ---- wire message: header | indices, padded to 16 bytes | values
struct WireWords {
    uint32_t w[sizeof(adatopk_wire_header) / 4];
};
// Headers of up to HDR_MAXSEG messages in one launch, after the compress kernels: workgroup s stores
// the header words of message s (built on the host; the error norm comes from err[s], which the
// compress kernels left in the workspace) and zeroes the padding between its index and value sections.
constexpr int HDR_MAXSEG = 48;
struct HeaderLaunch {
    WireWords hdr[HDR_MAXSEG];
    int64_t msg_off[HDR_MAXSEG];  // byte offset of the message in the buffer
    unsigned char *base;
    const float *err;
};
static_assert(sizeof(HeaderLaunch) <= 4096, "kernel arguments stay within 4 KB");
__global__ __launch_bounds__(BLOCK) void k_wire_header(const HeaderLaunch a) {
    const int s = blockIdx.x;
    const uint32_t t = threadIdx.x;
    unsigned char *msg = a.base + a.msg_off[s];
    constexpr uint32_t ERR_WORD = offsetof(adatopk_wire_header, err_norm) / 4;
    if (t < sizeof(adatopk_wire_header) / 4)
        reinterpret_cast<uint32_t *>(msg)[t] = (t == ERR_WORD) ? __float_as_uint(a.err[s]) : a.hdr[s].w[t];
    const WireWords &h = a.hdr[s];
    const uint64_t k = h.w[offsetof(adatopk_wire_header, k) / 4] |
                       (static_cast<uint64_t>(h.w[offsetof(adatopk_wire_header, k) / 4 + 1]) << 32);
    const uint64_t voff = h.w[offsetof(adatopk_wire_header, val_offset) / 4] |
                          (static_cast<uint64_t>(h.w[offsetof(adatopk_wire_header, val_offset) / 4 + 1]) << 32);
    const uint32_t ib = h.w[offsetof(adatopk_wire_header, index_bytes) / 4] & 0xFFu;
    const uint64_t pad_a = sizeof(adatopk_wire_header) + k * ib;
    if (pad_a + t < voff) msg[pad_a + t] = 0;  // at most 15 bytes
}

// Compress of S tensors into S wire messages in one buffer (message s at byte msg_off[s]).
adatopk_status compress_wire_impl(const void *const *dense, const int64_t *n, const int64_t *k, int32_t S,
                                  adatopk_dtype dt, int32_t index_bytes, const double *ratio, void *wire_out,
                                  const int64_t *msg_off, size_t wire_capacity, void *workspace,
                                  size_t workspace_bytes, hipStream_t st) {
    if (index_bytes != 4 && index_bytes != 8) return ADATOPK_EINVAL;
    if (!dtype_ok(dt) || S < 0) return ADATOPK_EINVAL;
    if (S == 0) return ADATOPK_OK;
    if (!dense || !n || !k || !msg_off || !wire_out || reinterpret_cast<uintptr_t>(wire_out) % 16) return ADATOPK_EINVAL;
    // messages in ascending, non-overlapping positions inside the buffer
    int64_t end_prev = 0;
    for (int32_t s = 0; s < S; ++s) {
        if (n[s] < 0 || k[s] < 0 || k[s] > n[s] || n[s] >= (static_cast<int64_t>(1) << 31)) return ADATOPK_EINVAL;
        const size_t bytes = adatopk_wire_bytes(k[s], dt, index_bytes);
        if (bytes == 0 || msg_off[s] % 16 || msg_off[s] < end_prev) return ADATOPK_EINVAL;
        end_prev = msg_off[s] + static_cast<int64_t>(bytes);
    }
    if (static_cast<uint64_t>(end_prev) > wire_capacity) return ADATOPK_EINVAL;
    const OutSpec out{wire_out, index_bytes, nullptr, msg_off, true};
    const adatopk_status rc = compress_impl(dense, n, k, S, dt, out, nullptr, workspace, workspace_bytes, st);
    if (rc != ADATOPK_OK) return rc;
    // the error norms are in the workspace now (stream order): write the headers around them
    int64_t n_total = 0;
    for (int32_t s = 0; s < S; ++s) n_total += n[s];
    int64_t max_chunks, list_slots;
    bounds_for(n_total, S, &max_chunks, &list_slots);
    const float *err = reinterpret_cast<const float *>(static_cast<char *>(workspace) +
                                                       carve(max_chunks, list_slots, S, dt).wire_err);
    for (int32_t s0 = 0; s0 < S; s0 += HDR_MAXSEG) {
        HeaderLaunch a{};
        const int32_t cnt = (S - s0 < HDR_MAXSEG) ? S - s0 : HDR_MAXSEG;
        for (int32_t i = 0; i < cnt; ++i) {
            const int32_t s = s0 + i;
            adatopk_wire_header h;
            memset(&h, 0, sizeof h);
            h.magic = ADATOPK_WIRE_MAGIC;
            h.version = ADATOPK_WIRE_VERSION;
            h.algorithm = ADATOPK_WIRE_TOPK;
            h.dtype = static_cast<uint8_t>(dt);
            h.index_bytes = static_cast<uint8_t>(index_bytes);
            h.n = n[s];
            h.k = k[s];
            h.ratio = ratio ? ratio[s] : (k[s] > 0 ? static_cast<double>(n[s]) / static_cast<double>(k[s]) : 0.0);
            h.idx_offset = sizeof(adatopk_wire_header);
            h.val_offset = static_cast<int64_t>(wire_val_offset(k[s], index_bytes));
            memcpy(&a.hdr[i], &h, sizeof h);
            a.msg_off[i] = msg_off[s];
        }
        a.base = static_cast<unsigned char *>(wire_out);
        a.err = err + s0;
        launch(ST_HEADER, k_wire_header, dim3(cnt), st, a);
        if (hipGetLastError() != hipSuccess) return ADATOPK_ERUNTIME;
    }
    return ADATOPK_OK;
}

// Device address of `scratch` on the current device: every GPU holds its own copy of the array at
// its own address, looked up on the first call made with that device current and kept.
constexpr int MAX_DEVICES = 64;
std::atomic<void *> g_scratch_ptr[MAX_DEVICES];
adatopk_status scratch_of_current_device(void **out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return ADATOPK_ERUNTIME;
    void *ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (ptr == nullptr) {
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) return ADATOPK_ERUNTIME;
        g_scratch_ptr[dev].store(ptr, std::memory_order_release);  // two threads racing here store the same address
    }
    *out = ptr;
    return ADATOPK_OK;
}

}  // namespace

// ------------------------------------------------------------------ C ABI
extern "C" {

size_t adatopk_workspace_bytes(int64_t n_total, int32_t num_segments, adatopk_dtype dt) {
    if (n_total < 0 || num_segments < 1 || !dtype_ok(dt)) return 0;
    int64_t max_chunks, list_slots;
    bounds_for(n_total, num_segments, &max_chunks, &list_slots);
    return carve(max_chunks, list_slots, num_segments, dt).total;
}

adatopk_status adatopk_compress(const void *dense, int64_t n, adatopk_dtype dt, int64_t k, int32_t *idx_out,
                                void *val_out, float *err_norm_out, void *workspace, size_t workspace_bytes,
                                void *hip_stream) {
    const void *ptrs[1] = {dense};
    const int64_t off[2] = {0, k};
    const OutSpec out{idx_out, 4, val_out, off, false};
    return compress_impl(ptrs, &n, &k, 1, dt, out, err_norm_out, workspace, workspace_bytes,
                         static_cast<hipStream_t>(hip_stream));
}

adatopk_status adatopk_compress_noalloc(const void *dense, int64_t n, adatopk_dtype dt, int64_t k, int32_t *idx_out,
                                        void *val_out, float *err_norm_out, void *hip_stream) {
    if (!dtype_ok(dt) || n < 0 || n >= (static_cast<int64_t>(1) << 31)) return ADATOPK_EINVAL;
    if (adatopk_workspace_bytes(n, 1, dt) > ADATOPK_NOALLOC_SCRATCH_BYTES) return ADATOPK_EWORKSPACE;
    void *ptr = nullptr;
    const adatopk_status rc = scratch_of_current_device(&ptr);
    if (rc != ADATOPK_OK) return rc;
    // Every kernel of the call clears what it accumulates into before using it, so what the previous
    // call left in the array does not matter.
    const void *ptrs[1] = {dense};
    const int64_t off[2] = {0, k};
    const OutSpec out{idx_out, 4, val_out, off, false};
    return compress_impl(ptrs, &n, &k, 1, dt, out, err_norm_out, ptr, ADATOPK_NOALLOC_SCRATCH_BYTES,
                         static_cast<hipStream_t>(hip_stream));
}

adatopk_status adatopk_compress_segmented(const void *const *dense, const int64_t *n, const int64_t *k, int32_t S,
                                          adatopk_dtype dt, int32_t *idx_out, void *val_out,
                                          const int64_t *out_offset, float *err_norm_out, void *workspace,
                                          size_t workspace_bytes, void *hip_stream) {
    const OutSpec out{idx_out, 4, val_out, out_offset, false};
    return compress_impl(dense, n, k, S, dt, out, err_norm_out, workspace, workspace_bytes,
                         static_cast<hipStream_t>(hip_stream));
}

adatopk_status adatopk_decompress(const int32_t *idx, const void *val, int64_t k, adatopk_dtype dt, void *dense_out,
                                  int64_t n, void *hip_stream) {
    return decompress_impl(idx, 4, val, k, dt, dense_out, n, static_cast<hipStream_t>(hip_stream));
}

adatopk_status adatopk_decompress_accumulate(const int32_t *idx, const void *val, int64_t k, adatopk_dtype dt,
                                             void *dense_inout, int64_t n, void *hip_stream) {
    return accumulate_impl(idx, 4, val, k, dt, dense_inout, n, static_cast<hipStream_t>(hip_stream));
}

adatopk_status adatopk_decompress_sorted(const int32_t *idx, const void *val, int64_t k, adatopk_dtype dt,
                                         void *dense_out, int64_t n, void *hip_stream) {
    return decompress_sorted_impl(idx, 4, val, k, dt, dense_out, n, static_cast<hipStream_t>(hip_stream));
}

adatopk_status adatopk_decompress_segmented(const int32_t *idx, const void *val, const int64_t *out_offset, int32_t S,
                                            adatopk_dtype dt, void *const *dense_out, const int64_t *n,
                                            void *hip_stream) {
    return decompress_segmented_impl(idx, val, out_offset, S, dt, dense_out, n, static_cast<hipStream_t>(hip_stream));
}

// ---- wire format (the host-only helpers are in adatopk_host.cpp)
adatopk_status adatopk_compress_wire(const void *dense, int64_t n, adatopk_dtype dt, int64_t k, int32_t index_bytes,
                                     double ratio, void *wire_out, size_t wire_capacity, void *workspace,
                                     size_t workspace_bytes, void *hip_stream) {
    const void *ptrs[1] = {dense};
    const int64_t off[1] = {0};
    return compress_wire_impl(ptrs, &n, &k, 1, dt, index_bytes, &ratio, wire_out, off, wire_capacity, workspace,
                              workspace_bytes, static_cast<hipStream_t>(hip_stream));
}

adatopk_status adatopk_compress_wire_segmented(const void *const *dense, const int64_t *n, const int64_t *k, int32_t S,
                                               adatopk_dtype dt, int32_t index_bytes, const double *ratio,
                                               void *wire_out, const int64_t *wire_offset, size_t wire_capacity,
                                               void *workspace, size_t workspace_bytes, void *hip_stream) {
    return compress_wire_impl(dense, n, k, S, dt, index_bytes, ratio, wire_out, wire_offset, wire_capacity, workspace,
                              workspace_bytes, static_cast<hipStream_t>(hip_stream));
}

adatopk_status adatopk_decompress_wire(const void *wire, size_t wire_bytes, adatopk_dtype dt, int32_t index_bytes,
                                       int64_t n, int32_t accumulate, void *dense, void *hip_stream) {
    const int64_t k = adatopk_wire_keep_count(wire_bytes, dt, index_bytes);
    if (k < 0 || n < 0 || k > n || !wire || reinterpret_cast<uintptr_t>(wire) % 16) return ADATOPK_EINVAL;
    const char *w = static_cast<const char *>(wire);
    const void *idx = w + sizeof(adatopk_wire_header);
    const void *val = w + wire_val_offset(k, index_bytes);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (accumulate) return accumulate_impl(idx, index_bytes, val, k, dt, dense, n, st);
    return decompress_sorted_impl(idx, index_bytes, val, k, dt, dense, n, st);
}

#ifdef ADATOPK_MEASURE_BUILD
// ---- measurement hooks
adatopk_status adatopk_measure_enable(int32_t on) {
    if (on && !g_events_made) {
        for (int i = 0; i < NSTAGE; ++i)
            if (hipEventCreate(&g_start[i]) != hipSuccess || hipEventCreate(&g_stop[i]) != hipSuccess)
                return ADATOPK_ERUNTIME;
        g_events_made = true;
    }
    g_measure = on != 0;
    for (int i = 0; i < NSTAGE; ++i) g_ran[i] = false;
    return ADATOPK_OK;
}

int32_t adatopk_measure_stage_count(void) { return NSTAGE; }

const char *adatopk_measure_stage_name(int32_t stage) {
    return (stage >= 0 && stage < NSTAGE) ? kStageNames[stage] : "";
}

adatopk_status adatopk_measure_read(float *ms_out) {
    if (!ms_out || !g_events_made) return ADATOPK_EINVAL;
    for (int i = 0; i < NSTAGE; ++i) {
        ms_out[i] = -1.0f;
        if (!g_ran[i]) continue;
        g_ran[i] = false;
        if (hipEventSynchronize(g_stop[i]) != hipSuccess) return ADATOPK_ERUNTIME;
        if (hipEventElapsedTime(&ms_out[i], g_start[i], g_stop[i]) != hipSuccess) return ADATOPK_ERUNTIME;
    }
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
#endif  // ADATOPK_MEASURE_BUILD

}  // extern "C"
