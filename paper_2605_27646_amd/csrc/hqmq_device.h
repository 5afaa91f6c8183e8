// Internal declarations shared by the HQMQ gfx950 kernels and the host-side launch code.
// Not part of the public ABI (that is include/hqmq.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "hqmq.h"

namespace hqmq {

constexpr int kChunksPerRow = 32;    // chunks of a row of D = 128 elements, and the most a row may have
constexpr int kSearchRowsSmall = 64;   // rows per search workgroup = granularity of the outlier scan:
constexpr int kSearchRowsLarge = 256;  // 64 for short segments (more workgroups), 256 from 2048 rows on,
constexpr int kSearchRowsHuge = 512;   // 512 from 4096 rows on (16-wave workgroups)
constexpr int kSearchRowsSwitch = 2048;
constexpr int kSearchRowsSwitchHuge = 4096;
constexpr int kThreads = 256;        // default workgroup: 4 wave64
constexpr int kATiles = 2;           // 64-lane x 16-byte MFMA A operand tiles per 16 secondaries (8 secondaries each)

// Radix select over the 63 value bits of a non-negative IEEE double.  The sequence-sharded select takes
// bits 62..50, then 10 bits per pass.  The single-tensor select takes exponent and 6 mantissa bits first
// (17-bit prefix minus kFineBase, clamped to the kBins0 bins: what squares of fp16 data need), collects the
// keys of that bin as candidates and, should they overflow their list, narrows by bits 45..36.
constexpr int kBits0 = 13, kShift0 = 50, kBins0 = 1 << kBits0;  // bits 62..50
constexpr int kBits1 = 10, kShift1 = 40, kBins1 = 1 << kBits1;  // bits 49..40
constexpr int kFineShift = 46;                      // first digit of the single-tensor select: key >> 46 ...
constexpr uint32_t kFineBase = (975u << 6) - 1u;    // ... minus this: 2^-48, the smallest square of an fp16 value, lands in bin 1
constexpr int kSecShift = kFineShift - kBits1;      // its second digit: bits 45..36
constexpr int kCandCap = 32768;      // candidate keys kept per head, at least (Geometry::cand_cap: more for very long heads)
static_assert(kBins0 * sizeof(uint32_t) <= kCandCap * sizeof(unsigned long long),
              "the sample histogram borrows the candidate list's memory");
constexpr int kSelectThreads = 1024; // workgroup of the select sweeps
constexpr int kSelectRows = 1024;    // rows of one (b, h) segment per select workgroup
constexpr int kScreenMaxS = 512;      // largest S whose search is screened on the matrix cores (operand tables in LDS)
constexpr int kSampleStride = 16;     // the sampled select reads every 16th row of a head first ...
constexpr int kSampleMinChunks = 1 << 17;  // ... when the head has at least this many chunks
constexpr int kSmallListRows = 4096;   // a tensor of at most this many rows and kSmallListBlocks search workgroups,
constexpr int kSmallListBlocks = 1024; // with thresholds known beforehand, is encoded by two launches

// Per-head state of the running radix select.
struct SelectState {
    unsigned long long prefix;  // key bits fixed so far (right aligned)
    uint32_t rank;              // rank still to be located inside the prefix bucket
    uint32_t pad;
};

// Per-head plan of the sampled select: the bins of the first digit whose keys the full sweep keeps as
// candidates (predicted from a sample of the rows), and what the full histogram then says.
struct SelectPlan {
    uint32_t lo, span;   // candidate bins lo .. lo + span (lo = kBins0: none)
    uint32_t bin0;       // the bin that holds the median, from the full histogram
    uint32_t before0;    // keys in the bins below it
    uint32_t need;       // 1: the prediction missed the bin or the list overflowed; a sweep of its own collects the bin
    uint32_t pad[3];
};

// Shape and addressing of one tensor, passed by value to every kernel.
struct Geometry {
    int32_t B, H, T;
    int32_t D;            // elements per row (head dimension), 1..128
    int32_t n_c;          // ceil(D / 4): chunks per row; a last partial chunk is zero-padded
    uint32_t n_c_magic;   // 2^32 / n_c + 1 (n_c >= 2): __umulhi(q, n_c_magic) == q / n_c for every q < 2^27
    int32_t row_words;    // ceil(n_c * w / 32): 32-bit words of one packed row (w when D = 128)
    int32_t vec_ok;       // D and the strides are multiples of 4: every chunk is one aligned 8-byte access
    int32_t S;            // secondaries per head
    int32_t S16;          // ceil(S / 16): groups of 16 secondaries (4 MFMA s-blocks) of the search loop
    int32_t A16;          // groups held as matrix operands and screened on the matrix cores: S16, or 0 for S > kScreenMaxS
                          // (every chunk then scores all S secondaries in fp32 on the vector ALUs: exact, slow)
    int32_t b_r, w_idx, w;
    int64_t sb, sh, st;   // element strides
    float inv_L;          // 1 / (2^b_r - 1)
    int32_t log2_S;       // log2(S) when S is a power of two, else -1
    float inv_S;          // (1/S)(1 + 2^-18): uint(float(k) * inv_S) == k / S for every k < 2^16, S <= 2730
    int32_t check_finite;  // HQMQ_FLAG_CHECK_FINITE: the search reports chunks holding an infinity or a NaN in the status word
    int32_t cand_cap;     // candidate keys kept per head: kCandCap, or 1/32 of the head's chunks if that is more
    int32_t select_sampled;  // the median select predicts the median's bin from a sample of the rows (large heads only)
    int32_t fused_by_head;  // fused search only: one workgroup per head takes the rows of all batch entries (B T <= 64)
    int32_t search_rows;               // rows per search workgroup (kSearchRowsSmall or kSearchRowsLarge)
    uint32_t n_search_blocks_per_seg;  // ceil(T / search_rows)
};

// Dynamic LDS of one search workgroup (host side; the kernels carve the same layout): the head's
// MFMA A operands and secondaries, and the per-row state, which for rows of
// 128 elements is two rows of code words per wave and a counter per row, and for other row lengths a
// running maximum, flag word, scale, counter and the code words of every row of the workgroup.
inline size_t search_lds_bytes(int S16, int A16, int D, int row_words, int waves, int rows)
{
    const size_t tables = (size_t)A16 * kATiles * 64 * 16 + (size_t)S16 * 16 * 4 * 4;
    if (D == 4 * kChunksPerRow)
        return tables + ((size_t)waves * 2 * 32 + (size_t)rows) * 4;
    return tables + (size_t)rows * (8 + 4 + 4 + 4 + 4 * (size_t)row_words);
}
constexpr size_t kLdsPerCu = 160 * 1024;

// Waves of a search workgroup.  256 or more rows per workgroup, and tables so large
// that fewer than four 4-wave workgroups fit a CU's LDS: one workgroup of 16 waves per CU when its LDS
// fits (four waves on every SIMD sharing one copy of the tables; measured 3 % faster than two
// workgroups of 4, while four or more small workgroups, where they fit, are 7 to 13 % faster than the large one).
// Otherwise 4 waves when two workgroups fit a CU's LDS, else one workgroup of 8, which keeps two waves
// on every SIMD.
inline int search_waves_for(int S16, int A16, int D, int row_words, int rows)
{
    if (A16 == 0)
        return 4;  // the unscreened search has one shape
    if (rows >= kSearchRowsLarge && kLdsPerCu / search_lds_bytes(S16, A16, D, row_words, 4, rows) < 4 &&
        search_lds_bytes(S16, A16, D, row_words, 16, rows) <= kLdsPerCu)
        return 16;
    return 2 * search_lds_bytes(S16, A16, D, row_words, 4, rows) > kLdsPerCu ? 8 : 4;
}

// Rows per search workgroup.  Four or more 4-wave workgroups per CU are the fastest shape (measured 3 to
// 7 % ahead of one 16-wave workgroup): the most rows with which they fit, 256 for long segments (the head's
// operand table is copied less often) or 64.  With tables too large for that: one 16-wave workgroup of 512
// or 256 rows per CU, else 64 rows.
inline int search_rows_for(int T, int S16, int A16, int D, int row_words)
{
    if (A16 == 0)
        return kSearchRowsSmall;  // the unscreened search has one shape
    const auto four_fit = [&](int rows) { return kLdsPerCu / search_lds_bytes(S16, A16, D, row_words, 4, rows) >= 4; };
    if (T >= kSearchRowsSwitch && four_fit(kSearchRowsLarge))
        return kSearchRowsLarge;
    if (four_fit(kSearchRowsSmall))
        return kSearchRowsSmall;
    if (T >= kSearchRowsSwitchHuge && search_waves_for(S16, A16, D, row_words, kSearchRowsHuge) == 16)
        return kSearchRowsHuge;
    if (T >= kSearchRowsSwitch &&
        (D == 4 * kChunksPerRow || 2 * search_lds_bytes(S16, A16, D, row_words, 4, kSearchRowsLarge) <= kLdsPerCu))
        return kSearchRowsLarge;
    return kSearchRowsSmall;
}

// Workspace carve-up (device pointers into the caller's workspace).
struct Workspace {
    SelectState *state;            // [H]
    double *thr;                   // [H] outlier threshold on squared norms
    uint32_t *hist0;               // [H][kBins0]
    uint32_t *hist1;               // [H][kBins1]
    uint32_t *hist_s;              // [H][kBins0] first digit of the sampled rows; shares the candidate list's memory (read
                                   // before the first candidate is written)
    SelectPlan *plan;              // [H]
    uint32_t *cand_count;          // [3][H] keys sent to the candidate list (any may exceed cand_cap): by the sweep that
                                   // collects one bin (or, in the sampled select, the predicted bins), by the sweep after
                                   // an overflow, by the sampled select's fallback sweep of one bin
    unsigned long long *cand;      // [H][cand_cap]
    uint32_t *block_sum;           // [B*H*n_search_blocks_per_seg] outliers per search workgroup
    uint32_t *block_pre;           // same shape, exclusive prefix
    uint4 *aop;                    // [H][kATiles * S16][64] MFMA A operands of the search, built once per call
};

struct EncodedPtrs {
    uint32_t *codes;
    uint16_t *sigma;
    uint32_t *flags;
    uint32_t *row_off;
    uint16_t *outliers;
    uint32_t *n_outliers;
    uint32_t *status;
};

// Byte offsets of the workspace parts inside one tensor's slice (same for every tensor of a shape).
struct WorkspaceOffsets {
    uint32_t state, thr, hist0, hist1, plan, cand_count, cand, block_sum, block_pre, aop;
};

// One tensor of an encode batch and the batch itself (passed by value as kernel arguments; every
// encode kernel takes blockIdx.z as the tensor index).
struct EncodeTensor {
    const _Float16 *x;
    const float *sec;
    EncodedPtrs enc;
    char *ws;                  // this tensor's slice of the workspace
    uint64_t outlier_capacity;
    const double *thr_given;   // caller's thresholds on squared norms [H], or null: take the median's
};
constexpr int kMaxEncodeBatch = 32;  // 32 * 96 B of descriptors stay inside the 4 KiB of kernel arguments
struct EncodeBatch {
    EncodeTensor t[kMaxEncodeBatch];
};

__device__ __forceinline__ Workspace carve_workspace(char *base, const WorkspaceOffsets &o)
{
    Workspace ws;
    ws.state = reinterpret_cast<SelectState *>(base + o.state);
    ws.thr = reinterpret_cast<double *>(base + o.thr);
    ws.hist0 = reinterpret_cast<uint32_t *>(base + o.hist0);
    ws.hist1 = reinterpret_cast<uint32_t *>(base + o.hist1);
    ws.hist_s = reinterpret_cast<uint32_t *>(base + o.cand);
    ws.plan = reinterpret_cast<SelectPlan *>(base + o.plan);
    ws.cand_count = reinterpret_cast<uint32_t *>(base + o.cand_count);
    ws.cand = reinterpret_cast<unsigned long long *>(base + o.cand);
    ws.block_sum = reinterpret_cast<uint32_t *>(base + o.block_sum);
    ws.block_pre = reinterpret_cast<uint32_t *>(base + o.block_pre);
    ws.aop = reinterpret_cast<uint4 *>(base + o.aop);
    return ws;
}

// One tensor of a decode batch and the batch itself (passed by value as kernel arguments).
struct DecodeTensor {
    uint32_t *codes;
    uint16_t *sigma;
    uint32_t *flags;
    uint32_t *row_off;
    uint16_t *outliers;
    const float *sec;
    _Float16 *out;
    uint64_t outlier_capacity;
};
constexpr int kMaxDecodeBatch = 32;  // 32 * 64 B of descriptors stay well inside the 4 KiB of kernel arguments
struct DecodeBatch {
    DecodeTensor t[kMaxDecodeBatch];
};

// Single-query attention over a packed K and a packed V cache (one query token per sequence).
constexpr int kMaxGroup = 16;        // query heads sharing one kv head (columns of one matrix-core product)
constexpr int kAttendTile = 64;      // rows per workgroup iteration (4 waves x 16 rows)
struct AttendSide {
    const uint32_t *codes;
    const uint16_t *sigma;
    const uint32_t *flags;
    const uint32_t *row_off;
    const uint16_t *outliers;
    const float *sec;
    uint64_t outlier_capacity;
};
struct AttendArgs {
    AttendSide k, v;
    const _Float16 *q;     // [B][H * G][D]
    _Float16 *out;         // [B][H * G][D]
    float *lse;            // [B][H * G] natural-log sum of exp(score) over the cached tokens, or null
    const int32_t *visible;  // [B][H * G] number of leading cached tokens each query head may see, or null (all)
    float *part_ml;        // [B * H * G][n_splits][2]: running maximum (log2 domain) and weight sum
    float *part_acc;       // [B * H * G][n_splits][128]: weighted value sum
    float qscale;          // softmax scale * log2(e), folded into the query
    int32_t G;             // query heads per kv head
    int32_t D;             // head dimension: 64, 96 or 128 (q and out rows; the partial sums keep a pitch of 128)
    int32_t n_splits;      // workgroups along the sequence
    int32_t rows_per_split;  // multiple of kAttendTile (of the table form's tile of 128 rows when joint)
    int32_t joint;           // the form that reads the reconstruction from half tables in LDS
};
// Split of the sequence over workgroups: enough of them to fill the chip, at least one tile each.
struct AttendPlan {
    int32_t n_splits, rows_per_split;
    int32_t joint;
    uint64_t ml_bytes, acc_bytes, total_bytes;
};
// tables_always: take the table form whenever its tables fit, whatever the size of the cache.
AttendPlan plan_attend(const Geometry &g, int G, bool tables_always);

// ---- device helpers --------------------------------------------------------------------

typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef float float4_t __attribute__((ext_vector_type(4)));

// Squared norm of a chunk in fp64, fixed order ((x0^2 + x1^2) + x2^2) + x3^2.  The products
// of fp16 values are exact in fp64, so only the three additions round.
__device__ __forceinline__ double chunk_norm2(const half4_t v)
{
    double x0 = (double)(float)v[0], x1 = (double)(float)v[1];
    double x2 = (double)(float)v[2], x3 = (double)(float)v[3];
    return ((x0 * x0 + x1 * x1) + x2 * x2) + x3 * x3;
}

// True when one of the chunk's four fp16 values is an infinity or a NaN (exponent field all ones).  Taken
// on the bit patterns: the build tells the compiler that no arithmetic sees a NaN, so a test on a computed
// value could be folded away.  Adding 0x0400 to a masked exponent field carries into bit 15 exactly when the
// field is 0x7c00.
__device__ __forceinline__ bool chunk_nonfinite(const half4_t v)
{
    const uint2 raw = __builtin_bit_cast(uint2, v);
    const uint32_t a = ((raw.x & 0x7c007c00u) + 0x04000400u) | ((raw.y & 0x7c007c00u) + 0x04000400u);
    return (a & 0x80008000u) != 0u;
}

__device__ __forceinline__ half4_t load_chunk(const _Float16 *p)
{
    uint2 raw = *reinterpret_cast<const uint2 *>(p);
    return __builtin_bit_cast(half4_t, raw);
}

// Chunk c of the row starting at `row`, for any head dimension.  kFull (D = 128, strides that keep
// every chunk 8-byte aligned) is the plain vector load.  Otherwise lanes past the row's chunks, and
// the elements past D inside the last chunk, read as +0: the zero padding of a head whose dimension
// is not a multiple of 4 (paper App. "Padding wrapper for d_h not divisible by 4").
template <bool kFull>
__device__ __forceinline__ half4_t load_row_chunk(const _Float16 *row, int c, const Geometry &g)
{
    if (kFull)
        return load_chunk(row + 4 * c);
    half4_t v = {0, 0, 0, 0};
    if (c < g.n_c) {
        if (g.vec_ok) {
            v = load_chunk(row + 4 * c);
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (4 * c + e < g.D)
                    v[e] = row[4 * c + e];
        }
    }
    return v;
}

// q / n_c for a flat chunk index q < 2^27 (one chunk per row: the multiplier would not fit 32 bits).
__device__ __forceinline__ int row_of_chunk(int q, const Geometry &g)
{
    return g.n_c == 1 ? q : (int)__umulhi((uint32_t)q, g.n_c_magic);
}

__device__ __forceinline__ unsigned long long key_of(double r2)
{
    return (unsigned long long)__double_as_longlong(r2);
}

// Launchers implemented in the kernel translation units (host side).
hipError_t launch_select_median(const Geometry &g, const WorkspaceOffsets &wo, const EncodeBatch &batch, int n_tensors,
                                float C, bool skip_select, hipStream_t stream);
hipError_t launch_shard_median_pass(const Geometry &g, const WorkspaceOffsets &wo, const EncodeBatch &batch, int pass,
                                    unsigned long long total_per_head, float C, hipStream_t stream);
hipError_t prepare_search_kernels();  // once per device, before the first launch_search on it
hipError_t launch_search(const Geometry &g, const WorkspaceOffsets &wo, const EncodeBatch &batch, int n_tensors,
                         hipStream_t stream);
bool search_fused_available(const Geometry &g);  // launch_search_fused has a kernel for this shape
hipError_t launch_search_fused(const Geometry &g, const WorkspaceOffsets &wo, const EncodeBatch &batch, int n_tensors,
                               hipStream_t stream);
hipError_t launch_outlier_list_small(const Geometry &g, const WorkspaceOffsets &wo, const EncodeBatch &batch,
                                     int n_tensors, hipStream_t stream);
hipError_t launch_outlier_list(const Geometry &g, const WorkspaceOffsets &wo, const EncodeBatch &batch, int n_tensors,
                               hipStream_t stream);
hipError_t launch_decode(const Geometry &g, const DecodeBatch &batch, int n_tensors, hipStream_t stream);
hipError_t prepare_attend_kernels();  // once per device, before the first launch_attend on it
hipError_t launch_attend(const Geometry &g, const AttendArgs &args, hipStream_t stream);

}  // namespace hqmq
