// Med3x outlier extraction, first half: the exact per-head median of the squared chunk norms
// (paper Sec. 3 "Median-multiplier outlier extraction", Alg. 1 "Outlier extraction").
//
// The median is the lower median (element (n-1)/2 of the sorted norms) of all B*T*ceil(D/4) chunks
// of a head.  Non-negative IEEE doubles order like their bit patterns read as unsigned integers,
// so the median is found by a most-significant-digit radix select on the 63 value bits of r^2:
//   sweep 0  histogram of a first digit made of the exponent and 6 mantissa bits (the squares of fp16
//            data span 83 binades, which at 64 bins each fit the 8192 bins of a workgroup's LDS)
//   sweep 1  the keys in the bin that holds the wanted rank (about one in 200 for smooth data) go to a
//            candidate list, and are counted by their next 10 bits
//   sweep 2  only for a head whose list overflowed: collects the keys that share both digits; returns
//            at once otherwise
//   finish   one workgroup per head selects the wanted rank among the candidates (radix select on
//            their low 46 or 36 bits) and writes the outlier threshold C^2 * median.
// Nothing is sorted and no float arithmetic is involved after r^2 itself, so the result is the
// exact order statistic.  Each sweep recomputes r^2 in registers from the fp16 tensor (8 B per
// chunk, HBM-bound); the bin choice of the previous sweep is re-derived by every workgroup
// from the (L2-resident) histogram instead of costing a kernel launch of its own.
// A head of at least kSampleMinChunks chunks skips sweep 1 (the sampled select): a histogram of every
// kSampleStride-th row predicts a few bins around the median's, sweep 0 keeps the keys of those bins as
// candidates while it counts all keys, and only a head whose prediction missed the bin that the full
// histogram names (or whose list overflowed) goes through sweep 1 after all.  The prediction decides which
// keys are kept, never the result.
// If a head has more keys sharing both digits than the list holds (many equal norms: a
// constant or coarsely quantised tensor), the finishing workgroup falls back to radix-selecting
// the low bits over the head's raw rows itself: slow, exact, and only for such inputs.
#include "hqmq_device.h"

namespace hqmq {

namespace {

constexpr unsigned long long kKeyMask = 0x7fffffffffffffffull;

// Exclusive scan position of `rank` in a histogram: returns the bin holding the rank-th key
// (0-based) and how many keys lie in earlier bins.  Called by every thread of the block with the
// same arguments; `hist` may be global memory.  kBins is a multiple of the block size.
template <int kBins, int kBlock>
__device__ __forceinline__ void pick_bin(const uint32_t *hist, uint32_t rank, uint32_t *scratch /* LDS, kBlock + 2 */,
                                         uint32_t &bin_out, uint32_t &before_out)
{
    constexpr int kPer = kBins / kBlock;
    static_assert(kBins % kBlock == 0 && kBlock % 64 == 0, "bins must tile the block");
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    uint32_t local[kPer];
    uint32_t sum = 0;
#pragma unroll
    for (int i = 0; i < kPer; ++i) {
        local[i] = hist[tid * kPer + i];
        sum += local[i];
    }
    // inclusive scan over the block: shuffle scan inside each wave, then wave totals through LDS
    uint32_t inc = sum;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        uint32_t o = __shfl_up(inc, d, 64);
        if (lane >= d)
            inc += o;
    }
    if (lane == 63)
        scratch[wv] = inc;
    __syncthreads();
    uint32_t wave_before = 0;
    for (int k = 0; k < kBlock / 64; ++k)
        if (k < wv)
            wave_before += scratch[k];
    uint32_t before = wave_before + inc - sum;
    if (rank >= before && rank < before + sum) {
        bool found = false;
#pragma unroll
        for (int i = 0; i < kPer; ++i) {
            if (!found && rank < before + local[i]) {
                scratch[kBlock] = tid * kPer + i;
                scratch[kBlock + 1] = before;
                found = true;
            }
            if (!found)
                before += local[i];
        }
    }
    __syncthreads();
    bin_out = scratch[kBlock];
    before_out = scratch[kBlock + 1];
    __syncthreads();
}

}  // namespace

// First digit of the two-sweep select: exponent and 6 mantissa bits of r^2, offset so that the squares
// that fp16 data can produce (0, and 2^-48 up to below 2^35) fill bins 0 and 1..5312.  Monotone; bins
// 1..kBins0-2 each hold exactly the keys of one 17-bit prefix bin + kFineBase; bin 0 holds the keys
// below 2^-48 (for fp16 data: zero only), the last bin everything from 2^(kBins0-2)/64 binades up
// (never reached by finite fp16 data).
__device__ __forceinline__ uint32_t fine_bin(unsigned long long key)
{
    const uint32_t p = (uint32_t)(key >> kFineShift);
    const uint32_t d = p > kFineBase ? p - kFineBase : 0u;
    return min(d, (uint32_t)kBins0 - 1u);
}
__device__ __forceinline__ bool fine_bin_is_prefix(uint32_t bin) { return bin >= 1u && bin <= (uint32_t)kBins0 - 2u; }

// ---------------------------------------------------------------------------------------
// reset of the per-call scratch state
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void k_init(Geometry g, WorkspaceOffsets wo, EncodeBatch batch)
{
    const EncodeTensor &tn = batch.t[blockIdx.z];
    const Workspace ws = carve_workspace(tn.ws, wo);
    const EncodedPtrs enc = tn.enc;
    const uint32_t i = blockIdx.x * kThreads + threadIdx.x;
    if (i < (uint32_t)g.H * kBins0) {
        ws.hist0[i] = 0;
        ws.hist_s[i] = 0;
    }
    if (i < (uint32_t)g.H * kBins1)
        ws.hist1[i] = 0;
    if (i < 3u * (uint32_t)g.H)
        ws.cand_count[i] = 0;
    if (i < (uint32_t)g.H) {
        // +inf: nothing is flagged (replaced by the select, unless the caller supplies the thresholds)
        ws.thr[i] = tn.thr_given ? tn.thr_given[i] : __longlong_as_double(0x7ff0000000000000LL);
    }
    if (i <= (uint32_t)g.H)
        enc.n_outliers[i] = 0;
    if (i == 0)
        enc.status[0] = 0;
}

// ---------------------------------------------------------------------------------------
// sweeps.  grid = (ceil(T / kSelectRows), B*H), 1024 threads: one lane per chunk, 32 rows per
// block iteration, four independent 8-byte loads in flight per lane.
//   MODE 0: histogram of the first digit (fine_bin), all keys; in the sampled select it also keeps the keys of
//           the predicted bins as candidates (staged like MODE 1's)
//   MODE 3: histogram of the first digit over every kSampleStride-th row (sampled select only)
//   MODE 1: picks the first digit (sampled select: returns at once unless the head needs it); the keys of that bin (about one in 200) go to the head's candidate
//           list, staged in LDS so that a workgroup costs the list's counter one update, and are
//           counted by their next 10 bits (45..36) in case the list overflows
//   MODE 2: returns at once unless the head's list overflowed; then picks both digits and collects the
//           keys that share them (the list's memory is reused, with a counter of its own)
// ---------------------------------------------------------------------------------------
// kFull: D = 128 (every lane of a 32-lane row slot holds a chunk); otherwise lanes past the row's
// chunks are idle and the loads go through the general path.
constexpr int kStageKeys = 1024;  // candidate keys a workgroup stages in LDS
constexpr int kFallbackSpan = 8;  // sampled select: a workgroup of MODE 1 or 2 covers this many times kSelectRows rows
// The counter of the list that holds the keys of the median's bin alone: MODE 1's.
__device__ __forceinline__ uint32_t *bin_list_counter(const Geometry &g, const Workspace &ws, int h)
{
    return ws.cand_count + (g.select_sampled ? 2 * g.H + h : h);
}
template <int MODE, bool kFull, bool kCollect = false>
__global__ __launch_bounds__(kSelectThreads) void k_select_sweep(Geometry g, WorkspaceOffsets wo, EncodeBatch batch)
{
    const EncodeTensor &tn = batch.t[blockIdx.z];
    const Workspace ws = carve_workspace(tn.ws, wo);
    const _Float16 *__restrict__ x = tn.x;
    constexpr bool kHist0 = MODE == 0 || MODE == 3;
    constexpr bool kStages = MODE == 1 || (MODE == 0 && kCollect);
    constexpr int kLdsBins = kHist0 ? kBins0 : kBins1;
    __shared__ uint32_t lh[MODE == 2 ? 1 : kLdsBins];
    __shared__ uint32_t scratch[kSelectThreads + 2];
    __shared__ unsigned long long staged[kStages ? kStageKeys : 1];
    __shared__ uint32_t n_staged, list_base;

    const int seg = blockIdx.y, b = seg / g.H, h = seg % g.H;
    const uint32_t rank0 = (uint32_t)(((uint64_t)g.B * g.T * g.n_c - 1) / 2);
    uint32_t bin0 = 0, before0 = 0, bin1 = 0, before1 = 0;
    uint32_t keep_lo = 0, keep_span = 0;
    if (MODE == 0 && kCollect) {
        keep_lo = ws.plan[h].lo;
        keep_span = ws.plan[h].span;
    }
    if ((MODE == 1 || MODE == 2) && g.select_sampled && !ws.plan[h].need)
        return;  // the candidates kept by MODE 0 hold the median's bin (uniform over the workgroup)
    uint32_t *const bin_count = bin_list_counter(g, ws, h);
    if (MODE == 2 && *bin_count <= (uint32_t)g.cand_cap)
        return;  // the list of MODE 1 holds every candidate (uniform over the workgroup)
    if (MODE == 1 || MODE == 2) {
        pick_bin<kBins0, kSelectThreads>(ws.hist0 + (size_t)h * kBins0, rank0, scratch, bin0, before0);
        if (!fine_bin_is_prefix(bin0))
            return;  // the finishing kernel knows the median of such a bin without candidates
    }
    if (MODE == 2)
        pick_bin<kBins1, kSelectThreads>(ws.hist1 + (size_t)h * kBins1, rank0 - before0, scratch, bin1, before1);
    if (MODE != 2) {
        for (int i = threadIdx.x; i < kLdsBins; i += kSelectThreads)
            lh[i] = 0;
        if (threadIdx.x == 0)
            n_staged = 0;
        __syncthreads();
    }

    const int c = threadIdx.x & 31, sub = threadIdx.x >> 5;  // 32 rows per iteration
    // MODE 3 walks the sampled rows: row j of its grid is token kSampleStride * j
    constexpr int kStep = MODE == 3 ? kSampleStride : 1;
    const int n_t = MODE == 3 ? (g.T + kSampleStride - 1) / kSampleStride : g.T;
    // the sweeps that a sampled select seldom needs are launched with fewer, longer workgroups
    const int rows = ((MODE == 1 || MODE == 2) && g.select_sampled) ? kSelectRows * kFallbackSpan : kSelectRows;
    const int t0 = blockIdx.x * rows;
    const int t1 = min(n_t, t0 + rows);
    const _Float16 *base = x + (int64_t)b * g.sb + (int64_t)h * g.sh;
    const int64_t row_stride = (int64_t)kStep * g.st;
    const bool active = kFull || c < g.n_c;
    unsigned long long *cand = ws.cand + (size_t)h * g.cand_cap;

    for (int tb = t0; tb < t1; tb += 128) {  // uniform over the block
        half4_t v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int tt = tb + sub + 32 * u;
            v[u] = (tt < t1) ? load_row_chunk<kFull>(base + (int64_t)tt * row_stride, c, g) : half4_t{0, 0, 0, 0};
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const bool in = active && (tb + sub + 32 * u) < t1;
            const unsigned long long key = key_of(chunk_norm2(v[u])) & kKeyMask;
            if (kHist0) {
                if (in) {
                    const uint32_t bin = fine_bin(key);
                    atomicAdd(&lh[bin], 1u);
                    if (kCollect && bin - keep_lo <= keep_span) {
                        const uint32_t pos = atomicAdd(&n_staged, 1u);
                        if (pos < (uint32_t)kStageKeys) {
                            staged[pos] = key;
                        } else {
                            const uint32_t gpos = atomicAdd(&ws.cand_count[h], 1u);
                            if (gpos < (uint32_t)g.cand_cap)
                                cand[gpos] = key;
                        }
                    }
                }
            } else if (MODE == 1) {
                if (in && fine_bin(key) == bin0) {
                    atomicAdd(&lh[(uint32_t)(key >> kSecShift) & (kBins1 - 1)], 1u);
                    const uint32_t pos = atomicAdd(&n_staged, 1u);
                    if (pos < (uint32_t)kStageKeys) {
                        staged[pos] = key;
                    } else {  // more than the stage holds (many equal norms): straight to the list
                        const uint32_t gpos = atomicAdd(bin_count, 1u);
                        if (gpos < (uint32_t)g.cand_cap)
                            cand[gpos] = key;
                    }
                }
            } else {
                // one counter update per wave: ballot, leader adds, lanes take consecutive slots
                const bool hit = in && fine_bin(key) == bin0 && ((uint32_t)(key >> kSecShift) & (kBins1 - 1)) == bin1;
                const unsigned long long m = __ballot(hit);
                if (m) {
                    uint32_t basepos = 0;
                    const int leader = __ffsll((long long)m) - 1;
                    if ((int)(threadIdx.x & 63) == leader)
                        basepos = atomicAdd(&ws.cand_count[g.H + h], (uint32_t)__popcll(m));
                    basepos = __shfl(basepos, leader, 64);
                    if (hit) {
                        const uint32_t pos = basepos + __popcll(m & ((1ull << (threadIdx.x & 63)) - 1ull));
                        if (pos < (uint32_t)g.cand_cap)
                            cand[pos] = key;
                    }
                }
            }
        }
    }
    if (MODE != 2) {
        __syncthreads();
        uint32_t *gh = MODE == 0   ? ws.hist0 + (size_t)h * kBins0
                       : MODE == 3 ? ws.hist_s + (size_t)h * kBins0
                                   : ws.hist1 + (size_t)h * kBins1;
        for (int i = threadIdx.x; i < kLdsBins; i += kSelectThreads) {
            const uint32_t n = lh[i];
            if (n)
                atomicAdd(&gh[i], n);
        }
    }
    if (kStages) {
        const uint32_t n = min(n_staged, (uint32_t)kStageKeys);
        uint32_t *const counter = MODE == 1 ? bin_count : ws.cand_count + h;
        if (threadIdx.x == 0)
            list_base = n ? atomicAdd(counter, n) : 0u;
        __syncthreads();
        const uint32_t at = list_base;
        for (uint32_t i = threadIdx.x; i < n; i += kSelectThreads)
            if (at + i < (uint32_t)g.cand_cap)
                cand[at + i] = staged[i];
    }
}

// ---------------------------------------------------------------------------------------
// The two small steps of the sampled select, one workgroup per head.
//   k_select_range   after MODE 3: the bins of the first digit that hold the sample's ranks within four
//                    standard deviations of its median rank (a binomial count: sqrt(n)/2 ranks each): for
//                    rows drawn from one distribution the full data's median falls outside them about once
//                    in 16000 heads
//   k_select_decide  after MODE 0: the median's bin from the full histogram, and whether the kept keys
//                    cover it (inside the predicted bins, list not overflowed)
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(kSelectThreads) void k_select_range(Geometry g, WorkspaceOffsets wo, EncodeBatch batch)
{
    const EncodeTensor &tn = batch.t[blockIdx.z];
    const Workspace ws = carve_workspace(tn.ws, wo);
    __shared__ uint32_t scratch[kSelectThreads + 2];
    const int h = blockIdx.x;
    const uint32_t n_s = (uint32_t)((uint64_t)g.B * ((g.T + kSampleStride - 1) / kSampleStride) * g.n_c);
    const uint32_t mid = (n_s - 1) / 2;
    const uint32_t margin = (uint32_t)(2.0f * sqrtf((float)n_s)) + 2u;
    uint32_t lo, hi, before;
    pick_bin<kBins0, kSelectThreads>(ws.hist_s + (size_t)h * kBins0, mid > margin ? mid - margin : 0u, scratch, lo, before);
    pick_bin<kBins0, kSelectThreads>(ws.hist_s + (size_t)h * kBins0, min(n_s - 1, mid + margin), scratch, hi, before);
    lo = max(lo, 1u);                      // only bins that are one 17-bit prefix each hold candidates
    hi = min(hi, (uint32_t)kBins0 - 2u);
    if (threadIdx.x == 0) {
        ws.plan[h].lo = lo <= hi ? lo : (uint32_t)kBins0;
        ws.plan[h].span = lo <= hi ? hi - lo : 0u;
    }
}

__global__ __launch_bounds__(kSelectThreads) void k_select_decide(Geometry g, WorkspaceOffsets wo, EncodeBatch batch)
{
    const EncodeTensor &tn = batch.t[blockIdx.z];
    const Workspace ws = carve_workspace(tn.ws, wo);
    __shared__ uint32_t scratch[kSelectThreads + 2];
    const int h = blockIdx.x;
    const uint32_t rank0 = (uint32_t)(((uint64_t)g.B * g.T * g.n_c - 1) / 2);
    uint32_t bin0, before0;
    pick_bin<kBins0, kSelectThreads>(ws.hist0 + (size_t)h * kBins0, rank0, scratch, bin0, before0);
    if (threadIdx.x == 0) {
        const bool covered = bin0 - ws.plan[h].lo <= ws.plan[h].span && ws.cand_count[h] <= (uint32_t)g.cand_cap;
        ws.plan[h].bin0 = bin0;
        ws.plan[h].before0 = before0;
        ws.plan[h].need = fine_bin_is_prefix(bin0) && !covered ? 1u : 0u;
    }
}

// ---------------------------------------------------------------------------------------
// finish: one workgroup per head.  Locates the first digit again; a head whose candidate list is
// complete has its median among the list's keys (they share the digit's 17-bit prefix): radix select on
// their low 46 bits.  After an overflow the second digit is located too and the select runs on the low
// 36 bits of the keys MODE 2 collected, or, if even those were too many (many equal norms: a constant or
// coarsely quantised tensor), over the head's raw rows: slow, exact, and only for such inputs.
// Writes thr[h] = fl(fl(C*C) * median).
// ---------------------------------------------------------------------------------------
template <bool kFull>
__global__ __launch_bounds__(kSelectThreads) void k_select_finish(Geometry g, WorkspaceOffsets wo, EncodeBatch batch,
                                                                  float C)
{
    const EncodeTensor &tn = batch.t[blockIdx.z];
    const Workspace ws = carve_workspace(tn.ws, wo);
    const _Float16 *__restrict__ x = tn.x;
    __shared__ uint32_t lh[kBins1];
    __shared__ uint32_t scratch[kSelectThreads + 2];
    const int h = blockIdx.x;
    uint32_t rank = (uint32_t)(((uint64_t)g.B * g.T * g.n_c - 1) / 2);
    uint32_t bin0, before0;
    pick_bin<kBins0, kSelectThreads>(ws.hist0 + (size_t)h * kBins0, rank, scratch, bin0, before0);
    rank -= before0;

    unsigned long long median_bits;
    if (bin0 == 0u) {
        median_bits = 0ull;  // fp16 data: the bin holds zeros only
    } else if (!fine_bin_is_prefix(bin0)) {
        median_bits = 0x7ff0000000000000ull;  // not reached by finite fp16 data: nothing is flagged
    } else {
        unsigned long long prefix = (unsigned long long)(bin0 + kFineBase);  // key bits fixed so far, right aligned
        int low_bits = kFineShift;
        // sampled select whose kept keys cover the bin: the list also holds keys of the neighbouring bins,
        // which the comparisons against the prefix below pass over
        const bool kept = g.select_sampled && !ws.plan[h].need;
        uint32_t n_cand = kept ? ws.cand_count[h] : *bin_list_counter(g, ws, h);
        if (n_cand > (uint32_t)g.cand_cap) {
            uint32_t bin1, before1;
            pick_bin<kBins1, kSelectThreads>(ws.hist1 + (size_t)h * kBins1, rank, scratch, bin1, before1);
            rank -= before1;
            prefix = (prefix << kBits1) | bin1;
            low_bits = kSecShift;
            n_cand = ws.cand_count[g.H + h];
        }
        const bool from_list = n_cand <= (uint32_t)g.cand_cap;
        const unsigned long long *cand = ws.cand + (size_t)h * g.cand_cap;

        unsigned long long low = 0;  // low-part digits fixed so far, right aligned
        int remaining = low_bits;    // low-part bits still open
        while (remaining > 0) {
            const int d = remaining < 10 ? remaining : 10;
            const int shift = remaining - d;
            const uint32_t dmask = (1u << d) - 1u;
            for (int i = threadIdx.x; i < kBins1; i += kSelectThreads)
                lh[i] = 0;
            __syncthreads();
            const unsigned long long want = (prefix << (low_bits - remaining)) | low;  // compare key >> remaining
            if (from_list) {
                // four keys requested before the first is used; a slot past the list reads as a key with
                // bit 63 set, which no prefix matches
                for (uint32_t i0 = 0; i0 < n_cand; i0 += 4 * kSelectThreads) {
                    unsigned long long key[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const uint32_t i = i0 + u * kSelectThreads + threadIdx.x;
                        key[u] = i < n_cand ? cand[i] : ~0ull;
                    }
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        if ((key[u] >> remaining) == want)
                            atomicAdd(&lh[(uint32_t)(key[u] >> shift) & dmask], 1u);
                }
            } else {
                // rare path: sweep the head's rows (every batch entry), one lane per chunk
                const int c = threadIdx.x & 31, sub = threadIdx.x >> 5;
                for (int b = 0; b < g.B; ++b) {
                    const _Float16 *base = x + (int64_t)b * g.sb + (int64_t)h * g.sh;
                    for (int t = sub; t < g.T; t += kSelectThreads / 32) {
                        const unsigned long long key =
                            key_of(chunk_norm2(load_row_chunk<kFull>(base + (int64_t)t * g.st, c, g))) & kKeyMask;
                        if ((kFull || c < g.n_c) && (key >> remaining) == want)
                            atomicAdd(&lh[(uint32_t)(key >> shift) & dmask], 1u);
                    }
                }
            }
            __syncthreads();
            uint32_t bin, before;
            pick_bin<kBins1, kSelectThreads>(lh, rank, scratch, bin, before);
            rank -= before;
            low = (low << d) | bin;
            remaining -= d;
        }
        median_bits = (prefix << low_bits) | low;
    }
    if (threadIdx.x == 0) {
        // threshold on squares: fl(fl(C*C) * median), C widened from fp32
        const double c = (double)C;
        const double c2 = c * c;
        ws.thr[h] = c2 * __longlong_as_double((long long)median_bits);
    }
}

// ---------------------------------------------------------------------------------------
// outlier bookkeeping after the search kernel has written the flag words, the per-row offsets
// local to its 64-row workgroup and the workgroup totals:
//   k_scan    exclusive scan of the workgroup totals (linear row order), per-head totals, status
//   k_gather  adds the workgroup prefix to every row offset and copies the flagged chunks into
//             the outlier list in ascending linear chunk order
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void k_scan(Geometry g, WorkspaceOffsets wo, EncodeBatch batch,
                                               uint32_t n_blocks, uint64_t n_rows)
{
    const EncodeTensor &tn = batch.t[blockIdx.z];
    const Workspace ws = carve_workspace(tn.ws, wo);
    const EncodedPtrs enc = tn.enc;
    const uint64_t outlier_capacity = tn.outlier_capacity;
    __shared__ uint32_t wave_tot[16];
    __shared__ uint32_t carry_s;
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const uint32_t blocks_per_seg = g.n_search_blocks_per_seg;
    if (threadIdx.x == 0)
        carry_s = 0;
    __syncthreads();
    for (uint32_t start = 0; start < n_blocks; start += 1024) {
        const uint32_t i = start + threadIdx.x;
        const uint32_t v = (i < n_blocks) ? ws.block_sum[i] : 0;
        uint32_t inc = v;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            uint32_t o = __shfl_up(inc, d, 64);
            if (lane >= d)
                inc += o;
        }
        if (lane == 63)
            wave_tot[wv] = inc;
        __syncthreads();
        uint32_t wave_before = 0, all = 0;
        for (int k = 0; k < 16; ++k) {
            const uint32_t wt = wave_tot[k];
            if (k < wv)
                wave_before += wt;
            all += wt;
        }
        const uint32_t carry = carry_s;
        if (i < n_blocks)
            ws.block_pre[i] = carry + wave_before + inc - v;
        __syncthreads();
        if (threadIdx.x == 0)
            carry_s = carry + all;
        __syncthreads();
    }
    const uint32_t total = carry_s;
    // per-head totals from the prefix array: a head's workgroups are contiguous inside each batch
    // entry's segment (the block's own global writes are visible to it after the barriers above)
    for (uint32_t h = threadIdx.x; h < (uint32_t)g.H; h += 1024) {
        uint32_t sum = 0;
        for (uint32_t b = 0; b < (uint32_t)g.B; ++b) {
            const uint32_t first = (b * (uint32_t)g.H + h) * blocks_per_seg, last = first + blocks_per_seg;
            const uint32_t hi = (last < n_blocks) ? ws.block_pre[last] : total;
            sum += hi - ws.block_pre[first];
        }
        enc.n_outliers[h] = sum;
    }
    if (threadIdx.x == 0) {
        enc.n_outliers[g.H] = total;
        enc.row_off[n_rows] = total;
        if ((uint64_t)total > outlier_capacity)
            atomicOr(enc.status, HQMQ_STATUS_OUTLIER_OVERFLOW);  // next to what the search may have reported
    }
}

// grid = (ceil(T / 256), B*H), one thread per row
template <bool kFull>
__global__ __launch_bounds__(kThreads) void k_gather(Geometry g, WorkspaceOffsets wo, EncodeBatch batch)
{
    const EncodeTensor &tn = batch.t[blockIdx.z];
    const Workspace ws = carve_workspace(tn.ws, wo);
    const EncodedPtrs enc = tn.enc;
    const uint64_t outlier_capacity = tn.outlier_capacity;
    const _Float16 *__restrict__ x = tn.x;
    const int seg = blockIdx.y, b = seg / g.H, h = seg % g.H;
    const int t = blockIdx.x * kThreads + threadIdx.x;
    if (t >= g.T)
        return;
    const int64_t R = (int64_t)seg * g.T + t;
    uint32_t word = enc.flags[R];
    const uint32_t off = enc.row_off[R] + ws.block_pre[(size_t)seg * g.n_search_blocks_per_seg + t / g.search_rows];
    enc.row_off[R] = off;
    if (!word)
        return;
    const _Float16 *row = x + (int64_t)b * g.sb + (int64_t)h * g.sh + (int64_t)t * g.st;
    uint64_t pos = off;
    while (word) {
        const int c = __ffs((int)word) - 1;
        word &= word - 1;
        if (pos < outlier_capacity)
            *reinterpret_cast<uint2 *>(enc.outliers + 4 * pos) =
                __builtin_bit_cast(uint2, load_row_chunk<kFull>(row, c, g));
        ++pos;
    }
}

// The outlier list of a small tensor whose search ran in its fused form (no kernel before it): one
// workgroup per tensor does what k_scan and k_gather do, and what k_init would have done for them:
//   scan    exclusive scan of the search workgroups' totals (at most kSmallListBlocks of them, one per
//           thread), per-head totals, grand total, status word (overflow; non-finite input, which the search
//           workgroups report in bit 31 of their totals)
//   gather  every row adds its workgroup's prefix to its offset and copies its flagged chunks
// grid = (1, 1, tensors), 1024 threads.
template <bool kFull>
__global__ __launch_bounds__(1024) void k_list_small(Geometry g, WorkspaceOffsets wo, EncodeBatch batch)
{
    const EncodeTensor &tn = batch.t[blockIdx.z];
    const Workspace ws = carve_workspace(tn.ws, wo);
    const EncodedPtrs enc = tn.enc;
    const uint64_t outlier_capacity = tn.outlier_capacity;
    const _Float16 *__restrict__ x = tn.x;
    __shared__ uint32_t pre[kSmallListBlocks + 1];  // exclusive prefix of the workgroup totals, then the grand total
    __shared__ uint32_t wave_tot[16];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const uint32_t blocks_per_seg = g.n_search_blocks_per_seg;
    const uint32_t n_blocks = (uint32_t)g.B * g.H * blocks_per_seg;  // <= kSmallListBlocks (checked by the host)
    const uint32_t n_rows = (uint32_t)g.B * g.H * g.T;
    // the first round of rows: flag word and local offset requested together with the workgroup totals
    uint32_t word0 = 0, off0 = 0;
    if ((uint32_t)tid < n_rows) {
        word0 = enc.flags[tid];
        off0 = enc.row_off[tid];
    }
    const uint32_t raw = (uint32_t)tid < n_blocks ? ws.block_sum[tid] : 0u;
    const uint32_t v = raw & 0x7fffffffu;
    const int bad = __syncthreads_or((int)(raw >> 31));
    uint32_t inc = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        uint32_t o = __shfl_up(inc, d, 64);
        if (lane >= d)
            inc += o;
    }
    if (lane == 63)
        wave_tot[wv] = inc;
    __syncthreads();
    uint32_t wave_before = 0, total = 0;
    for (int k = 0; k < 16; ++k) {
        const uint32_t wt = wave_tot[k];
        if (k < wv)
            wave_before += wt;
        total += wt;
    }
    if ((uint32_t)tid < n_blocks)
        pre[tid] = wave_before + inc - v;
    if (tid == 0)
        pre[n_blocks] = total;
    __syncthreads();
    for (uint32_t h = tid; h < (uint32_t)g.H; h += 1024) {
        uint32_t sum = 0;
        for (uint32_t b = 0; b < (uint32_t)g.B; ++b) {
            const uint32_t first = (b * (uint32_t)g.H + h) * blocks_per_seg;
            sum += pre[first + blocks_per_seg] - pre[first];
        }
        enc.n_outliers[h] = sum;
    }
    if (tid == 0) {
        enc.n_outliers[g.H] = total;
        enc.row_off[n_rows] = total;
        enc.status[0] = ((uint64_t)total > outlier_capacity ? HQMQ_STATUS_OUTLIER_OVERFLOW : 0u) |
                        (bad ? HQMQ_STATUS_NONFINITE : 0u);
    }
    for (uint32_t R = tid; R < n_rows; R += 1024) {
        const uint32_t seg = R / (uint32_t)g.T, t = R - seg * (uint32_t)g.T;
        const uint32_t b = seg / (uint32_t)g.H, h = seg - b * (uint32_t)g.H;
        uint32_t word = R == (uint32_t)tid ? word0 : enc.flags[R];
        const uint32_t off = (R == (uint32_t)tid ? off0 : enc.row_off[R]) +
                             pre[seg * blocks_per_seg + t / (uint32_t)g.search_rows];
        enc.row_off[R] = off;
        const _Float16 *row = x + (int64_t)b * g.sb + (int64_t)h * g.sh + (int64_t)t * g.st;
        uint64_t pos = off;
        while (word) {
            const int c = __ffs((int)word) - 1;
            word &= word - 1;
            if (pos < outlier_capacity)
                *reinterpret_cast<uint2 *>(enc.outliers + 4 * pos) =
                    __builtin_bit_cast(uint2, load_row_chunk<kFull>(row, c, g));
            ++pos;
        }
    }
}

// ---------------------------------------------------------------------------------------
// The median of a head whose token axis is split over several shards (a context-parallel cache: every
// shard holds a slice of T; paper Sec. 3 takes the median per (layer, head, role) over the whole
// batch).  Plain most-significant-digit radix select with histograms only, so that the one thing the
// shards have to exchange is a histogram: pass 0 counts bits 62..50 of every key, passes 1..5 the
// next 10 bits of the keys under the prefix fixed so far; the caller sums the pass's histogram over
// the shards before the next call, and every shard then takes the same decisions.
//   k_shard_pick   one workgroup per head: (pass > 0) locates the wanted rank in the summed histogram
//                  of the previous pass and extends the prefix; clears the histogram of this pass;
//                  (finish) writes the threshold fl(fl(C C) median)
//   k_shard_hist   sweep of this shard's rows, as k_select_sweep
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ int shard_digit_bits(int pass) { return pass == 0 ? kBits0 : kBits1; }
__device__ __forceinline__ int shard_digit_shift(int pass) { return pass == 0 ? kShift0 : kShift1 - 10 * (pass - 1); }

// pass: the pass about to run (0..5), or 6 = finish.
__global__ __launch_bounds__(kSelectThreads) void k_shard_pick(Geometry g, WorkspaceOffsets wo, EncodeBatch batch,
                                                               int pass, unsigned long long total_per_head, float C)
{
    const EncodeTensor &tn = batch.t[blockIdx.z];
    const Workspace ws = carve_workspace(tn.ws, wo);
    __shared__ uint32_t scratch[kSelectThreads + 2];
    const int h = blockIdx.x;
    unsigned long long prefix = 0;
    uint32_t rank = (uint32_t)((total_per_head - 1) / 2);
    if (pass > 0) {
        prefix = ws.state[h].prefix;
        rank = ws.state[h].rank;
        uint32_t bin, before;
        if (pass == 1)
            pick_bin<kBins0, kSelectThreads>(ws.hist0 + (size_t)h * kBins0, rank, scratch, bin, before);
        else
            pick_bin<kBins1, kSelectThreads>(ws.hist1 + (size_t)h * kBins1, rank, scratch, bin, before);
        prefix = (prefix << shard_digit_bits(pass - 1)) | bin;
        rank -= before;
    }
    if (pass < 6) {
        uint32_t *hist = pass == 0 ? ws.hist0 + (size_t)h * kBins0 : ws.hist1 + (size_t)h * kBins1;
        const int bins = pass == 0 ? kBins0 : kBins1;
        for (int i = threadIdx.x; i < bins; i += kSelectThreads)
            hist[i] = 0;  // after pick_bin's barriers: every thread has read the previous counts
    }
    if (threadIdx.x == 0) {
        ws.state[h].prefix = prefix;
        ws.state[h].rank = rank;
        if (pass == 6) {
            const double c = (double)C;
            const double c2 = c * c;
            ws.thr[h] = c2 * __longlong_as_double((long long)prefix);  // all 63 bits fixed: the median itself
        }
    }
}

template <bool kFull>
__global__ __launch_bounds__(kSelectThreads) void k_shard_hist(Geometry g, WorkspaceOffsets wo, EncodeBatch batch, int pass)
{
    const EncodeTensor &tn = batch.t[blockIdx.z];
    const Workspace ws = carve_workspace(tn.ws, wo);
    const _Float16 *__restrict__ x = tn.x;
    __shared__ uint32_t lh[kBins0];
    const int seg = blockIdx.y, b = seg / g.H, h = seg % g.H;
    const int bins = pass == 0 ? kBins0 : kBins1;
    const int shift = shard_digit_shift(pass), nbits = shard_digit_bits(pass);
    const unsigned long long prefix = ws.state[h].prefix;  // pass 0: zero, and every key matches
    for (int i = threadIdx.x; i < bins; i += kSelectThreads)
        lh[i] = 0;
    __syncthreads();
    const int c = threadIdx.x & 31, sub = threadIdx.x >> 5;
    const int t0 = blockIdx.x * kSelectRows;
    const int t1 = min(g.T, t0 + kSelectRows);
    const _Float16 *base = x + (int64_t)b * g.sb + (int64_t)h * g.sh;
    if (kFull || c < g.n_c) {
        for (int t = t0 + sub; t < t1; t += kSelectThreads / 32) {
            const unsigned long long key =
                key_of(chunk_norm2(load_row_chunk<kFull>(base + (int64_t)t * g.st, c, g))) & kKeyMask;
            // (key >> 63) == 0 == prefix in pass 0; a shift by shift + nbits <= 63 is always defined
            if ((key >> (shift + nbits)) == prefix)
                atomicAdd(&lh[(uint32_t)(key >> shift) & (uint32_t)(bins - 1)], 1u);
        }
    }
    __syncthreads();
    uint32_t *gh = pass == 0 ? ws.hist0 + (size_t)h * kBins0 : ws.hist1 + (size_t)h * kBins1;
    for (int i = threadIdx.x; i < bins; i += kSelectThreads) {
        const uint32_t n = lh[i];
        if (n)
            atomicAdd(&gh[i], n);
    }
}

hipError_t launch_shard_median_pass(const Geometry &g, const WorkspaceOffsets &wo, const EncodeBatch &batch, int pass,
                                    unsigned long long total_per_head, float C, hipStream_t stream)
{
    hipLaunchKernelGGL(k_shard_pick, dim3(g.H, 1, 1), dim3(kSelectThreads), 0, stream, g, wo, batch, pass,
                       total_per_head, C);
    if (pass < 6) {
        dim3 grid((g.T + kSelectRows - 1) / kSelectRows, g.B * g.H, 1);
        if (g.D == 4 * kChunksPerRow)
            hipLaunchKernelGGL(k_shard_hist<true>, grid, dim3(kSelectThreads), 0, stream, g, wo, batch, pass);
        else
            hipLaunchKernelGGL(k_shard_hist<false>, grid, dim3(kSelectThreads), 0, stream, g, wo, batch, pass);
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// host-side launch sequences
// ---------------------------------------------------------------------------------------
template <bool kFull>
static void select_sweeps_for(Geometry g, const WorkspaceOffsets &wo, const EncodeBatch &batch, unsigned n, float C,
                              hipStream_t stream)
{
    const dim3 grid((g.T + kSelectRows - 1) / kSelectRows, g.B * g.H, n), heads(g.H, 1, n), block(kSelectThreads);
    g.select_sampled = (uint64_t)g.B * g.T * g.n_c >= (uint64_t)kSampleMinChunks ? 1 : 0;
    if (g.select_sampled) {
        const int n_t = (g.T + kSampleStride - 1) / kSampleStride;
        const dim3 grid_s((n_t + kSelectRows - 1) / kSelectRows, g.B * g.H, n);
        hipLaunchKernelGGL((k_select_sweep<3, kFull>), grid_s, block, 0, stream, g, wo, batch);
        hipLaunchKernelGGL(k_select_range, heads, block, 0, stream, g, wo, batch);
        hipLaunchKernelGGL((k_select_sweep<0, kFull, true>), grid, block, 0, stream, g, wo, batch);
        hipLaunchKernelGGL(k_select_decide, heads, block, 0, stream, g, wo, batch);
    } else {
        hipLaunchKernelGGL((k_select_sweep<0, kFull>), grid, block, 0, stream, g, wo, batch);
    }
    const int rows_late = g.select_sampled ? kSelectRows * kFallbackSpan : kSelectRows;
    const dim3 grid_late((g.T + rows_late - 1) / rows_late, g.B * g.H, n);
    hipLaunchKernelGGL((k_select_sweep<1, kFull>), grid_late, block, 0, stream, g, wo, batch);
    hipLaunchKernelGGL((k_select_sweep<2, kFull>), grid_late, block, 0, stream, g, wo, batch);
    hipLaunchKernelGGL(k_select_finish<kFull>, heads, block, 0, stream, g, wo, batch, C);
}
static void select_sweeps(const Geometry &g, const WorkspaceOffsets &wo, const EncodeBatch &batch, unsigned n, float C,
                          bool full, hipStream_t stream)
{
    if (full)
        select_sweeps_for<true>(g, wo, batch, n, C, stream);
    else
        select_sweeps_for<false>(g, wo, batch, n, C, stream);
}

hipError_t launch_select_median(const Geometry &g, const WorkspaceOffsets &wo, const EncodeBatch &batch, int n_tensors,
                                float C, bool skip_select, hipStream_t stream)
{
    const unsigned n = (unsigned)n_tensors;
    uint32_t n_init = (uint32_t)g.H * kBins0;
    hipLaunchKernelGGL(k_init, dim3((n_init + kThreads - 1) / kThreads, 1, n), dim3(kThreads), 0, stream, g, wo, batch);
    if (!skip_select) {
        select_sweeps(g, wo, batch, n, C, g.D == 4 * kChunksPerRow, stream);
    }
    return hipGetLastError();
}

hipError_t launch_outlier_list_small(const Geometry &g, const WorkspaceOffsets &wo, const EncodeBatch &batch,
                                     int n_tensors, hipStream_t stream)
{
    const dim3 grid(1, 1, (unsigned)n_tensors);
    if (g.D == 4 * kChunksPerRow)
        hipLaunchKernelGGL(k_list_small<true>, grid, dim3(1024), 0, stream, g, wo, batch);
    else
        hipLaunchKernelGGL(k_list_small<false>, grid, dim3(1024), 0, stream, g, wo, batch);
    return hipGetLastError();
}

hipError_t launch_outlier_list(const Geometry &g, const WorkspaceOffsets &wo, const EncodeBatch &batch, int n_tensors,
                               hipStream_t stream)
{
    const unsigned n = (unsigned)n_tensors;
    const uint32_t n_blocks = (uint32_t)g.B * g.H * g.n_search_blocks_per_seg;
    const uint64_t n_rows = (uint64_t)g.B * g.H * g.T;
    hipLaunchKernelGGL(k_scan, dim3(1, 1, n), dim3(1024), 0, stream, g, wo, batch, n_blocks, n_rows);
    dim3 grid((g.T + kThreads - 1) / kThreads, g.B * g.H, n);
    if (g.D == 4 * kChunksPerRow)
        hipLaunchKernelGGL(k_gather<true>, grid, dim3(kThreads), 0, stream, g, wo, batch);
    else
        hipLaunchKernelGGL(k_gather<false>, grid, dim3(kThreads), 0, stream, g, wo, batch);
    return hipGetLastError();
}

}  // namespace hqmq
