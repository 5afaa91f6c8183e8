// Med3x outlier extraction, first half: the exact per-head median of the squared chunk norms
// and the outlier mask (paper Sec. 3 "Median-multiplier outlier extraction", Alg. 1 "Outlier
// extraction").
//
// The median is the lower median (element (n-1)/2 of the sorted norms) of all B*T*32 chunks of
// a head.  Non-negative IEEE doubles order like their bit patterns read as unsigned integers,
// so the median is found by a most-significant-digit radix select on the 63 value bits of r^2:
// each pass histograms one digit of the keys that still match the digits fixed so far, a tiny
// kernel picks the digit bucket holding the wanted rank.  Nothing is sorted and no float
// arithmetic is involved after r^2 itself, so the result is the exact order statistic.
//
// All passes are HBM-bound sweeps over the fp16 tensor (8 B per chunk); r^2 is recomputed in
// registers each time, which costs less than storing and reloading 8-byte keys.
#include "hqmq_device.h"

namespace hqmq {

// ---------------------------------------------------------------------------------------
// reset of the per-call scratch state
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void k_init(Geometry g, Workspace ws, EncodedPtrs enc,
                                                   uint32_t n_hist, uint32_t n_blocks)
{
    uint32_t i = blockIdx.x * kThreads + threadIdx.x;
    if (i < n_hist)
        ws.hist[i] = 0;
    if (i < n_blocks)
        ws.block_sum[i] = 0;
    if (i < (uint32_t)g.H) {
        uint64_t n_h = (uint64_t)g.B * g.T * kChunksPerRow;
        ws.state[i].prefix = 0;
        ws.state[i].rank = (uint32_t)((n_h - 1) / 2);
        ws.state[i].pad = 0;
        ws.thr[i] = __longlong_as_double(0x7ff0000000000000LL);  // +inf: nothing is flagged
    }
    if (i <= (uint32_t)g.H)
        enc.n_outliers[i] = 0;
    if (i == 0)
        enc.status[0] = 0;
}

// ---------------------------------------------------------------------------------------
// one radix pass: histogram digit `pass` of the keys matching the current prefix
// grid = (ceil(T / kHistRows), B*H); one lane per chunk, 8 rows per block iteration
// ---------------------------------------------------------------------------------------
template <int PASS>
__global__ __launch_bounds__(kThreads) void k_hist(const _Float16 *__restrict__ x, Geometry g,
                                                   Workspace ws)
{
    constexpr int kBits = pass_bits(PASS);
    constexpr int kShift = pass_shift(PASS);
    constexpr int kBins = 1 << kBits;
    __shared__ uint32_t lh[kBins];

    const int seg = blockIdx.y, b = seg / g.H, h = seg % g.H;
    for (int i = threadIdx.x; i < kBins; i += kThreads)
        lh[i] = 0;
    __syncthreads();

    const unsigned long long prefix = (PASS == 0) ? 0ull : ws.state[h].prefix;
    const int c = threadIdx.x & 31, sub = threadIdx.x >> 5;
    const int t0 = blockIdx.x * kHistRows;
    const int t1 = min(g.T, t0 + kHistRows);
    const _Float16 *base = x + (int64_t)b * g.sb + (int64_t)h * g.sh + 4 * c;

    for (int t = t0 + sub; t < t1; t += 32) {
        // four independent 8-byte loads in flight per lane
        half4_t v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            int tt = t + 8 * u;
            v[u] = (tt < t1) ? load_chunk(base + (int64_t)tt * g.st) : half4_t{0, 0, 0, 0};
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (t + 8 * u < t1) {
                unsigned long long key = key_of(chunk_norm2(v[u])) & 0x7fffffffffffffffull;
                if (PASS == 0 || (key >> (kShift + kBits)) == prefix)
                    atomicAdd(&lh[(uint32_t)(key >> kShift) & (kBins - 1)], 1u);
            }
        }
    }
    __syncthreads();
    uint32_t *gh = ws.hist + (size_t)h * kHistBins;
    for (int i = threadIdx.x; i < kBins; i += kThreads) {
        uint32_t n = lh[i];
        if (n)
            atomicAdd(&gh[i], n);
    }
}

// ---------------------------------------------------------------------------------------
// pick the bucket that holds the wanted rank; one block per head.
// After the last pass the prefix is the full key: the median's bit pattern.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void k_pick(Geometry g, Workspace ws, int pass, float C)
{
    const int h = blockIdx.x;
    const int bits = pass_bits(pass);
    const int bins = 1 << bits;
    const int per = bins / kThreads;  // 32 or 16 consecutive bins per thread
    uint32_t *gh = ws.hist + (size_t)h * kHistBins;
    __shared__ uint32_t part[kThreads];
    __shared__ uint32_t sel_bin, sel_before;

    uint32_t local[32];
    uint32_t sum = 0;
#pragma unroll
    for (int i = 0; i < 32; ++i) {
        local[i] = (i < per) ? gh[threadIdx.x * per + i] : 0u;
        sum += local[i];
    }
    part[threadIdx.x] = sum;
    __syncthreads();
    // exclusive prefix of the per-thread sums (256 values: a serial scan by one thread is
    // cheap next to the sweeps around it)
    if (threadIdx.x == 0) {
        uint32_t run = 0;
        for (int i = 0; i < kThreads; ++i) {
            uint32_t v = part[i];
            part[i] = run;
            run += v;
        }
    }
    __syncthreads();
    const uint32_t rank = ws.state[h].rank;
    uint32_t before = part[threadIdx.x];
    if (rank >= before && rank < before + sum) {
        bool found = false;
#pragma unroll
        for (int i = 0; i < 32; ++i) {
            if (!found && rank < before + local[i]) {
                sel_bin = threadIdx.x * per + i;
                sel_before = before;
                found = true;
            }
            if (!found)
                before += local[i];
        }
    }
    __syncthreads();
    for (int i = 0; i < per; ++i)
        gh[threadIdx.x * per + i] = 0;  // ready for the next pass
    if (threadIdx.x == 0) {
        unsigned long long prefix = (ws.state[h].prefix << bits) | sel_bin;
        ws.state[h].prefix = prefix;
        ws.state[h].rank = rank - sel_before;
        if (pass == kNumPasses - 1) {
            // threshold on squares: fl(fl(C*C) * median), C widened from fp32
            double c = (double)C;
            double c2 = c * c;
            ws.thr[h] = c2 * __longlong_as_double((long long)prefix);
        }
    }
}

// ---------------------------------------------------------------------------------------
// outlier mask: one flag word per row, the outlier count of every block of kMaskRows rows
// and the per-head totals.  grid = (ceil(T / kMaskRows), B*H)
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void k_mask(const _Float16 *__restrict__ x, Geometry g,
                                                   Workspace ws, EncodedPtrs enc)
{
    const int seg = blockIdx.y, b = seg / g.H, h = seg % g.H;
    const double thr = ws.thr[h];
    const int c = threadIdx.x & 31, sub = threadIdx.x >> 5;
    const int t0 = blockIdx.x * kMaskRows;
    const int t1 = min(g.T, t0 + kMaskRows);
    const _Float16 *base = x + (int64_t)b * g.sb + (int64_t)h * g.sh + 4 * c;
    const int64_t row0 = (int64_t)seg * g.T;
    uint32_t count = 0;  // per wave (uniform)

    // tb is uniform over the block, so every lane reaches every ballot
    for (int tb = t0; tb < t1; tb += 32) {
        half4_t v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            int tt = tb + sub + 8 * u;
            v[u] = (tt < t1) ? load_chunk(base + (int64_t)tt * g.st) : half4_t{0, 0, 0, 0};
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            int tt = tb + sub + 8 * u;
            bool flag = (tt < t1) && (chunk_norm2(v[u]) > thr);
            unsigned long long ballot = __ballot(flag);
            uint32_t word = (threadIdx.x & 32) ? (uint32_t)(ballot >> 32) : (uint32_t)ballot;
            if (c == 0 && tt < t1)
                enc.flags[row0 + tt] = word;
            count += __popcll(ballot);
        }
    }
    __shared__ uint32_t wave_count[kThreads / 64];
    if ((threadIdx.x & 63) == 0)
        wave_count[threadIdx.x >> 6] = count;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t total = wave_count[0] + wave_count[1] + wave_count[2] + wave_count[3];
        ws.block_sum[(size_t)seg * g.n_mask_blocks_per_seg + blockIdx.x] = total;
        if (total)
            atomicAdd(&enc.n_outliers[h], total);
    }
}

// ---------------------------------------------------------------------------------------
// exclusive scan of the block sums (linear row order), totals and overflow status.
// One block; the number of entries is n_rows / 256, a few thousand at most per tensor.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void k_scan(Geometry g, Workspace ws, EncodedPtrs enc,
                                               uint32_t n_blocks, uint64_t n_rows,
                                               uint64_t outlier_capacity)
{
    __shared__ uint32_t wave_tot[16];
    __shared__ uint32_t carry_s;
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    if (threadIdx.x == 0)
        carry_s = 0;
    __syncthreads();
    for (uint32_t start = 0; start < n_blocks; start += 1024) {
        uint32_t i = start + threadIdx.x;
        uint32_t v = (i < n_blocks) ? ws.block_sum[i] : 0;
        // inclusive scan inside the wave
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
            uint32_t wt = wave_tot[k];
            if (k < wv)
                wave_before += wt;
            all += wt;
        }
        uint32_t carry = carry_s;
        if (i < n_blocks)
            ws.block_pre[i] = carry + wave_before + inc - v;
        __syncthreads();
        if (threadIdx.x == 0)
            carry_s = carry + all;
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        uint32_t total = carry_s;
        enc.n_outliers[g.H] = total;
        enc.row_off[n_rows] = total;
        if ((uint64_t)total > outlier_capacity)
            enc.status[0] = HQMQ_STATUS_OUTLIER_OVERFLOW;
    }
}

// ---------------------------------------------------------------------------------------
// host-side launch sequences
// ---------------------------------------------------------------------------------------
hipError_t launch_select_median(const _Float16 *x, const Geometry &g, const Workspace &ws, float C,
                                bool no_outliers, const EncodedPtrs &enc, hipStream_t stream)
{
    const uint32_t n_hist = (uint32_t)g.H * kHistBins;
    const uint32_t n_blocks = (uint32_t)g.B * g.H * g.n_mask_blocks_per_seg;
    uint32_t n_init = n_hist > n_blocks ? n_hist : n_blocks;
    if (n_init < (uint32_t)g.H + 1)
        n_init = g.H + 1;
    hipLaunchKernelGGL(k_init, dim3((n_init + kThreads - 1) / kThreads), dim3(kThreads), 0, stream, g,
                       ws, enc, n_hist, n_blocks);
    if (!no_outliers) {
        dim3 grid((g.T + kHistRows - 1) / kHistRows, g.B * g.H);
        hipLaunchKernelGGL(k_hist<0>, grid, dim3(kThreads), 0, stream, x, g, ws);
        hipLaunchKernelGGL(k_pick, dim3(g.H), dim3(kThreads), 0, stream, g, ws, 0, C);
        hipLaunchKernelGGL(k_hist<1>, grid, dim3(kThreads), 0, stream, x, g, ws);
        hipLaunchKernelGGL(k_pick, dim3(g.H), dim3(kThreads), 0, stream, g, ws, 1, C);
        hipLaunchKernelGGL(k_hist<2>, grid, dim3(kThreads), 0, stream, x, g, ws);
        hipLaunchKernelGGL(k_pick, dim3(g.H), dim3(kThreads), 0, stream, g, ws, 2, C);
        hipLaunchKernelGGL(k_hist<3>, grid, dim3(kThreads), 0, stream, x, g, ws);
        hipLaunchKernelGGL(k_pick, dim3(g.H), dim3(kThreads), 0, stream, g, ws, 3, C);
        hipLaunchKernelGGL(k_hist<4>, grid, dim3(kThreads), 0, stream, x, g, ws);
        hipLaunchKernelGGL(k_pick, dim3(g.H), dim3(kThreads), 0, stream, g, ws, 4, C);
    }
    return hipGetLastError();
}

hipError_t launch_mask_scan(const _Float16 *x, const Geometry &g, const Workspace &ws,
                            const EncodedPtrs &enc, uint64_t outlier_capacity, hipStream_t stream)
{
    dim3 grid(g.n_mask_blocks_per_seg, g.B * g.H);
    hipLaunchKernelGGL(k_mask, grid, dim3(kThreads), 0, stream, x, g, ws, enc);
    const uint32_t n_blocks = (uint32_t)g.B * g.H * g.n_mask_blocks_per_seg;
    const uint64_t n_rows = (uint64_t)g.B * g.H * g.T;
    hipLaunchKernelGGL(k_scan, dim3(1), dim3(1024), 0, stream, g, ws, enc, n_blocks, n_rows,
                       outlier_capacity);
    return hipGetLastError();
}

}  // namespace hqmq
