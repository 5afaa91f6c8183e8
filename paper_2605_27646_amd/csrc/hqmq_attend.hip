// Single-query attention straight from the packed cache (paper App. F, the fused attention
// kernel: O = softmax(Q K^T scale) V with K and V decoded inside the attention loop and never
// written out in fp16).  This is the generation step's shape: one query token per sequence, G
// query heads sharing each kv head.
//
// Bound by the decode arithmetic and the packed bytes: per cached token it reads 2 * (4 w + 10)
// bytes plus the outlier payloads, where plain fp16 attention reads 512.  Shape:
//   * split-K over the sequence: workgroup (split, b * H + h) walks its rows in tiles of 64, a wave
//     takes 16 rows of a tile; the encoded rows of K and of V arrive with coalesced loads that are
//     issued one tile ahead and re-distributed through LDS exactly as in the stand-alone decode;
//   * a lane owns two adjacent chunks (8 of the 128 dimensions) of four of the wave's rows: the
//     query-key products are partial sums over those 8 dimensions, completed across the 16 lanes
//     of a row with a butterfly; every reconstructed K or V chunk serves all G query heads;
//   * online softmax in the log2 domain (the scale and log2 e are folded into the query), one
//     rescale per group of 4 rows; each 16-lane group keeps its own running maximum / sum /
//     weighted value sum, merged across groups, waves and finally splits (second kernel);
//   * flagged chunks take their stored fp16 payload, from the wave's window of the outlier list.
#include <type_traits>

#include "hqmq_device.h"

namespace hqmq {

namespace {

constexpr int kAttThreads = 256;
constexpr int kAttWaves = kAttThreads / 64;
constexpr int kStageRows = 16;                      // rows per wave and tile
constexpr int kSubs = kStageRows / 4;               // a wave handles 4 rows at a time
constexpr int kMaxW = 24;                           // w <= 22
constexpr int kStageWords = kStageRows * kMaxW + 2; // + 2 words of padding for the 3-word window
constexpr int kPaySlots = 64;                       // outlier payloads of a wave's 16 rows kept in LDS
constexpr int kSideWords = kStageWords + 3 * kStageRows + 2 * kPaySlots;  // one side (K or V) of one wave
constexpr int kLoadsPerLane = (kStageRows * kMaxW + 63) / 64;
constexpr float kNegBig = -1.0e30f;                 // "no row seen yet" (finite, so differences stay finite)
#ifndef HQMQ_ATTEND_TARGET_BLOCKS
#define HQMQ_ATTEND_TARGET_BLOCKS 2048
#endif
constexpr int kAttendTargetBlocks = HQMQ_ATTEND_TARGET_BLOCKS;  // workgroups to aim for across the chip
constexpr int kRedStride = 2 + 128;                 // one partial state: maximum, sum, 128 weighted values

static_assert(kAttendTile == kAttWaves * kStageRows, "tile = rows of all waves");
static_assert(kAttWaves * kMaxGroup * kRedStride <= kAttWaves * 2 * kSideWords,
              "the end-of-workgroup reduction re-uses the staging area");

__device__ __forceinline__ void wave_lds_sync()
{
    // LDS serves the instructions of one wave in order; this only stops the compiler from moving
    // LDS accesses of other lanes' data across the point.
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// One tile's encoded rows of one side on their way from memory to LDS.
struct TileRegs {
    uint32_t cw[kLoadsPerLane];
    uint32_t fw, sg, ro;
};

__device__ __forceinline__ void load_tile(TileRegs &t, const AttendSide &s, int64_t R0, int nrows,
                                          uint32_t w, int lane)
{
#pragma unroll
    for (int j = 0; j < kLoadsPerLane; ++j)
        t.cw[j] = 0;
    t.fw = t.sg = t.ro = 0;
    if (nrows > 0) {
        const uint32_t *cw = s.codes + R0 * w;
        const int ncw = nrows * (int)w;
#pragma unroll
        for (int j = 0; j < kLoadsPerLane; ++j)
            if (lane + 64 * j < ncw)
                t.cw[j] = cw[lane + 64 * j];
        if (lane < nrows) {
            t.fw = s.flags[R0 + lane];
            t.sg = s.sigma[R0 + lane];
            t.ro = s.row_off[R0 + lane];
        }
    }
}

__device__ __forceinline__ void stage_tile(const TileRegs &t, uint32_t *stage, int lane)
{
#pragma unroll
    for (int j = 0; j < kLoadsPerLane; ++j)
        stage[lane + 64 * j] = t.cw[j];
    if (lane < 2)
        stage[kStageWords - 2 + lane] = 0;
    if (lane < kStageRows) {
        stage[kStageWords + lane] = t.fw;
        stage[kStageWords + kStageRows + lane] = t.sg;
        stage[kStageWords + 2 * kStageRows + lane] = t.ro;
    }
}

// Sum over the 16 lanes of a row (quad swaps, then the two mirror patterns: after each step the
// partial sums are uniform over a block twice as large, so a mirror pairs the right blocks).
template <int kCtrl>
__device__ __forceinline__ float dpp_move(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), kCtrl, 0xf, 0xf, true));
}
__device__ __forceinline__ float row16_sum(float v)
{
    v += dpp_move<0xB1>(v);   // quad_perm [1, 0, 3, 2]
    v += dpp_move<0x4E>(v);   // quad_perm [2, 3, 0, 1]
    v += dpp_move<0x141>(v);  // row_half_mirror
    v += dpp_move<0x140>(v);  // row_mirror
    return v;
}

// m, l, acc <- merge of two partial softmax states (log2 domain)
template <int N>
__device__ __forceinline__ void merge_state(float &m, float &l, float (&acc)[N], float m2, float l2,
                                            const float (&acc2)[N])
{
    const float mn = fmaxf(m, m2);
    const float c1 = __builtin_amdgcn_exp2f(m - mn), c2 = __builtin_amdgcn_exp2f(m2 - mn);
    l = l * c1 + l2 * c2;
#pragma unroll
    for (int i = 0; i < N; ++i)
        acc[i] = acc[i] * c1 + acc2[i] * c2;
    m = mn;
}

}  // namespace

// grid = (n_splits, B*H), block = 256.
// dynamic LDS: prim [48][4] f32 | staging [4 waves][K, V][kSideWords] u32 | q [G][128] f32 |
//              secondaries of K [S][4] f32 | secondaries of V [S][4] f32
template <bool kPow2, int G>
__global__ __launch_bounds__(kAttThreads) void k_attend_partial(Geometry g, AttendArgs a)
{
    extern __shared__ float lds[];
    float *prim = lds;
    uint32_t *stage_all = reinterpret_cast<uint32_t *>(prim + 48 * 4);
    float *q_l = reinterpret_cast<float *>(stage_all + kAttWaves * 2 * kSideWords);
    float *sec_k = q_l + G * 128;
    float *sec_v = sec_k + 4 * g.S;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform, and known to be
    const int seg = blockIdx.y, b = seg / g.H, h = seg % g.H;
    const int split = blockIdx.x;
    const int cp = lane & 15, rsub = lane >> 4;
    const uint32_t w = g.w, w_idx = g.w_idx;
    const int row_begin = split * a.rows_per_split;
    const int row_end = min(g.T, row_begin + a.rows_per_split);

    uint32_t *stage_k = stage_all + (wv * 2 + 0) * kSideWords;
    uint32_t *stage_v = stage_all + (wv * 2 + 1) * kSideWords;

    // ---- first tile on its way while the tables are set up ----------------------------------------------
    TileRegs tk, tv;
    {
        const int tg = row_begin + wv * kStageRows;
        const int nrows = min(kStageRows, row_end - tg);
        const int64_t R0 = (int64_t)seg * g.T + tg;
        load_tile(tk, a.k, R0, nrows, w, lane);
        load_tile(tv, a.v, R0, nrows, w, lane);
    }
    {
        const float *sk = a.k.sec + (size_t)h * g.S * 4, *sv = a.v.sec + (size_t)h * g.S * 4;
        for (int s = tid; s < g.S; s += kAttThreads) {
            *reinterpret_cast<float4_t *>(sec_k + 4 * s) = *reinterpret_cast<const float4_t *>(sk + 4 * s);
            *reinterpret_cast<float4_t *>(sec_v + 4 * s) = *reinterpret_cast<const float4_t *>(sv + 4 * s);
        }
        if (tid < 48 * 4) {
            const int p = tid >> 2, i = tid & 3;
            float v = 0.f;
            if (p < 8)
                v = ((p >> 1) == i) ? ((p & 1) ? -1.f : 1.f) : 0.f;
            else if (p < 24)
                v = (((p - 8) >> (3 - i)) & 1) ? -0.5f : 0.5f;
            prim[tid] = v;
        }
        const _Float16 *qh = a.q + ((size_t)b * g.H + h) * G * 128;  // the G query heads of this kv head
        for (int i = tid; i < G * 128; i += kAttThreads)
            q_l[i] = (float)qh[i] * a.qscale;
    }
    __syncthreads();

    float m[G], l[G], acc[G][8];
#pragma unroll
    for (int gq = 0; gq < G; ++gq) {
        m[gq] = kNegBig;
        l[gq] = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i)
            acc[gq][i] = 0.f;
    }

    const uint32_t bitpos = (uint32_t)(2 * cp) * w;
    const uint32_t i0 = bitpos >> 5, sh0 = bitpos & 31;
    const uint32_t sh1 = sh0 + w;
    const bool second_in_low = sh1 < 32;
    const uint32_t code_mask = (1u << w) - 1u, idx_mask = (1u << w_idx) - 1u;
    const float inv_L = g.inv_L;

    // Outlier payloads of a wave's 16 rows: one contiguous window of the list.  Opened from the
    // tile's registers (offset of the first row, offset + count of the last) half a tile ahead.
    struct Window {
        uint32_t base;
        bool ok;     // the whole window fits the LDS slots and the list's capacity
        uint2 mine;  // this lane's entry of the window, on its way to LDS
    };
    auto open_window = [&](const AttendSide &s, const TileRegs &t, int nrows) {
        Window wd;
        wd.base = 0;
        wd.ok = true;
        wd.mine = make_uint2(0u, 0u);
        if (nrows > 0) {
            const int last_row = nrows - 1;
            wd.base = (uint32_t)__builtin_amdgcn_readlane((int)t.ro, 0);
            const uint32_t ro_l = (uint32_t)__builtin_amdgcn_readlane((int)t.ro, last_row);
            const uint32_t fw_l = (uint32_t)__builtin_amdgcn_readlane((int)t.fw, last_row);
            const uint32_t pay_n = ro_l + __popc(fw_l) - wd.base;
            // unconditional load: lanes past the window (or the list's capacity) re-read a neighbour's
            // entry; a wave without outliers reads 8 harmless bytes of the offset array
            const bool has_pay = pay_n > 0 && (uint64_t)wd.base < s.outlier_capacity;
            const uint64_t last = has_pay ? min((uint64_t)pay_n, s.outlier_capacity - wd.base) - 1u : 0u;
            const uint2 *src = has_pay ? reinterpret_cast<const uint2 *>(s.outliers) + wd.base
                                       : reinterpret_cast<const uint2 *>(s.row_off);
            wd.mine = src[min((uint64_t)lane, last)];
            wd.ok = pay_n <= (uint32_t)kPaySlots && (uint64_t)wd.base + pay_n <= s.outlier_capacity;
        }
        return wd;
    };

    // ---- reconstruction of the lane's two chunks of row 4 sub + rsub --------------------------------
    auto decode_chunk = [&](uint32_t code, float sol, const float *secl, float *y) {
        const uint32_t rq = code >> w_idx;
        uint32_t p_off, s_off;
        if (kPow2) {
            p_off = ((code >> g.log2_S) & 31u) << 4;
            s_off = (code << 4) & (((uint32_t)g.S - 1u) << 4);
        } else {
            const uint32_t k = code & idx_mask;
            const uint32_t p = (uint32_t)((float)k * g.inv_S);  // exact for k < 48 S
            p_off = p << 4;
            s_off = (k - __umul24(p, (uint32_t)g.S)) << 4;
        }
        const float4_t P = *reinterpret_cast<const float4_t *>(reinterpret_cast<const char *>(prim) + p_off);
        const float4_t q = *reinterpret_cast<const float4_t *>(reinterpret_cast<const char *>(secl) + s_off);
        const float rh = (float)rq * sol;
        const float R0 = rh * P[0], R1 = rh * P[1], R2 = rh * P[2], R3 = rh * P[3];
        y[0] = fmaf(-R3, q[3], fmaf(-R2, q[2], fmaf(-R1, q[1], R0 * q[0])));
        y[1] = fmaf(-R3, q[2], fmaf(R2, q[3], fmaf(R1, q[0], R0 * q[1])));
        y[2] = fmaf(R3, q[1], fmaf(R2, q[0], fmaf(-R1, q[3], R0 * q[2])));
        y[3] = fmaf(R3, q[0], fmaf(-R2, q[1], fmaf(R1, q[2], R0 * q[3])));
    };
    // the 8 values of the lane's chunk pair: reconstruction, flagged chunks replaced by their payload
    // (kFast: the wave's whole payload window sits in LDS, so the patch is branch-free; the other
    // form serves windows beyond the LDS slots or the list's capacity.  The choice is made per tile,
    // outside the loop over row groups, which keeps each group's code straight-line.)
    auto row_values = [&](auto fast_tag, const AttendSide &s, const uint32_t *stage, const float *secl,
                          uint32_t base, int sub, int nrows, float *y) {
        constexpr bool kFast = decltype(fast_tag)::value;
        const int r = 4 * sub + rsub;
        const uint32_t *rw = stage + r * w + i0;
        const uint32_t d0 = rw[0], d1 = rw[1], d2 = rw[2];
        const uint32_t word = stage[kStageWords + r];
        const float sigma = (float)__builtin_bit_cast(_Float16, (uint16_t)stage[kStageWords + kStageRows + r]);
        const uint32_t code0 = __builtin_amdgcn_alignbit(d1, d0, sh0) & code_mask;
        const uint32_t lo_win = __builtin_amdgcn_alignbit(d1, d0, sh1);
        const uint32_t hi_win = __builtin_amdgcn_alignbit(d2, d1, sh1);
        const uint32_t code1 = (second_in_low ? lo_win : hi_win) & code_mask;
        const uint32_t fl = (r < nrows) ? ((word >> (2 * cp)) & 3u) : 0u;
        const uint32_t pos = stage[kStageWords + 2 * kStageRows + r] + __popc(word & ((1u << (2 * cp)) - 1u)) - base;
        const float sol = sigma * inv_L;
        decode_chunk(code0, sol, secl, y);
        decode_chunk(code1, sol, secl, y + 4);
        const uint2 *st_pay = reinterpret_cast<const uint2 *>(stage + kStageWords + 3 * kStageRows);
        uint2 pa = make_uint2(0u, 0u), pb = make_uint2(0u, 0u);
        if (kFast) {
            pa = st_pay[min(pos, (uint32_t)kPaySlots - 1u)];
            pb = st_pay[min(pos + (fl & 1u), (uint32_t)kPaySlots - 1u)];
        } else {
            // per chunk, still without branches: from LDS, from memory beyond the slots (the load is
            // unconditional, its index clamped into the list), zeros beyond the list's capacity
            const bool any = s.outlier_capacity > 0;
            const uint2 *src = any ? reinterpret_cast<const uint2 *>(s.outliers)
                                   : reinterpret_cast<const uint2 *>(s.row_off);
            const uint64_t last = any ? s.outlier_capacity - 1u : 0u;
            auto fetch = [&](uint32_t slot) {
                const uint64_t at = (uint64_t)base + slot;
                const uint2 far = src[min(at, last)];
                const uint2 near = st_pay[min(slot, (uint32_t)kPaySlots - 1u)];
                uint2 v = (slot < (uint32_t)kPaySlots) ? near : far;
                if (at >= s.outlier_capacity)
                    v = make_uint2(0u, 0u);
                return v;
            };
            pa = fetch(pos);
            pb = fetch(pos + (fl & 1u));
        }
        const half4_t ha = __builtin_bit_cast(half4_t, pa), hb = __builtin_bit_cast(half4_t, pb);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            y[i] = (fl & 1u) ? (float)ha[i] : y[i];
            y[4 + i] = (fl & 2u) ? (float)hb[i] : y[4 + i];
        }
    };

    int nrows = min(kStageRows, row_end - (row_begin + wv * kStageRows));
    Window wk = open_window(a.k, tk, nrows), wvw = open_window(a.v, tv, nrows);

    for (int t0 = row_begin; t0 < row_end; t0 += kAttendTile) {
        // ---- this tile's rows and payload windows into LDS; the next tile's rows requested -----------
        stage_tile(tk, stage_k, lane);
        stage_tile(tv, stage_v, lane);
        reinterpret_cast<uint2 *>(stage_k + kStageWords + 3 * kStageRows)[lane] = wk.mine;
        reinterpret_cast<uint2 *>(stage_v + kStageWords + 3 * kStageRows)[lane] = wvw.mine;
        wave_lds_sync();
        const uint32_t base_k = wk.base, base_v = wvw.base;
        const bool ok_k = wk.ok, ok_v = wvw.ok;
        const bool more = t0 + kAttendTile < row_end;
        const int tgn = t0 + kAttendTile + wv * kStageRows;
        const int nn = more ? min(kStageRows, row_end - tgn) : 0;
        if (more) {
            const int64_t R0n = (int64_t)seg * g.T + tgn;
            load_tile(tk, a.k, R0n, nn, w, lane);
            load_tile(tv, a.v, R0n, nn, w, lane);
        }

        // ---- scores of 4 rows x G heads -------------------------------------------------------------------
        float pw[G][kSubs];
        auto scores = [&](auto fast_tag) {
#pragma unroll
            for (int sub = 0; sub < kSubs; ++sub) {
                // the query is re-read from LDS for every row group (an opaque offset keeps the
                // compiler from parking all 8 G values in registers)
                int q_off = 8 * cp;
                asm volatile("" : "+v"(q_off));
                float y[8];
                row_values(fast_tag, a.k, stage_k, sec_k, base_k, sub, nrows, y);
#pragma unroll
                for (int gq = 0; gq < G; ++gq) {
                    const float4_t qa = *reinterpret_cast<const float4_t *>(q_l + gq * 128 + q_off);
                    const float4_t qb = *reinterpret_cast<const float4_t *>(q_l + gq * 128 + q_off + 4);
                    float s = qa[0] * y[0];
                    s = fmaf(qa[1], y[1], s);
                    s = fmaf(qa[2], y[2], s);
                    s = fmaf(qa[3], y[3], s);
                    s = fmaf(qb[0], y[4], s);
                    s = fmaf(qb[1], y[5], s);
                    s = fmaf(qb[2], y[6], s);
                    s = fmaf(qb[3], y[7], s);
                    pw[gq][sub] = row16_sum(s);
                }
                // keep the four row groups apart: interleaving them only lengthens live ranges
                //SB __builtin_amdgcn_sched_barrier(0);
            }
        };
        if (nrows > 0) {
            if (ok_k)
                scores(std::true_type{});
            else
                scores(std::false_type{});
            // ---- softmax update, one rescale per 4 rows ---------------------------------------------------
#pragma unroll
            for (int gq = 0; gq < G; ++gq) {
                float mn = m[gq];
#pragma unroll
                for (int sub = 0; sub < kSubs; ++sub)
                    mn = fmaxf(mn, (4 * sub + rsub < nrows) ? pw[gq][sub] : kNegBig);
                const float corr = __builtin_amdgcn_exp2f(m[gq] - mn);
                float psum = 0.f;
#pragma unroll
                for (int sub = 0; sub < kSubs; ++sub) {
                    const float e = __builtin_amdgcn_exp2f(pw[gq][sub] - mn);
                    pw[gq][sub] = (4 * sub + rsub < nrows) ? e : 0.f;
                    psum += pw[gq][sub];
                }
                l[gq] = l[gq] * corr + psum;
#pragma unroll
                for (int i = 0; i < 8; ++i)
                    acc[gq][i] *= corr;
                m[gq] = mn;
            }
        }

        // ---- the next tile's payload windows (its offsets have arrived by now) ---------------------------
        if (more) {
            wk = open_window(a.k, tk, nn);
            wvw = open_window(a.v, tv, nn);
        }

        // ---- weighted values ----------------------------------------------------------------------------
        auto weighted_values = [&](auto fast_tag) {
#pragma unroll
            for (int sub = 0; sub < kSubs; ++sub) {
                float vx[8];
                row_values(fast_tag, a.v, stage_v, sec_v, base_v, sub, nrows, vx);
#pragma unroll
                for (int gq = 0; gq < G; ++gq)
#pragma unroll
                    for (int i = 0; i < 8; ++i)
                        acc[gq][i] = fmaf(pw[gq][sub], vx[i], acc[gq][i]);
                //SB __builtin_amdgcn_sched_barrier(0);
            }
        };
        if (nrows > 0) {
            if (ok_v)
                weighted_values(std::true_type{});
            else
                weighted_values(std::false_type{});
        }
        nrows = nn;
    }

    // ---- merge: the 4 row groups of a wave (lanes l, l^16, l^32, l^48), then the 4 waves -----------------
#pragma unroll
    for (int gq = 0; gq < G; ++gq) {
#pragma unroll
        for (int step = 16; step <= 32; step <<= 1) {
            const float m2 = __shfl_xor(m[gq], step), l2 = __shfl_xor(l[gq], step);
            float a2[8];
#pragma unroll
            for (int i = 0; i < 8; ++i)
                a2[i] = __shfl_xor(acc[gq][i], step);
            merge_state(m[gq], l[gq], acc[gq], m2, l2, a2);
        }
    }
    __syncthreads();  // every wave is done with its staging area
    float *red = reinterpret_cast<float *>(stage_all);
    if (rsub == 0) {
#pragma unroll
        for (int gq = 0; gq < G; ++gq) {
            float *dst = red + (wv * G + gq) * kRedStride;
            if (cp == 0) {
                dst[0] = m[gq];
                dst[1] = l[gq];
            }
#pragma unroll
            for (int i = 0; i < 8; ++i)
                dst[2 + 8 * cp + i] = acc[gq][i];
        }
    }
    __syncthreads();
    for (int idx = tid; idx < G * 128; idx += kAttThreads) {
        const int gq = idx >> 7, d = idx & 127;
        float mm = kNegBig;
#pragma unroll
        for (int wq = 0; wq < kAttWaves; ++wq)
            mm = fmaxf(mm, red[(wq * G + gq) * kRedStride]);
        float ll = 0.f, oo = 0.f;
#pragma unroll
        for (int wq = 0; wq < kAttWaves; ++wq) {
            const float *src = red + (wq * G + gq) * kRedStride;
            const float c = __builtin_amdgcn_exp2f(src[0] - mm);
            ll = fmaf(src[1], c, ll);
            oo = fmaf(src[2 + d], c, oo);
        }
        const size_t head = (size_t)seg * G + gq;  // = b * (H G) + h * G + gq
        a.part_acc[(head * a.n_splits + split) * 128 + d] = oo;
        if (d == 0) {
            a.part_ml[(head * a.n_splits + split) * 2 + 0] = mm;
            a.part_ml[(head * a.n_splits + split) * 2 + 1] = ll;
        }
    }
}

// grid = (B * H * G, 8): workgroup (head, y) produces 16 of the head's 128 output dimensions.
// First the global maximum and the weight 2^(m_s - M) of every split (kept in LDS), then plain
// weighted sums with independent loads: thread (j, i) adds the splits j, j + 16, ... for dimension i.
constexpr int kMergeDims = 16;
constexpr int kMergeWays = kAttThreads / kMergeDims;
__global__ __launch_bounds__(kAttThreads) void k_attend_merge(AttendArgs a)
{
    extern __shared__ float wts[];  // [n_splits] weights, then [kMergeWays][kMergeDims + 1] partial sums
    __shared__ float red[kAttWaves];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const size_t head = blockIdx.x;
    const int d0 = blockIdx.y * kMergeDims;
    const int n = a.n_splits;
    const float2 *ml = reinterpret_cast<const float2 *>(a.part_ml) + head * n;
    const float *pa = a.part_acc + head * n * 128;

    float mx = kNegBig;
    for (int s = tid; s < n; s += kAttThreads)
        mx = fmaxf(mx, ml[s].x);
#pragma unroll
    for (int step = 32; step >= 1; step >>= 1)
        mx = fmaxf(mx, __shfl_xor(mx, step));
    if (lane == 0)
        red[wv] = mx;
    __syncthreads();
    mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    __syncthreads();
    float lsum = 0.f;
    for (int s = tid; s < n; s += kAttThreads) {
        const float2 st = ml[s];
        const float wgt = __builtin_amdgcn_exp2f(st.x - mx);
        wts[s] = wgt;
        lsum = fmaf(st.y, wgt, lsum);
    }
#pragma unroll
    for (int step = 32; step >= 1; step >>= 1)
        lsum += __shfl_xor(lsum, step);
    if (lane == 0)
        red[wv] = lsum;
    __syncthreads();
    lsum = (red[0] + red[1]) + (red[2] + red[3]);

    const int i = tid % kMergeDims, j = tid / kMergeDims;
    float o = 0.f;
    int s = j;
    for (; s + 3 * kMergeWays < n; s += 4 * kMergeWays) {  // four loads in flight
        const float v0 = pa[(size_t)s * 128 + d0 + i];
        const float v1 = pa[(size_t)(s + kMergeWays) * 128 + d0 + i];
        const float v2 = pa[(size_t)(s + 2 * kMergeWays) * 128 + d0 + i];
        const float v3 = pa[(size_t)(s + 3 * kMergeWays) * 128 + d0 + i];
        o = fmaf(v0, wts[s], o);
        o = fmaf(v1, wts[s + kMergeWays], o);
        o = fmaf(v2, wts[s + 2 * kMergeWays], o);
        o = fmaf(v3, wts[s + 3 * kMergeWays], o);
    }
    for (; s < n; s += kMergeWays)
        o = fmaf(pa[(size_t)s * 128 + d0 + i], wts[s], o);
    float *sums = wts + n;
    sums[j * (kMergeDims + 1) + i] = o;
    __syncthreads();
    if (tid < kMergeDims) {
        float tot = 0.f;
#pragma unroll
        for (int jj = 0; jj < kMergeWays; ++jj)
            tot += sums[jj * (kMergeDims + 1) + tid];
        a.out[head * 128 + d0 + tid] = (_Float16)(tot / lsum);
    }
}

AttendPlan plan_attend(const Geometry &g, int G)
{
    AttendPlan p;
    const int64_t n_tiles = ((int64_t)g.T + kAttendTile - 1) / kAttendTile;
    const int64_t segs = (int64_t)g.B * g.H;
    int64_t want = (kAttendTargetBlocks + segs - 1) / segs;
    if (want > n_tiles)
        want = n_tiles;
    if (want < 1)
        want = 1;
    const int64_t tiles_per_split = (n_tiles + want - 1) / want;
    p.rows_per_split = (int32_t)(tiles_per_split * kAttendTile);
    p.n_splits = (int32_t)((n_tiles + tiles_per_split - 1) / tiles_per_split);
    const uint64_t heads = (uint64_t)segs * G;
    p.ml_bytes = (heads * p.n_splits * 2 * sizeof(float) + 255) / 256 * 256;
    p.acc_bytes = (heads * p.n_splits * 128 * sizeof(float) + 255) / 256 * 256;
    p.total_bytes = p.ml_bytes + p.acc_bytes;
    return p;
}

template <bool kPow2, int G>
static void launch_partial(const Geometry &g, const AttendArgs &a, size_t lds, hipStream_t stream)
{
    dim3 grid((unsigned)a.n_splits, (unsigned)(g.B * g.H));
    hipLaunchKernelGGL((k_attend_partial<kPow2, G>), grid, dim3(kAttThreads), lds, stream, g, a);
}

template <bool kPow2>
static bool launch_partial_g(const Geometry &g, const AttendArgs &a, size_t lds, hipStream_t stream)
{
    switch (a.G) {
    case 1: launch_partial<kPow2, 1>(g, a, lds, stream); return true;
    case 2: launch_partial<kPow2, 2>(g, a, lds, stream); return true;
    case 3: launch_partial<kPow2, 3>(g, a, lds, stream); return true;
    case 4: launch_partial<kPow2, 4>(g, a, lds, stream); return true;
    case 5: launch_partial<kPow2, 5>(g, a, lds, stream); return true;
    case 6: launch_partial<kPow2, 6>(g, a, lds, stream); return true;
    case 7: launch_partial<kPow2, 7>(g, a, lds, stream); return true;
    case 8: launch_partial<kPow2, 8>(g, a, lds, stream); return true;
    default: return false;
    }
}

hipError_t launch_attend(const Geometry &g, const AttendArgs &a, hipStream_t stream)
{
    const size_t lds = (size_t)(48 * 4 + a.G * 128 + 8 * g.S) * sizeof(float) +
                       (size_t)kAttWaves * 2 * kSideWords * sizeof(uint32_t);
    const bool ok = ((g.S & (g.S - 1)) == 0) ? launch_partial_g<true>(g, a, lds, stream)
                                             : launch_partial_g<false>(g, a, lds, stream);
    if (!ok)
        return hipErrorInvalidValue;
    hipError_t err = hipGetLastError();
    if (err != hipSuccess)
        return err;
    const size_t merge_lds = ((size_t)a.n_splits + kMergeWays * (kMergeDims + 1)) * sizeof(float);
    hipLaunchKernelGGL(k_attend_merge, dim3((unsigned)(g.B * g.H * a.G), 128 / kMergeDims), dim3(kAttThreads),
                       merge_lds, stream, a);
    return hipGetLastError();
}

}  // namespace hqmq
