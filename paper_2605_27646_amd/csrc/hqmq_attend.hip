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

    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
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

    for (int t0 = row_begin; t0 < row_end; t0 += kAttendTile) {
        const int tg = t0 + wv * kStageRows;
        const int nrows = min(kStageRows, row_end - tg);  // <= 0: this wave has no rows in the tile
        stage_tile(tk, stage_k, lane);
        stage_tile(tv, stage_v, lane);
        wave_lds_sync();

        // ---- payload windows of the wave's rows (K and V), then the next tile's encoded rows ---------
        struct Window {
            uint32_t base;
            bool ok;
            uint2 mine;
        };
        auto open_window = [&](const AttendSide &s, const uint32_t *stage) {
            Window wd;
            wd.base = 0;
            wd.ok = true;
            wd.mine = make_uint2(0u, 0u);
            if (nrows > 0) {
                const uint32_t *st_flags = stage + kStageWords, *st_roff = stage + kStageWords + 2 * kStageRows;
                wd.base = st_roff[0];
                const uint32_t pay_n = st_roff[nrows - 1] + __popc(st_flags[nrows - 1]) - wd.base;
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
        const Window wk = open_window(a.k, stage_k), wvw = open_window(a.v, stage_v);
        if (t0 + kAttendTile < row_end) {
            const int tgn = tg + kAttendTile;
            const int nn = min(kStageRows, row_end - tgn);
            const int64_t R0n = (int64_t)seg * g.T + tgn;
            load_tile(tk, a.k, R0n, nn, w, lane);
            load_tile(tv, a.v, R0n, nn, w, lane);
        }
        if (nrows <= 0)
            continue;

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
        auto decode_pair = [&](const uint32_t *stage, const float *secl, uint32_t base, int sub, float *y,
                               uint32_t &fl, uint32_t &pos) {
            const int r = 4 * sub + rsub;
            const uint32_t *rw = stage + r * w + i0;
            const uint32_t d0 = rw[0], d1 = rw[1], d2 = rw[2];
            const uint32_t word = stage[kStageWords + r];
            const float sigma = (float)__builtin_bit_cast(_Float16, (uint16_t)stage[kStageWords + kStageRows + r]);
            const uint32_t code0 = __builtin_amdgcn_alignbit(d1, d0, sh0) & code_mask;
            const uint32_t lo_win = __builtin_amdgcn_alignbit(d1, d0, sh1);
            const uint32_t hi_win = __builtin_amdgcn_alignbit(d2, d1, sh1);
            const uint32_t code1 = (second_in_low ? lo_win : hi_win) & code_mask;
            fl = (r < nrows) ? ((word >> (2 * cp)) & 3u) : 0u;
            pos = stage[kStageWords + 2 * kStageRows + r] + __popc(word & ((1u << (2 * cp)) - 1u)) - base;
            const float sol = sigma * inv_L;
            decode_chunk(code0, sol, secl, y);
            decode_chunk(code1, sol, secl, y + 4);
        };
        // flagged chunks: the stored fp16 values replace the reconstruction
        auto patch = [&](const AttendSide &s, const uint32_t *stage, const Window &wd, uint32_t fl, uint32_t pos,
                         float *y) {
            const uint2 *st_pay = reinterpret_cast<const uint2 *>(stage + kStageWords + 3 * kStageRows);
            uint2 pa = make_uint2(0u, 0u), pb = make_uint2(0u, 0u);
            if (wd.ok) {
                pa = st_pay[min(pos, (uint32_t)kPaySlots - 1u)];
                pb = st_pay[min(pos + (fl & 1u), (uint32_t)kPaySlots - 1u)];
            } else if (fl) {
                // window larger than the LDS slots, or a list shorter than the offsets say: per chunk
                auto fetch = [&](uint32_t slot) {
                    uint2 v = make_uint2(0u, 0u);
                    const uint64_t at = (uint64_t)wd.base + slot;
                    if (at < s.outlier_capacity)
                        v = (slot < (uint32_t)kPaySlots) ? st_pay[slot]
                                                         : *reinterpret_cast<const uint2 *>(s.outliers + 4 * at);
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

        float kx[kSubs][8];
        uint32_t kfl[kSubs], kpos[kSubs];
#pragma unroll
        for (int sub = 0; sub < kSubs; ++sub)
            decode_pair(stage_k, sec_k, wk.base, sub, kx[sub], kfl[sub], kpos[sub]);
        // the payload windows land in LDS only now, after the arithmetic that does not need them
        reinterpret_cast<uint2 *>(stage_k + kStageWords + 3 * kStageRows)[lane] = wk.mine;
        reinterpret_cast<uint2 *>(stage_v + kStageWords + 3 * kStageRows)[lane] = wvw.mine;
        wave_lds_sync();
#pragma unroll
        for (int sub = 0; sub < kSubs; ++sub)
            patch(a.k, stage_k, wk, kfl[sub], kpos[sub], kx[sub]);

        // ---- scores of 4 rows x G heads, softmax update --------------------------------------------------
        float pw[G][kSubs];
#pragma unroll
        for (int gq = 0; gq < G; ++gq) {
            const float4_t qa = *reinterpret_cast<const float4_t *>(q_l + gq * 128 + 8 * cp);
            const float4_t qb = *reinterpret_cast<const float4_t *>(q_l + gq * 128 + 8 * cp + 4);
            float sc[kSubs];
#pragma unroll
            for (int sub = 0; sub < kSubs; ++sub) {
                const float *y = kx[sub];
                float s = qa[0] * y[0];
                s = fmaf(qa[1], y[1], s);
                s = fmaf(qa[2], y[2], s);
                s = fmaf(qa[3], y[3], s);
                s = fmaf(qb[0], y[4], s);
                s = fmaf(qb[1], y[5], s);
                s = fmaf(qb[2], y[6], s);
                s = fmaf(qb[3], y[7], s);
                s += __shfl_xor(s, 1);
                s += __shfl_xor(s, 2);
                s += __shfl_xor(s, 4);
                s += __shfl_xor(s, 8);
                sc[sub] = (4 * sub + rsub < nrows) ? s : kNegBig;
            }
            const float mn = fmaxf(fmaxf(fmaxf(sc[0], sc[1]), fmaxf(sc[2], sc[3])), m[gq]);
            const float corr = __builtin_amdgcn_exp2f(m[gq] - mn);
            float psum = 0.f;
#pragma unroll
            for (int sub = 0; sub < kSubs; ++sub) {
                const float e = __builtin_amdgcn_exp2f(sc[sub] - mn);
                pw[gq][sub] = (4 * sub + rsub < nrows) ? e : 0.f;
                psum += pw[gq][sub];
            }
            l[gq] = l[gq] * corr + psum;
#pragma unroll
            for (int i = 0; i < 8; ++i)
                acc[gq][i] *= corr;
            m[gq] = mn;
        }

        // ---- weighted values ----------------------------------------------------------------------------
#pragma unroll
        for (int sub = 0; sub < kSubs; ++sub) {
            float vx[8];
            uint32_t vfl, vpos;
            decode_pair(stage_v, sec_v, wvw.base, sub, vx, vfl, vpos);
            patch(a.v, stage_v, wvw, vfl, vpos, vx);
#pragma unroll
            for (int gq = 0; gq < G; ++gq)
#pragma unroll
                for (int i = 0; i < 8; ++i)
                    acc[gq][i] = fmaf(pw[gq][sub], vx[i], acc[gq][i]);
        }
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

// grid = B * H * G (one workgroup per query head), block = 256: wave wq folds splits wq, wq + 4, ...,
// a lane holding two of the 128 dimensions; the four waves meet in LDS.
__global__ __launch_bounds__(kAttThreads) void k_attend_merge(AttendArgs a)
{
    __shared__ float red[kAttWaves][kRedStride];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const size_t head = blockIdx.x;
    const float *ml = a.part_ml + head * a.n_splits * 2;
    const float *pa = a.part_acc + head * a.n_splits * 128;
    float m = kNegBig, l = 0.f, o[2] = {0.f, 0.f};
    for (int s = wv; s < a.n_splits; s += kAttWaves) {
        const float2 st = *reinterpret_cast<const float2 *>(ml + 2 * s);
        const float2 av = *reinterpret_cast<const float2 *>(pa + (size_t)s * 128 + 2 * lane);
        const float a2[2] = {av.x, av.y};
        merge_state(m, l, o, st.x, st.y, a2);
    }
    if (lane == 0) {
        red[wv][0] = m;
        red[wv][1] = l;
    }
    red[wv][2 + 2 * lane] = o[0];
    red[wv][2 + 2 * lane + 1] = o[1];
    __syncthreads();
    if (tid < 128) {
        float mm = kNegBig;
#pragma unroll
        for (int wq = 0; wq < kAttWaves; ++wq)
            mm = fmaxf(mm, red[wq][0]);
        float ll = 0.f, oo = 0.f;
#pragma unroll
        for (int wq = 0; wq < kAttWaves; ++wq) {
            const float c = __builtin_amdgcn_exp2f(red[wq][0] - mm);
            ll = fmaf(red[wq][1], c, ll);
            oo = fmaf(red[wq][2 + tid], c, oo);
        }
        a.out[head * 128 + tid] = (_Float16)(oo / ll);
    }
}

AttendPlan plan_attend(const Geometry &g, int G)
{
    AttendPlan p;
    const int64_t n_tiles = ((int64_t)g.T + kAttendTile - 1) / kAttendTile;
    const int64_t segs = (int64_t)g.B * g.H;
    int64_t want = (2048 + segs - 1) / segs;  // about 8 workgroups per compute unit
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
    hipLaunchKernelGGL(k_attend_merge, dim3((unsigned)(g.B * g.H * a.G)), dim3(kAttThreads), 0, stream, a);
    return hipGetLastError();
}

}  // namespace hqmq
