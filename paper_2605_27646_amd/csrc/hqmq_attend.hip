// Single-query attention straight from the packed cache (paper App. F, the fused attention
// kernel: O = softmax(Q K^T scale) V with K and V decoded inside the attention loop, handed to the
// matrix cores as fp16 tiles and never written out).  This is the generation step's shape: one
// query token per sequence, G query heads sharing each kv head.
//
// Bound by the decode arithmetic: per cached token it reads 2 * (4 w + 10) bytes plus the outlier
// payloads, where plain fp16 attention reads 512.  Shape:
//   * split-K over the sequence: workgroup (split, b * H + h) walks its rows in tiles of 64, a wave
//     takes 16 rows of a tile; the encoded rows of K and of V arrive with coalesced loads issued one
//     tile ahead and are re-distributed through LDS as in the stand-alone decode;
//   * both products run on v_mfma_f32_16x16x16_f16, and the lane-to-chunk assignment of each decode
//     is the operand layout of its product, so no value crosses lanes:
//       scores  S[row][head]  = K_hat[16 rows x 128] * Q^T : lane (row = l % 16, j = l / 16) decodes
//               chunks 4 m + j, m = 0..7, i.e. exactly the four k-values it owes to product m;
//       values  O[head][dim] += P^T[head x 16 rows] * V_hat : lane (n = l % 16, j) decodes chunks
//               n and n + 16 of rows 4 j .. 4 j + 3; a 4 x 4 (row x component) block, regrouped by
//               component with byte permutes, feeds four products whose output column n stands for
//               dimension 4 n + e (+ 64 for the upper chunk);
//     the scores of product one land as lane (head = l % 16, rows 4 j .. 4 j + 3), which is the
//     layout product two wants for P^T;
//   * online softmax in the log2 domain, fp32; the weights enter the second product as an fp16
//     pair (high part + remainder), so they carry about 22 bits; the accumulators are rescaled only
//     when a tile raises a head's running maximum;
//   * a flagged chunk takes its stored fp16 payload from the wave's window of the outlier list.
// The work per cached token does not depend on G (up to 16 heads ride in one product).
// Written out for 128-element heads (32 chunks per row); heads of 96 and 64 elements run the same code
// with 6 or 4 score products per tile and 2 (the second half empty) or 1 column groups on the value side.
#include <type_traits>

#include "hqmq_device.h"

namespace hqmq {

namespace {

constexpr int kAttThreads = 256;
constexpr int kAttWaves = kAttThreads / 64;
constexpr int kStageRows = 16;                      // rows per wave and tile
constexpr int kMaxW = 24;                           // w = w_idx + b_r <= 16 + 8
constexpr int kStageWords = kStageRows * kMaxW + 4; // + padding: a 2-word window may start at the last word
constexpr int kPaySlots = 128;                      // outlier payloads of a wave's 16 rows kept in LDS
constexpr int kSideWords = kStageWords + 3 * kStageRows + 2 * kPaySlots;  // one side (K or V) of one wave
constexpr int kLoadsPerLane = (kStageRows * kMaxW + 63) / 64;
constexpr float kNegBig = -1.0e30f;                 // "no row seen yet" (finite, so differences stay finite)
constexpr int kRedStride = 2 + 128;                 // one partial state: maximum, sum, 128 weighted values
constexpr int kAttendTargetBlocks = 512;            // two resident workgroups per compute unit
constexpr uint32_t kHalfOfMaxHalf = 0x77ffu;        // 32752 = 65504 / 2 as fp16 bits
constexpr float kWeightScale = 16384.f;             // softmax weights enter the value products times 2^14

static_assert(kAttendTile == kAttWaves * kStageRows, "tile = rows of all waves");
static_assert(kStageWords % 4 == 0 && kSideWords % 4 == 0, "16-byte LDS reads of the per-row words");

typedef uint32_t uint4v __attribute__((ext_vector_type(4)));

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
                                          uint32_t row_words, int lane)
{
#pragma unroll
    for (int j = 0; j < kLoadsPerLane; ++j)
        t.cw[j] = 0;
    t.fw = t.sg = t.ro = 0;
    if (nrows > 0) {
        const uint32_t *cw = s.codes + R0 * row_words;
        const int ncw = nrows * (int)row_words;
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

// LDS image of one side: code words [16 rows][row_words] | padding | flag words [16] | scales [16] |
// offsets [16] | payload window [64] x 8 bytes
__device__ __forceinline__ void stage_tile(const TileRegs &t, uint32_t *stage, int lane)
{
#pragma unroll
    for (int j = 0; j < kLoadsPerLane; ++j)
        stage[lane + 64 * j] = t.cw[j];
    if (lane < 4)
        stage[kStageWords - 4 + lane] = 0;
    if (lane < kStageRows) {
        stage[kStageWords + lane] = t.fw;
        stage[kStageWords + kStageRows + lane] = t.sg;
        stage[kStageWords + 2 * kStageRows + lane] = t.ro;
    }
}

__device__ __forceinline__ uint32_t pack_half2(float lo, float hi)
{
    typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
    half2_t v;
    v[0] = (_Float16)lo;
    v[1] = (_Float16)hi;
    return __builtin_bit_cast(uint32_t, v);
}

__device__ __forceinline__ float4_t mfma16(uint2 a, uint2 b, float4_t c)
{
    return __builtin_amdgcn_mfma_f32_16x16x16f16(__builtin_bit_cast(half4_t, a), __builtin_bit_cast(half4_t, b), c,
                                                 0, 0, 0);
}

}  // namespace

// grid = (n_splits, B*H), block = 256.
// dynamic LDS: prim [48][4] f32 | max(staging [4 waves][K, V][kSideWords] u32, merge buffer
//              [4 waves][G][130] f32) | secondaries of K [S][4] f32 | secondaries of V [S][4] f32
// kNc: chunks per row, 32, 24 or 16 for head dimensions 128, 96, 64 (multiples of 16 elements, so that
// the score products take whole groups of 4 chunks).  The value side always works in column groups of
// 16 chunks; chunks past the row (the upper 8 of the second group at 24) read as code 0 = zeros.
template <bool kPow2, int kNc>
__global__ __launch_bounds__(kAttThreads, 2) void k_attend_partial(Geometry g, AttendArgs a, int stage_floats)
{
    constexpr int kM = kNc / 4;          // score products per tile (16 dimensions each)
    constexpr int kU = (kNc + 15) / 16;  // column groups of 16 chunks on the value side
    constexpr int kD = 4 * kNc;
    extern __shared__ float lds[];
    float *prim = lds;
    uint32_t *stage_all = reinterpret_cast<uint32_t *>(prim + 48 * 4);
    float *sec_k = reinterpret_cast<float *>(stage_all) + stage_floats;
    float *sec_v = sec_k + 4 * g.S;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int seg = blockIdx.y, b = seg / g.H, h = seg % g.H;
    const int split = blockIdx.x;
    const int n16 = lane & 15, j4 = lane >> 4;
    const int n16_ = n16, j4_ = j4;
    const int G = a.G;
    // tokens this lane's query head (n16) may see: all of them unless the caller limits it (a query
    // token of a multi-token step sees the cache only up to its own position)
    int vis = 0x7fffffff;
    if (a.visible)
        vis = (n16 < G) ? a.visible[((size_t)b * g.H + h) * G + n16] : 0;
    const uint32_t w = g.w, w_idx = g.w_idx;
    const uint32_t row_words = kNc == 32 ? w : (uint32_t)g.row_words;
    const int row_begin = split * a.rows_per_split;
    const int row_end = min(g.T, row_begin + a.rows_per_split);

    uint32_t *stage_k = stage_all + (wv * 2 + 0) * kSideWords;
    uint32_t *stage_v = stage_all + (wv * 2 + 1) * kSideWords;

    // ---- first tile on its way while the tables are set up ----------------------------------------------
    TileRegs tk, tv;
    int nrows = min(kStageRows, row_end - (row_begin + wv * kStageRows));
    {
        const int64_t R0 = (int64_t)seg * g.T + row_begin + wv * kStageRows;
        load_tile(tk, a.k, R0, nrows, row_words, lane);
        load_tile(tv, a.v, R0, nrows, row_words, lane);
    }
    // Q^T as the B operand of the score products: lane (head n16, j4) holds q[head][16 m + 4 j4 + 0..3]
    uint2 qb[kM];
    {
        const _Float16 *qh = a.q + (((size_t)b * g.H + h) * G + min(n16, G - 1)) * kD + 4 * j4;
#pragma unroll
        for (int m = 0; m < kM; ++m) {
            const uint2 v = *reinterpret_cast<const uint2 *>(qh + 16 * m);
            qb[m] = (n16 < G) ? v : make_uint2(0u, 0u);
        }
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
    }
    __syncthreads();

    // running state of head n16 (m_run is the same in all four j4 groups; l_run holds this lane's
    // rows only and is summed over j4 at the end)
    float m_run = kNegBig, l_run = 0.f;
    // [upper chunk u][component e]: element i = head 4 j4 + i, output column n16 = dimension 64 u + 4 n16 + e
    float4_t acc[kU][4];
#pragma unroll
    for (int u = 0; u < kU; ++u)
#pragma unroll
        for (int e = 0; e < 4; ++e)
            acc[u][e] = float4_t{0.f, 0.f, 0.f, 0.f};

    const uint32_t code_mask = (1u << w) - 1u, idx_mask = (1u << w_idx) - 1u;
    const float inv_L = g.inv_L;

    // Outlier payloads of a wave's 16 rows: one contiguous window of the list, its first 128 entries
    // copied to LDS (zeros for entries beyond the list's capacity).  The first 64 are requested half
    // a tile ahead, from the tile's registers (offset of the first row, offset + count of the last);
    // the next 64 (rare) are copied when the tile is staged; a still larger window (more than a
    // quarter of the chunks flagged) sends the tile down the careful path, which reads the list.
    struct Window {
        uint32_t base, n;
        uint2 mine;  // entry `lane` of the window, on its way to LDS
    };
    auto open_window = [&](const AttendSide &s, const TileRegs &t, int nr) {
        Window wd;
        wd.base = 0;
        wd.n = 0;
        wd.mine = make_uint2(0u, 0u);
        if (nr > 0) {
            const int last_row = nr - 1;
            wd.base = (uint32_t)__builtin_amdgcn_readlane((int)t.ro, 0);
            const uint32_t ro_l = (uint32_t)__builtin_amdgcn_readlane((int)t.ro, last_row);
            const uint32_t fw_l = (uint32_t)__builtin_amdgcn_readlane((int)t.fw, last_row);
            wd.n = ro_l + __popc(fw_l) - wd.base;
            // unconditional load (a conditional one would be waited for on the spot): lanes past the
            // window or the list's capacity re-read a neighbour's entry; a wave without outliers reads
            // 8 harmless bytes of the offset array
            const bool has_pay = wd.n > 0 && (uint64_t)wd.base < s.outlier_capacity;
            const uint64_t last = has_pay ? min((uint64_t)wd.n, s.outlier_capacity - wd.base) - 1u : 0u;
            const uint2 *src = has_pay ? reinterpret_cast<const uint2 *>(s.outliers) + wd.base
                                       : reinterpret_cast<const uint2 *>(s.row_off);
            wd.mine = src[min((uint64_t)lane, last)];
            if (!has_pay || (uint64_t)lane > last)
                wd.mine = make_uint2(0u, 0u);
        }
        return wd;
    };
    auto stage_window = [&](const AttendSide &s, const Window &wd, uint32_t *stage) {
        uint2 *st_pay = reinterpret_cast<uint2 *>(stage + kStageWords + 3 * kStageRows);
        st_pay[lane] = wd.mine;
        if (wd.n > 64u) {  // wave-uniform and rare: more than 64 outliers in 16 rows
            for (uint32_t k = 64u + lane; k < min(wd.n, (uint32_t)kPaySlots); k += 64u) {
                const uint64_t at = (uint64_t)wd.base + k;
                st_pay[k] = at < s.outlier_capacity ? reinterpret_cast<const uint2 *>(s.outliers)[at]
                                                    : make_uint2(0u, 0u);
            }
        }
    };

    // One chunk of `row` as the library's decode returns it (four fp16 values, two dwords), in three
    // steps so that the LDS round trips of neighbouring chunks overlap: the code, then the table
    // entries and the payload slot it selects, then the arithmetic.
    // kFast: the wave's whole payload window sits in LDS and no scale of the tile can push a product
    // beyond the fp16 range, so there is neither a far load nor a clamp.  The choice is made per
    // tile and side.
    auto read_code = [&](const uint32_t *stage, int row, uint32_t c) {
        const uint32_t bitpos = c * w;
        const uint32_t *rw = stage + row * row_words + (bitpos >> 5);
        const uint32_t d0 = rw[0], d1 = rw[1];
        const uint32_t code = __builtin_amdgcn_alignbit(d1, d0, bitpos & 31u) & code_mask;
        // a chunk slot past the row's chunks (value side, 24 chunks per row): what was read lies inside
        // the staged words but means nothing; code 0 decodes to zeros and its flag bit is never set
        return (kNc % 16 == 0 || c < (uint32_t)kNc) ? code : 0u;
    };
    struct Fetched {
        float4_t P, q;
        uint2 pay;
        uint32_t pos;
    };
    auto fetch = [&](const uint32_t *stage, const float *secl, uint32_t base, uint32_t code, uint32_t c,
                     uint32_t word, uint32_t roff) {
        Fetched f;
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
        f.P = *reinterpret_cast<const float4_t *>(reinterpret_cast<const char *>(prim) + p_off);
        f.q = *reinterpret_cast<const float4_t *>(reinterpret_cast<const char *>(secl) + s_off);
        // list slot of this chunk if it is flagged (any in-range slot otherwise: the value is unused)
        f.pos = roff + __popc(word & ((1u << c) - 1u)) - base;
        const uint2 *st_pay = reinterpret_cast<const uint2 *>(stage + kStageWords + 3 * kStageRows);
        f.pay = st_pay[min(f.pos, (uint32_t)kPaySlots - 1u)];
        return f;
    };
    auto finish = [&](auto fast_tag, const AttendSide &s, uint32_t base, const Fetched &f, uint32_t code,
                      uint32_t c, uint32_t word, float sol, bool row_valid) {
        constexpr bool kFast = decltype(fast_tag)::value;
        const float rh = (float)(code >> w_idx) * sol;
        const float4_t P = f.P, q = f.q;
        const float R0 = rh * P[0], R1 = rh * P[1], R2 = rh * P[2], R3 = rh * P[3];
        float y0 = fmaf(-R3, q[3], fmaf(-R2, q[2], fmaf(-R1, q[1], R0 * q[0])));
        float y1 = fmaf(-R3, q[2], fmaf(R2, q[3], fmaf(R1, q[0], R0 * q[1])));
        float y2 = fmaf(R3, q[1], fmaf(R2, q[0], fmaf(-R1, q[3], R0 * q[2])));
        float y3 = fmaf(R3, q[0], fmaf(-R2, q[1], fmaf(R1, q[2], R0 * q[3])));
        if (!kFast) {
            const float lim = 65504.f;  // the decode saturates instead of overflowing to infinity
            y0 = __builtin_amdgcn_fmed3f(y0, -lim, lim);
            y1 = __builtin_amdgcn_fmed3f(y1, -lim, lim);
            y2 = __builtin_amdgcn_fmed3f(y2, -lim, lim);
            y3 = __builtin_amdgcn_fmed3f(y3, -lim, lim);
        }
        uint2 out = make_uint2(pack_half2(y0, y1), pack_half2(y2, y3));
        // flagged: the stored payload replaces the reconstruction
        const bool fl = row_valid && ((word >> c) & 1u);
        uint2 pay = f.pay;
        if (!kFast) {
            // beyond the LDS slots: straight from the list (unconditional load, index clamped into
            // the list), zeros beyond the list's capacity
            const bool any = s.outlier_capacity > 0;
            const uint2 *src = any ? reinterpret_cast<const uint2 *>(s.outliers)
                                   : reinterpret_cast<const uint2 *>(s.row_off);
            const uint64_t last = any ? s.outlier_capacity - 1u : 0u;
            const uint64_t at = (uint64_t)base + f.pos;
            const uint2 far = src[min(at, last)];
            if (f.pos >= (uint32_t)kPaySlots)
                pay = at < s.outlier_capacity ? far : make_uint2(0u, 0u);
        }
        out.x = fl ? pay.x : out.x;
        out.y = fl ? pay.y : out.y;
        return out;
    };

    Window wk = open_window(a.k, tk, nrows), wvw = open_window(a.v, tv, nrows);

    for (int t0 = row_begin; t0 < row_end; t0 += kAttendTile) {
        // ---- this tile's rows and payload windows into LDS; the next tile's rows requested -----------
        stage_tile(tk, stage_k, lane);
        stage_tile(tv, stage_v, lane);
        stage_window(a.k, wk, stage_k);
        stage_window(a.v, wvw, stage_v);
        wave_lds_sync();
        const uint32_t base_k = wk.base, base_v = wvw.base;
        // a product r_hat * c_i can leave the fp16 range only when the row's scale is within a factor
        // |c_i| < 2 of the largest half
        const bool big_k = __any(tk.sg >= kHalfOfMaxHalf) != 0, big_v = __any(tv.sg >= kHalfOfMaxHalf) != 0;
        const bool fast_k = !big_k && wk.n <= (uint32_t)kPaySlots, fast_v = !big_v && wvw.n <= (uint32_t)kPaySlots;
        const bool more = t0 + kAttendTile < row_end;
        const int tgn = t0 + kAttendTile + wv * kStageRows;
        const int nn = more ? min(kStageRows, row_end - tgn) : 0;
        if (more) {
            const int64_t R0n = (int64_t)seg * g.T + tgn;
            load_tile(tk, a.k, R0n, nn, row_words, lane);
            load_tile(tv, a.v, R0n, nn, row_words, lane);
        }

        uint2 p_hi = make_uint2(0u, 0u), p_lo = make_uint2(0u, 0u);
        if (nrows > 0) {
            // ---- scores: lane (row n16, j4) supplies chunks 4 m + j4 ------------------------------------
            float4_t sc = float4_t{0.f, 0.f, 0.f, 0.f};
            auto scores = [&](auto fast_tag) {
                // The careful form is rare: its lane indices are made opaque so that the compiler does
                // not hoist a second set of per-lane address constants out of the tile loop, which
                // would cost the common form its registers.
                int n16 = n16_, j4 = j4_;
                if (!decltype(fast_tag)::value)
                    asm volatile("" : "+v"(n16), "+v"(j4));
                const uint32_t word = stage_k[kStageWords + n16];
                const float sigma =
                    (float)__builtin_bit_cast(_Float16, (uint16_t)stage_k[kStageWords + kStageRows + n16]);
                const uint32_t roff = stage_k[kStageWords + 2 * kStageRows + n16];
                const float sol = sigma * inv_L;
                const bool valid = n16 < nrows;
                uint32_t code[kM];
#pragma unroll
                for (int m = 0; m < kM; ++m)
                    code[m] = read_code(stage_k, n16, (uint32_t)(4 * m + j4));
                Fetched cur = fetch(stage_k, sec_k, base_k, code[0], (uint32_t)j4, word, roff);
#pragma unroll
                for (int m = 0; m < kM; ++m) {
                    Fetched nxt = cur;
                    if (m + 1 < kM)
                        nxt = fetch(stage_k, sec_k, base_k, code[m + 1], (uint32_t)(4 * (m + 1) + j4), word, roff);
                    const uint2 kh = finish(fast_tag, a.k, base_k, cur, code[m], (uint32_t)(4 * m + j4), word, sol, valid);
                    sc = mfma16(kh, qb[m], sc);
                    cur = nxt;
                    __builtin_amdgcn_sched_barrier(0);  // keep the one-chunk-ahead order
                }
            };
            if (fast_k)
                scores(std::true_type{});
            else
                scores(std::false_type{});

            // ---- softmax update: lane (head n16, j4) holds the scores of rows 4 j4 + i --------------------
            float s4[4];
            float mx = kNegBig;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const bool seen = 4 * j4 + i < nrows && t0 + wv * kStageRows + 4 * j4 + i < vis;
                s4[i] = seen ? sc[i] * a.qscale : kNegBig;
                mx = fmaxf(mx, s4[i]);
            }
            mx = fmaxf(mx, __shfl_xor(mx, 16));
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            const float mn = fmaxf(m_run, mx);
            if (__any(mn > m_run)) {
                // some head's maximum rose: rescale.  The accumulators of this lane belong to heads
                // 4 j4 + i, whose factors live in lanes 4 j4 + i.
                const float corr = __builtin_amdgcn_exp2f(m_run - mn);
                l_run *= corr;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float ci = __shfl(corr, 4 * j4 + i);
#pragma unroll
                    for (int u = 0; u < kU; ++u)
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            acc[u][e][i] *= ci;
                }
                m_run = mn;
            }
            float pw[4], ph[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float e = __builtin_amdgcn_exp2f(s4[i] - m_run);
                const bool seen = 4 * j4 + i < nrows && t0 + wv * kStageRows + 4 * j4 + i < vis;
                pw[i] = seen ? e : 0.f;
                l_run += pw[i];
            }
            // P^T as the A operand of the value products, split into an fp16 pair.  The weights (<= 1)
            // are scaled by 2^14 first: unscaled, the remainder part of every weight below 1/8 and both
            // parts of a weight below 2^-14 would be fp16 subnormals, i.e. carry an absolute error of
            // 2^-25 however small the weight, which adds up over a long cache.  The accumulators hold
            // 2^14 times the weighted sums; the factor is taken out when the partial sums are written.
            {
                float ps[4];
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    ps[i] = pw[i] * kWeightScale;
                p_hi = make_uint2(pack_half2(ps[0], ps[1]), pack_half2(ps[2], ps[3]));
                const half4_t hv = __builtin_bit_cast(half4_t, p_hi);
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    ph[i] = ps[i] - (float)hv[i];
                p_lo = make_uint2(pack_half2(ph[0], ph[1]), pack_half2(ph[2], ph[3]));
            }
        }

        // ---- the next tile's payload windows (its offsets have arrived by now) ---------------------------
        if (more) {
            wk = open_window(a.k, tk, nn);
            wvw = open_window(a.v, tv, nn);
        }

        // ---- weighted values: lane (n16, j4) supplies chunks n16 and n16 + 16 of rows 4 j4 + i -----------
        if (nrows > 0) {
            auto weighted_values = [&](auto fast_tag) {
                int n16 = n16_, j4 = j4_;
                if (!decltype(fast_tag)::value)
                    asm volatile("" : "+v"(n16), "+v"(j4));
                const uint4v word4 = *reinterpret_cast<const uint4v *>(stage_v + kStageWords + 4 * j4);
                const uint4v sig4 = *reinterpret_cast<const uint4v *>(stage_v + kStageWords + kStageRows + 4 * j4);
                const uint4v roff4 =
                    *reinterpret_cast<const uint4v *>(stage_v + kStageWords + 2 * kStageRows + 4 * j4);
                uint32_t code[4 * kU];
                float sol[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    sol[i] = (float)__builtin_bit_cast(_Float16, (uint16_t)sig4[i]) * inv_L;
#pragma unroll
                    for (int u = 0; u < kU; ++u)
                        code[4 * u + i] = read_code(stage_v, 4 * j4 + i, (uint32_t)(n16 + 16 * u));
                }
                Fetched cur = fetch(stage_v, sec_v, base_v, code[0], (uint32_t)n16, word4[0], roff4[0]);
#pragma unroll
                for (int u = 0; u < kU; ++u) {
                    uint2 vh[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int at = 4 * u + i, nx = at + 1;
                        Fetched nxt = cur;
                        if (nx < 4 * kU)
                            nxt = fetch(stage_v, sec_v, base_v, code[nx], (uint32_t)(n16 + 16 * (nx >> 2)),
                                        word4[nx & 3], roff4[nx & 3]);
                        vh[i] = finish(fast_tag, a.v, base_v, cur, code[at], (uint32_t)(n16 + 16 * u), word4[i],
                                       sol[i], 4 * j4 + i < nrows);
                        cur = nxt;
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    // regroup the 4 x 4 block by component: operand e = (rows 0..3 of component e)
                    const uint32_t lo_sel = 0x05040100u, hi_sel = 0x07060302u;  // low / high halves of (b, a)
                    uint2 be[4];
                    be[0] = make_uint2(__builtin_amdgcn_perm(vh[1].x, vh[0].x, lo_sel),
                                       __builtin_amdgcn_perm(vh[3].x, vh[2].x, lo_sel));
                    be[1] = make_uint2(__builtin_amdgcn_perm(vh[1].x, vh[0].x, hi_sel),
                                       __builtin_amdgcn_perm(vh[3].x, vh[2].x, hi_sel));
                    be[2] = make_uint2(__builtin_amdgcn_perm(vh[1].y, vh[0].y, lo_sel),
                                       __builtin_amdgcn_perm(vh[3].y, vh[2].y, lo_sel));
                    be[3] = make_uint2(__builtin_amdgcn_perm(vh[1].y, vh[0].y, hi_sel),
                                       __builtin_amdgcn_perm(vh[3].y, vh[2].y, hi_sel));
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        acc[u][e] = mfma16(p_hi, be[e], acc[u][e]);
                        acc[u][e] = mfma16(p_lo, be[e], acc[u][e]);
                    }
                }
            };
            if (fast_v)
                weighted_values(std::true_type{});
            else
                weighted_values(std::false_type{});
        }
        nrows = nn;
    }

    // ---- merge: the row groups of a wave (sum of l_run over j4), then the 4 waves -----------------------
    l_run += __shfl_xor(l_run, 16);
    l_run += __shfl_xor(l_run, 32);
    __syncthreads();  // every wave is done with its staging area
    float *red = reinterpret_cast<float *>(stage_all);
    if (j4 == 0 && n16 < G) {
        red[(wv * G + n16) * kRedStride + 0] = m_run;
        red[(wv * G + n16) * kRedStride + 1] = l_run;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int head = 4 * j4 + i;
        if (head < G) {
#pragma unroll
            for (int u = 0; u < kU; ++u) {
                float *dst = red + (wv * G + head) * kRedStride + 2 + 64 * u + 4 * n16;
                *reinterpret_cast<float2 *>(dst) = make_float2(acc[u][0][i], acc[u][1][i]);
                *reinterpret_cast<float2 *>(dst + 2) = make_float2(acc[u][2][i], acc[u][3][i]);
            }
        }
    }
    __syncthreads();
    for (int idx = tid; idx < G * 128; idx += kAttThreads) {
        const int gq = idx >> 7, d = idx & 127;
        if (d >= kD)
            continue;  // dimensions past the head (the partial arrays keep a pitch of 128)
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
        a.part_acc[(head * a.n_splits + split) * 128 + d] = oo * (1.0f / kWeightScale);
        if (d == 0) {
            a.part_ml[(head * a.n_splits + split) * 2 + 0] = mm;
            a.part_ml[(head * a.n_splits + split) * 2 + 1] = ll;
        }
    }
}

// ---------------------------------------------------------------------------------------
// The same kernel with the reconstruction read from tables (paper App. E / App. F: the per-head joint table
// of codeword directions).  2T is closed under negation, so a table of the 12 primaries with a positive
// first non-zero component, 12 S entries of 16 B per side, serves all 24: K's and V's fit one compute unit's
// LDS together up to S = 256 (2 x 52 KB with a block of zeros for indices past the codebook, beside 44 KB of
// staging).  A chunk then costs the primary's entry of a 48-word look-up table (row offset and sign), one table
// read and four multiplications by the signed radius instead of two table reads, four multiplications and
// sixteen fused ones.  An entry is the product of the primary and the secondary in the decode's order of
// operations with the radius left out; scaling it afterwards rounds differently from the decode in the last
// fp32 bit, which can move an element whose exact value sits on the midpoint of two fp16 values, and nothing
// else.  One workgroup of 8 waves per compute unit (tiles of 128 rows); everything else as k_attend_partial.
// grid = (n_splits, B*H), block = 512.
// dynamic LDS: max(lut [48] u32 | table K [13 S][4] f32 | table V | staging [8 waves][K, V][kSideWords] u32,
//                  merge buffer [8 waves][G][130] f32)
// ---------------------------------------------------------------------------------------
constexpr int kJointWaves = 8;
constexpr int kJointThreads = 64 * kJointWaves;
constexpr int kJointTile = kJointWaves * kStageRows;

// Six entries of a half table: the canonical primaries 6 kGroup .. 6 kGroup + 5 (+1, +i, +j, +k, then
// (+1/2, s1/2, s2/2, s3/2) with the signs counted up in binary, - for a set bit) times the secondary q.
// dst: the entry of the first of them; entries of one primary are S apart.
template <int kGroup>
__device__ __forceinline__ void half_table_entries(float4_t q, float4_t *dst, int S)
{
#pragma unroll
    for (int j = 0; j < 6; ++j) {
        const int c = 6 * kGroup + j;
        float P[4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
            P[i] = c < 4 ? (c == i ? 1.f : 0.f) : (i == 0 ? 0.5f : ((((c - 4) >> (3 - i)) & 1) ? -0.5f : 0.5f));
        float4_t d;
        d[0] = fmaf(-P[3], q[3], fmaf(-P[2], q[2], fmaf(-P[1], q[1], P[0] * q[0])));
        d[1] = fmaf(-P[3], q[2], fmaf(P[2], q[3], fmaf(P[1], q[0], P[0] * q[1])));
        d[2] = fmaf(P[3], q[1], fmaf(P[2], q[0], fmaf(-P[1], q[3], P[0] * q[2])));
        d[3] = fmaf(P[3], q[0], fmaf(-P[2], q[1], fmaf(P[1], q[2], P[0] * q[3])));
        dst[(size_t)j * S] = d;
    }
}

template <bool kPow2, int kNc>
__global__ __launch_bounds__(kJointThreads, 1) void k_attend_joint(Geometry g, AttendArgs a, int table_floats)
{
    constexpr int kM = kNc / 4;          // score products per tile (16 dimensions each)
    constexpr int kU = (kNc + 15) / 16;  // column groups of 16 chunks on the value side
    constexpr int kD = 4 * kNc;
    extern __shared__ float lds[];
    uint32_t *lut = reinterpret_cast<uint32_t *>(lds);      // [48] byte offset of the primary's rows in a table | sign
    float *tab_k = lds + 48;                                // [13 S][4]: 12 primaries, then zeros
    float *tab_v = tab_k + table_floats;
    uint32_t *stage_all = reinterpret_cast<uint32_t *>(tab_v + table_floats);

    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int seg = blockIdx.y, b = seg / g.H, h = seg % g.H;
    const int split = blockIdx.x;
    const int n16 = lane & 15, j4 = lane >> 4;
    const int n16_ = n16, j4_ = j4;
    const int G = a.G;
    // tokens this lane's query head (n16) may see: all of them unless the caller limits it (a query
    // token of a multi-token step sees the cache only up to its own position)
    int vis = 0x7fffffff;
    if (a.visible)
        vis = (n16 < G) ? a.visible[((size_t)b * g.H + h) * G + n16] : 0;
    const uint32_t w = g.w, w_idx = g.w_idx;
    const uint32_t row_words = kNc == 32 ? w : (uint32_t)g.row_words;
    const int row_begin = split * a.rows_per_split;
    const int row_end = min(g.T, row_begin + a.rows_per_split);

    uint32_t *stage_k = stage_all + (wv * 2 + 0) * kSideWords;
    uint32_t *stage_v = stage_all + (wv * 2 + 1) * kSideWords;

    // ---- first tile on its way while the tables are set up ----------------------------------------------
    TileRegs tk, tv;
    int nrows = min(kStageRows, row_end - (row_begin + wv * kStageRows));
    {
        const int64_t R0 = (int64_t)seg * g.T + row_begin + wv * kStageRows;
        load_tile(tk, a.k, R0, nrows, row_words, lane);
        load_tile(tv, a.v, R0, nrows, row_words, lane);
    }
    // Q^T as the B operand of the score products: lane (head n16, j4) holds q[head][16 m + 4 j4 + 0..3]
    uint2 qb[kM];
    {
        const _Float16 *qh = a.q + (((size_t)b * g.H + h) * G + min(n16, G - 1)) * kD + 4 * j4;
#pragma unroll
        for (int m = 0; m < kM; ++m) {
            const uint2 v = *reinterpret_cast<const uint2 *>(qh + 16 * m);
            qb[m] = (n16 < G) ? v : make_uint2(0u, 0u);
        }
    }
    {
        // Half tables: entry (c, s) = P_c (x) q_s for the 12 primaries with a positive first non-zero component
        // (+1, +i, +j, +k and (+1/2, +-1/2, +-1/2, +-1/2)); primary p is one of them or its negative, which the
        // look-up table records as a sign to be put on the radius.
        const float *sk = a.k.sec + (size_t)h * g.S * 4, *sv = a.v.sec + (size_t)h * g.S * 4;
        for (uint32_t i = tid; i < 4u * (uint32_t)g.S; i += kJointThreads) {
            const uint32_t side_grp = (uint32_t)((float)i * g.inv_S);  // i / S: 0, 1 = K's two groups of six, 2, 3 = V's
            const uint32_t sidx = i - side_grp * (uint32_t)g.S;
            const bool is_v = side_grp >= 2;
            const float4_t q = *reinterpret_cast<const float4_t *>((is_v ? sv : sk) + 4 * sidx);
            float4_t *dst = reinterpret_cast<float4_t *>(is_v ? tab_v : tab_k) + (size_t)6 * (side_grp & 1u) * g.S + sidx;
            if (side_grp & 1u)
                half_table_entries<1>(q, dst, g.S);
            else
                half_table_entries<0>(q, dst, g.S);
        }
        for (int sidx = tid; sidx < g.S; sidx += kJointThreads) {  // a thirteenth block of zeros: for an index past the codebook
            *reinterpret_cast<float4_t *>(tab_k + 4 * (12 * g.S + sidx)) = float4_t{0.f, 0.f, 0.f, 0.f};
            *reinterpret_cast<float4_t *>(tab_v + 4 * (12 * g.S + sidx)) = float4_t{0.f, 0.f, 0.f, 0.f};
        }
        if (tid < 48) {
            const uint32_t p = tid;
            uint32_t c = 12u, neg = 0u;          // p >= 24: the block of zeros
            if (p < 8) {
                c = p >> 1;
                neg = p & 1u;
            } else if (p < 24) {
                const uint32_t b = p - 8u;       // sign bits of the four halves, first component in bit 3
                neg = b >> 3;
                c = 4u + ((neg ? ~b : b) & 7u);
            }
            lut[p] = (c * (uint32_t)g.S * 16u) | (neg << 31);
        }
    }
    __syncthreads();

    // running state of head n16 (m_run is the same in all four j4 groups; l_run holds this lane's
    // rows only and is summed over j4 at the end)
    float m_run = kNegBig, l_run = 0.f;
    // [upper chunk u][component e]: element i = head 4 j4 + i, output column n16 = dimension 64 u + 4 n16 + e
    float4_t acc[kU][4];
#pragma unroll
    for (int u = 0; u < kU; ++u)
#pragma unroll
        for (int e = 0; e < 4; ++e)
            acc[u][e] = float4_t{0.f, 0.f, 0.f, 0.f};

    const uint32_t code_mask = (1u << w) - 1u, idx_mask = (1u << w_idx) - 1u;
    const float inv_L = g.inv_L;

    // Outlier payloads of a wave's 16 rows: one contiguous window of the list, its first 128 entries
    // copied to LDS (zeros for entries beyond the list's capacity).  The first 64 are requested half
    // a tile ahead, from the tile's registers (offset of the first row, offset + count of the last);
    // the next 64 (rare) are copied when the tile is staged; a still larger window (more than a
    // quarter of the chunks flagged) sends the tile down the careful path, which reads the list.
    struct Window {
        uint32_t base, n;
        uint2 mine;  // entry `lane` of the window, on its way to LDS
    };
    auto open_window = [&](const AttendSide &s, const TileRegs &t, int nr) {
        Window wd;
        wd.base = 0;
        wd.n = 0;
        wd.mine = make_uint2(0u, 0u);
        if (nr > 0) {
            const int last_row = nr - 1;
            wd.base = (uint32_t)__builtin_amdgcn_readlane((int)t.ro, 0);
            const uint32_t ro_l = (uint32_t)__builtin_amdgcn_readlane((int)t.ro, last_row);
            const uint32_t fw_l = (uint32_t)__builtin_amdgcn_readlane((int)t.fw, last_row);
            wd.n = ro_l + __popc(fw_l) - wd.base;
            // unconditional load (a conditional one would be waited for on the spot): lanes past the
            // window or the list's capacity re-read a neighbour's entry; a wave without outliers reads
            // 8 harmless bytes of the offset array
            const bool has_pay = wd.n > 0 && (uint64_t)wd.base < s.outlier_capacity;
            const uint64_t last = has_pay ? min((uint64_t)wd.n, s.outlier_capacity - wd.base) - 1u : 0u;
            const uint2 *src = has_pay ? reinterpret_cast<const uint2 *>(s.outliers) + wd.base
                                       : reinterpret_cast<const uint2 *>(s.row_off);
            wd.mine = src[min((uint64_t)lane, last)];
            if (!has_pay || (uint64_t)lane > last)
                wd.mine = make_uint2(0u, 0u);
        }
        return wd;
    };
    auto stage_window = [&](const AttendSide &s, const Window &wd, uint32_t *stage) {
        uint2 *st_pay = reinterpret_cast<uint2 *>(stage + kStageWords + 3 * kStageRows);
        st_pay[lane] = wd.mine;
        if (wd.n > 64u) {  // wave-uniform and rare: more than 64 outliers in 16 rows
            for (uint32_t k = 64u + lane; k < min(wd.n, (uint32_t)kPaySlots); k += 64u) {
                const uint64_t at = (uint64_t)wd.base + k;
                st_pay[k] = at < s.outlier_capacity ? reinterpret_cast<const uint2 *>(s.outliers)[at]
                                                    : make_uint2(0u, 0u);
            }
        }
    };

    // One chunk of `row` as the library's decode returns it (four fp16 values, two dwords), in three
    // steps so that the LDS round trips of neighbouring chunks overlap: the code, then the table
    // entries and the payload slot it selects, then the arithmetic.
    // kFast: the wave's whole payload window sits in LDS and no scale of the tile can push a product
    // beyond the fp16 range, so there is neither a far load nor a clamp.  The choice is made per
    // tile and side.
    auto read_code = [&](const uint32_t *stage, int row, uint32_t c) {
        const uint32_t bitpos = c * w;
        const uint32_t *rw = stage + row * row_words + (bitpos >> 5);
        const uint32_t d0 = rw[0], d1 = rw[1];
        const uint32_t code = __builtin_amdgcn_alignbit(d1, d0, bitpos & 31u) & code_mask;
        // a chunk slot past the row's chunks (value side, 24 chunks per row): what was read lies inside
        // the staged words but means nothing; code 0 decodes to zeros and its flag bit is never set
        return (kNc % 16 == 0 || c < (uint32_t)kNc) ? code : 0u;
    };
    // A chunk is reconstructed in three steps so that the LDS round trips of neighbouring chunks overlap: the
    // primary's entry of the look-up table and the payload slot (pre), the table entry (fetch), the arithmetic
    // (finish).
    struct Pre {
        uint32_t lutv, s_off, pos;
        uint2 pay;
    };
    struct Fetched {
        float4_t d;
        uint32_t lutv, pos;
        uint2 pay;
    };
    auto pre = [&](const uint32_t *stage, uint32_t base, uint32_t code, uint32_t c, uint32_t word, uint32_t roff) {
        Pre f;
        uint32_t p;
        if (kPow2) {
            p = (code >> g.log2_S) & 31u;
            f.s_off = (code << 4) & (((uint32_t)g.S - 1u) << 4);
        } else {
            const uint32_t kk = code & idx_mask;
            p = (uint32_t)((float)kk * g.inv_S);  // < 48
            f.s_off = (kk - __umul24(p, (uint32_t)g.S)) << 4;
        }
        f.lutv = lut[p];
        f.pos = roff + __popc(word & ((1u << c) - 1u)) - base;
        const uint2 *st_pay = reinterpret_cast<const uint2 *>(stage + kStageWords + 3 * kStageRows);
        f.pay = st_pay[min(f.pos, (uint32_t)kPaySlots - 1u)];
        return f;
    };
    auto fetch = [&](const float *tab, const Pre &q) {
        Fetched f;
        f.d = *reinterpret_cast<const float4_t *>(reinterpret_cast<const char *>(tab) + (q.lutv & 0x7fffffffu) + q.s_off);
        f.lutv = q.lutv;
        f.pos = q.pos;
        f.pay = q.pay;
        return f;
    };
    auto finish = [&](auto fast_tag, const AttendSide &s, uint32_t base, const Fetched &f, uint32_t code,
                      uint32_t c, uint32_t word, float sol, bool row_valid) {
        constexpr bool kFast = decltype(fast_tag)::value;
        // the radius with the primary's sign
        const float rh = __uint_as_float(__float_as_uint((float)(code >> w_idx) * sol) | (f.lutv & 0x80000000u));
        float y0 = rh * f.d[0], y1 = rh * f.d[1], y2 = rh * f.d[2], y3 = rh * f.d[3];
        if (!kFast) {
            const float lim = 65504.f;  // the decode saturates instead of overflowing to infinity
            y0 = __builtin_amdgcn_fmed3f(y0, -lim, lim);
            y1 = __builtin_amdgcn_fmed3f(y1, -lim, lim);
            y2 = __builtin_amdgcn_fmed3f(y2, -lim, lim);
            y3 = __builtin_amdgcn_fmed3f(y3, -lim, lim);
        }
        uint2 out = make_uint2(pack_half2(y0, y1), pack_half2(y2, y3));
        const bool fl = row_valid && ((word >> c) & 1u);
        uint2 pay = f.pay;
        if (!kFast) {
            const bool any = s.outlier_capacity > 0;
            const uint2 *src = any ? reinterpret_cast<const uint2 *>(s.outliers)
                                   : reinterpret_cast<const uint2 *>(s.row_off);
            const uint64_t last = any ? s.outlier_capacity - 1u : 0u;
            const uint64_t at = (uint64_t)base + f.pos;
            const uint2 far = src[min(at, last)];
            if (f.pos >= (uint32_t)kPaySlots)
                pay = at < s.outlier_capacity ? far : make_uint2(0u, 0u);
        }
        out.x = fl ? pay.x : out.x;
        out.y = fl ? pay.y : out.y;
        return out;
    };

    Window wk = open_window(a.k, tk, nrows), wvw = open_window(a.v, tv, nrows);

    for (int t0 = row_begin; t0 < row_end; t0 += kJointTile) {
        // ---- this tile's rows and payload windows into LDS; the next tile's rows requested -----------
        stage_tile(tk, stage_k, lane);
        stage_tile(tv, stage_v, lane);
        stage_window(a.k, wk, stage_k);
        stage_window(a.v, wvw, stage_v);
        wave_lds_sync();
        const uint32_t base_k = wk.base, base_v = wvw.base;
        // a product r_hat * c_i can leave the fp16 range only when the row's scale is within a factor
        // |c_i| < 2 of the largest half
        const bool big_k = __any(tk.sg >= kHalfOfMaxHalf) != 0, big_v = __any(tv.sg >= kHalfOfMaxHalf) != 0;
        const bool fast_k = !big_k && wk.n <= (uint32_t)kPaySlots, fast_v = !big_v && wvw.n <= (uint32_t)kPaySlots;
        const bool more = t0 + kJointTile < row_end;
        const int tgn = t0 + kJointTile + wv * kStageRows;
        const int nn = more ? min(kStageRows, row_end - tgn) : 0;
        if (more) {
            const int64_t R0n = (int64_t)seg * g.T + tgn;
            load_tile(tk, a.k, R0n, nn, row_words, lane);
            load_tile(tv, a.v, R0n, nn, row_words, lane);
        }

        uint2 p_hi = make_uint2(0u, 0u), p_lo = make_uint2(0u, 0u);
        if (nrows > 0) {
            // ---- scores: lane (row n16, j4) supplies chunks 4 m + j4 ------------------------------------
            float4_t sc = float4_t{0.f, 0.f, 0.f, 0.f};
            auto scores = [&](auto fast_tag) {
                // The careful form is rare: its lane indices are made opaque so that the compiler does
                // not hoist a second set of per-lane address constants out of the tile loop, which
                // would cost the common form its registers.
                int n16 = n16_, j4 = j4_;
                if (!decltype(fast_tag)::value)
                    asm volatile("" : "+v"(n16), "+v"(j4));
                const uint32_t word = stage_k[kStageWords + n16];
                const float sigma =
                    (float)__builtin_bit_cast(_Float16, (uint16_t)stage_k[kStageWords + kStageRows + n16]);
                const uint32_t roff = stage_k[kStageWords + 2 * kStageRows + n16];
                const float sol = sigma * inv_L;
                const bool valid = n16 < nrows;
                uint32_t code[kM];
#pragma unroll
                for (int m = 0; m < kM; ++m)
                    code[m] = read_code(stage_k, n16, (uint32_t)(4 * m + j4));
                Pre pb = pre(stage_k, base_k, code[0], (uint32_t)j4, word, roff);
                Fetched cur = fetch(tab_k, pb);
                if (kM > 1)
                    pb = pre(stage_k, base_k, code[1], (uint32_t)(4 + j4), word, roff);
#pragma unroll
                for (int m = 0; m < kM; ++m) {
                    Fetched nxt = cur;
                    if (m + 1 < kM)
                        nxt = fetch(tab_k, pb);
                    if (m + 2 < kM)
                        pb = pre(stage_k, base_k, code[m + 2], (uint32_t)(4 * (m + 2) + j4), word, roff);
                    const uint2 kh = finish(fast_tag, a.k, base_k, cur, code[m], (uint32_t)(4 * m + j4), word, sol, valid);
                    sc = mfma16(kh, qb[m], sc);
                    cur = nxt;
                    __builtin_amdgcn_sched_barrier(0);  // keep the order of the three steps
                }
            };
            if (fast_k)
                scores(std::true_type{});
            else
                scores(std::false_type{});

            // ---- softmax update: lane (head n16, j4) holds the scores of rows 4 j4 + i --------------------
            float s4[4];
            float mx = kNegBig;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const bool seen = 4 * j4 + i < nrows && t0 + wv * kStageRows + 4 * j4 + i < vis;
                s4[i] = seen ? sc[i] * a.qscale : kNegBig;
                mx = fmaxf(mx, s4[i]);
            }
            mx = fmaxf(mx, __shfl_xor(mx, 16));
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            const float mn = fmaxf(m_run, mx);
            if (__any(mn > m_run)) {
                // some head's maximum rose: rescale.  The accumulators of this lane belong to heads
                // 4 j4 + i, whose factors live in lanes 4 j4 + i.
                const float corr = __builtin_amdgcn_exp2f(m_run - mn);
                l_run *= corr;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float ci = __shfl(corr, 4 * j4 + i);
#pragma unroll
                    for (int u = 0; u < kU; ++u)
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            acc[u][e][i] *= ci;
                }
                m_run = mn;
            }
            float pw[4], ph[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float e = __builtin_amdgcn_exp2f(s4[i] - m_run);
                const bool seen = 4 * j4 + i < nrows && t0 + wv * kStageRows + 4 * j4 + i < vis;
                pw[i] = seen ? e : 0.f;
                l_run += pw[i];
            }
            // P^T as the A operand of the value products, split into an fp16 pair.  The weights (<= 1)
            // are scaled by 2^14 first: unscaled, the remainder part of every weight below 1/8 and both
            // parts of a weight below 2^-14 would be fp16 subnormals, i.e. carry an absolute error of
            // 2^-25 however small the weight, which adds up over a long cache.  The accumulators hold
            // 2^14 times the weighted sums; the factor is taken out when the partial sums are written.
            {
                float ps[4];
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    ps[i] = pw[i] * kWeightScale;
                p_hi = make_uint2(pack_half2(ps[0], ps[1]), pack_half2(ps[2], ps[3]));
                const half4_t hv = __builtin_bit_cast(half4_t, p_hi);
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    ph[i] = ps[i] - (float)hv[i];
                p_lo = make_uint2(pack_half2(ph[0], ph[1]), pack_half2(ph[2], ph[3]));
            }
        }

        // ---- the next tile's payload windows (its offsets have arrived by now) ---------------------------
        if (more) {
            wk = open_window(a.k, tk, nn);
            wvw = open_window(a.v, tv, nn);
        }

        // ---- weighted values: lane (n16, j4) supplies chunks n16 and n16 + 16 of rows 4 j4 + i -----------
        if (nrows > 0) {
            auto weighted_values = [&](auto fast_tag) {
                int n16 = n16_, j4 = j4_;
                if (!decltype(fast_tag)::value)
                    asm volatile("" : "+v"(n16), "+v"(j4));
                const uint4v word4 = *reinterpret_cast<const uint4v *>(stage_v + kStageWords + 4 * j4);
                const uint4v sig4 = *reinterpret_cast<const uint4v *>(stage_v + kStageWords + kStageRows + 4 * j4);
                const uint4v roff4 =
                    *reinterpret_cast<const uint4v *>(stage_v + kStageWords + 2 * kStageRows + 4 * j4);
                uint32_t code[4 * kU];
                float sol[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    sol[i] = (float)__builtin_bit_cast(_Float16, (uint16_t)sig4[i]) * inv_L;
#pragma unroll
                    for (int u = 0; u < kU; ++u)
                        code[4 * u + i] = read_code(stage_v, 4 * j4 + i, (uint32_t)(n16 + 16 * u));
                }
                Pre pb = pre(stage_v, base_v, code[0], (uint32_t)n16, word4[0], roff4[0]);
                Fetched cur = fetch(tab_v, pb);
                pb = pre(stage_v, base_v, code[1], (uint32_t)n16, word4[1], roff4[1]);
#pragma unroll
                for (int u = 0; u < kU; ++u) {
                    uint2 vh[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int at = 4 * u + i, nx = at + 1, n2 = at + 2;
                        Fetched nxt = cur;
                        if (nx < 4 * kU)
                            nxt = fetch(tab_v, pb);
                        if (n2 < 4 * kU)
                            pb = pre(stage_v, base_v, code[n2], (uint32_t)(n16 + 16 * (n2 >> 2)), word4[n2 & 3], roff4[n2 & 3]);
                        vh[i] = finish(fast_tag, a.v, base_v, cur, code[at], (uint32_t)(n16 + 16 * u), word4[i],
                                       sol[i], 4 * j4 + i < nrows);
                        cur = nxt;
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    // regroup the 4 x 4 block by component: operand e = (rows 0..3 of component e)
                    const uint32_t lo_sel = 0x05040100u, hi_sel = 0x07060302u;  // low / high halves of (b, a)
                    uint2 be[4];
                    be[0] = make_uint2(__builtin_amdgcn_perm(vh[1].x, vh[0].x, lo_sel),
                                       __builtin_amdgcn_perm(vh[3].x, vh[2].x, lo_sel));
                    be[1] = make_uint2(__builtin_amdgcn_perm(vh[1].x, vh[0].x, hi_sel),
                                       __builtin_amdgcn_perm(vh[3].x, vh[2].x, hi_sel));
                    be[2] = make_uint2(__builtin_amdgcn_perm(vh[1].y, vh[0].y, lo_sel),
                                       __builtin_amdgcn_perm(vh[3].y, vh[2].y, lo_sel));
                    be[3] = make_uint2(__builtin_amdgcn_perm(vh[1].y, vh[0].y, hi_sel),
                                       __builtin_amdgcn_perm(vh[3].y, vh[2].y, hi_sel));
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        acc[u][e] = mfma16(p_hi, be[e], acc[u][e]);
                        acc[u][e] = mfma16(p_lo, be[e], acc[u][e]);
                    }
                }
            };
            if (fast_v)
                weighted_values(std::true_type{});
            else
                weighted_values(std::false_type{});
        }
        nrows = nn;
    }

    // ---- merge: the row groups of a wave (sum of l_run over j4), then the 4 waves -----------------------
    l_run += __shfl_xor(l_run, 16);
    l_run += __shfl_xor(l_run, 32);
    __syncthreads();  // every wave is done with its staging area
    float *red = lds;  // over the tables: no wave reads them any more
    if (j4 == 0 && n16 < G) {
        red[(wv * G + n16) * kRedStride + 0] = m_run;
        red[(wv * G + n16) * kRedStride + 1] = l_run;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int head = 4 * j4 + i;
        if (head < G) {
#pragma unroll
            for (int u = 0; u < kU; ++u) {
                float *dst = red + (wv * G + head) * kRedStride + 2 + 64 * u + 4 * n16;
                *reinterpret_cast<float2 *>(dst) = make_float2(acc[u][0][i], acc[u][1][i]);
                *reinterpret_cast<float2 *>(dst + 2) = make_float2(acc[u][2][i], acc[u][3][i]);
            }
        }
    }
    __syncthreads();
    for (int idx = tid; idx < G * 128; idx += kJointThreads) {
        const int gq = idx >> 7, d = idx & 127;
        if (d >= kD)
            continue;  // dimensions past the head (the partial arrays keep a pitch of 128)
        float mm = kNegBig;
#pragma unroll
        for (int wq = 0; wq < kJointWaves; ++wq)
            mm = fmaxf(mm, red[(wq * G + gq) * kRedStride]);
        float ll = 0.f, oo = 0.f;
#pragma unroll
        for (int wq = 0; wq < kJointWaves; ++wq) {
            const float *src = red + (wq * G + gq) * kRedStride;
            const float c = __builtin_amdgcn_exp2f(src[0] - mm);
            ll = fmaf(src[1], c, ll);
            oo = fmaf(src[2 + d], c, oo);
        }
        const size_t head = (size_t)seg * G + gq;  // = b * (H G) + h * G + gq
        a.part_acc[(head * a.n_splits + split) * 128 + d] = oo * (1.0f / kWeightScale);
        if (d == 0) {
            a.part_ml[(head * a.n_splits + split) * 2 + 0] = mm;
            a.part_ml[(head * a.n_splits + split) * 2 + 1] = ll;
        }
    }
}

// grid = (B * H * G, D / 16): workgroup (head, y) produces 16 of the head's D output dimensions.
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

    // the first four partial sums of this thread's dimension are requested before anything waits on the maxima
    const int i = tid % kMergeDims, j = tid / kMergeDims;
    float early[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int sp = j + u * kMergeWays;
        early[u] = sp < n ? pa[(size_t)sp * 128 + d0 + i] : 0.f;
    }
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

    float o = 0.f;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int sp = j + u * kMergeWays;
        if (sp < n)
            o = fmaf(early[u], wts[sp], o);
    }
    int s = j + 4 * kMergeWays;
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
        // a head that may see no token at all has an empty softmax: zeros
        a.out[head * a.D + d0 + tid] = lsum > 0.f ? (_Float16)(tot / lsum) : (_Float16)0.f;
    }
    // log-sum-exp of the head's scores (the running maximum is kept in the log2 domain)
    if (a.lse && blockIdx.y == 0 && tid == 0)
        a.lse[head] = lsum > 0.f ? (mx + __builtin_amdgcn_logf(lsum)) * 0.693147180559945309417f
                                 : -__builtin_inff();
}

// LDS of the table form: look-up table, the two half tables and the staging during the loop, the merge buffer
// after it.
static size_t joint_lds_bytes(const Geometry &g, int G, int *table_floats)
{
    const int tf = 13 * g.S * 4;
    if (table_floats)
        *table_floats = tf;
    const size_t loop = (48 + 2 * (size_t)tf + (size_t)kJointWaves * 2 * kSideWords) * sizeof(float);
    const size_t merge = (size_t)kJointWaves * G * kRedStride * sizeof(float);
    return loop > merge ? loop : merge;
}

// The table form pays two tables per workgroup (about a microsecond at S = 256) and runs one workgroup per compute
// unit: taken from 128 tiles of 128 rows over all (b, kv head) on, where it was measured level with or ahead of the
// other form at every shape tried (below that both are bound by launch latency).
constexpr int kJointTargetBlocks = 256;
constexpr int kJointMinTiles = 128;

AttendPlan plan_attend(const Geometry &g, int G, bool tables_always)
{
    AttendPlan p;
    const int64_t segs = (int64_t)g.B * g.H;
    const int64_t joint_tiles = ((int64_t)g.T + kJointTile - 1) / kJointTile;
    p.joint = joint_lds_bytes(g, G, nullptr) <= kLdsPerCu && (tables_always || joint_tiles * segs >= kJointMinTiles);
    const int tile = p.joint ? kJointTile : kAttendTile;
    const int64_t n_tiles = ((int64_t)g.T + tile - 1) / tile;
    int64_t want = ((p.joint ? kJointTargetBlocks : kAttendTargetBlocks) + segs - 1) / segs;
    if (want > n_tiles)
        want = n_tiles;
    if (want < 1)
        want = 1;
    const int64_t tiles_per_split = (n_tiles + want - 1) / want;
    p.rows_per_split = (int32_t)(tiles_per_split * tile);
    p.n_splits = (int32_t)((n_tiles + tiles_per_split - 1) / tiles_per_split);
    const uint64_t heads = (uint64_t)segs * G;
    p.ml_bytes = (heads * p.n_splits * 2 * sizeof(float) + 255) / 256 * 256;
    p.acc_bytes = (heads * p.n_splits * 128 * sizeof(float) + 255) / 256 * 256;
    p.total_bytes = p.ml_bytes + p.acc_bytes;
    return p;
}

// Codebooks of more than about 1300 secondaries put the two tables of a head past the 64 KiB of LDS that a
// launch gets without asking.
hipError_t prepare_attend_kernels()
{
    const void *variants[] = {
        reinterpret_cast<const void *>(&k_attend_partial<true, 32>), reinterpret_cast<const void *>(&k_attend_partial<false, 32>),
        reinterpret_cast<const void *>(&k_attend_partial<true, 24>), reinterpret_cast<const void *>(&k_attend_partial<false, 24>),
        reinterpret_cast<const void *>(&k_attend_partial<true, 16>), reinterpret_cast<const void *>(&k_attend_partial<false, 16>),
        reinterpret_cast<const void *>(&k_attend_joint<true, 32>),   reinterpret_cast<const void *>(&k_attend_joint<false, 32>),
        reinterpret_cast<const void *>(&k_attend_joint<true, 24>),   reinterpret_cast<const void *>(&k_attend_joint<false, 24>),
        reinterpret_cast<const void *>(&k_attend_joint<true, 16>),   reinterpret_cast<const void *>(&k_attend_joint<false, 16>),
    };
    hipError_t err = hipSuccess;
    for (size_t i = 0; i < sizeof(variants) / sizeof(variants[0]) && err == hipSuccess; ++i)
        err = hipFuncSetAttribute(variants[i], hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsPerCu);
    return err;
}

hipError_t launch_attend(const Geometry &g, const AttendArgs &a, hipStream_t stream)
{
    if (a.G < 1 || a.G > kMaxGroup)
        return hipErrorInvalidValue;
    dim3 grid((unsigned)a.n_splits, (unsigned)(g.B * g.H));
    const bool pow2 = (g.S & (g.S - 1)) == 0;
    if (a.joint) {
        int table_floats = 0;
        const size_t lds = joint_lds_bytes(g, a.G, &table_floats);
#define HQMQ_LAUNCH_JOINT(NC)                                                                                        \
    do {                                                                                                             \
        if (pow2)                                                                                                    \
            hipLaunchKernelGGL((k_attend_joint<true, NC>), grid, dim3(kJointThreads), lds, stream, g, a, table_floats);  \
        else                                                                                                         \
            hipLaunchKernelGGL((k_attend_joint<false, NC>), grid, dim3(kJointThreads), lds, stream, g, a, table_floats); \
    } while (0)
        if (g.D == 128)
            HQMQ_LAUNCH_JOINT(32);
        else if (g.D == 96)
            HQMQ_LAUNCH_JOINT(24);
        else if (g.D == 64)
            HQMQ_LAUNCH_JOINT(16);
        else
            return hipErrorInvalidValue;
#undef HQMQ_LAUNCH_JOINT
    } else {
        // the staging area doubles as the end-of-workgroup merge buffer
        int stage_floats = kAttWaves * 2 * kSideWords;
        if (stage_floats < kAttWaves * a.G * kRedStride)
            stage_floats = kAttWaves * a.G * kRedStride;
        stage_floats = (stage_floats + 3) / 4 * 4;
        const size_t lds = (size_t)(48 * 4 + stage_floats + 8 * g.S) * sizeof(float);
#define HQMQ_LAUNCH_ATTEND(NC)                                                                                       \
    do {                                                                                                             \
        if (pow2)                                                                                                    \
            hipLaunchKernelGGL((k_attend_partial<true, NC>), grid, dim3(kAttThreads), lds, stream, g, a, stage_floats);  \
        else                                                                                                         \
            hipLaunchKernelGGL((k_attend_partial<false, NC>), grid, dim3(kAttThreads), lds, stream, g, a, stage_floats); \
    } while (0)
        if (g.D == 128)
            HQMQ_LAUNCH_ATTEND(32);
        else if (g.D == 96)
            HQMQ_LAUNCH_ATTEND(24);
        else if (g.D == 64)
            HQMQ_LAUNCH_ATTEND(16);
        else
            return hipErrorInvalidValue;
#undef HQMQ_LAUNCH_ATTEND
    }
    hipError_t err = hipGetLastError();
    if (err != hipSuccess)
        return err;
    const size_t merge_lds = ((size_t)a.n_splits + kMergeWays * (kMergeDims + 1)) * sizeof(float);
    hipLaunchKernelGGL(k_attend_merge, dim3((unsigned)(g.B * g.H * a.G), (unsigned)(g.D / kMergeDims)), dim3(kAttThreads),
                       merge_lds, stream, a);
    return hipGetLastError();
}

}  // namespace hqmq
