// HQMQ decode (paper Alg. 1 "Decode", App. D "Decode"): x_hat = r_hat * (P_p (x) q_s) with
// r_hat = r_q * sigma / (2^b_r - 1); flagged chunks are restored verbatim from the outlier list.
//
// HBM-bound: per chunk it reads w/8 bytes of code (+ 1/8 flag, 1/16 scale, 1/8 offset) and
// writes 8 bytes of fp16.  The kernel is shaped like a streaming copy:
//   * small one-shot workgroups (4 wave64, 128 rows, ~21 KiB of LDS) launched in row order: the
//     hardware dispatcher hands the next rows to whichever CU frees up, so the set of rows in
//     flight is a compact window moving front to back through the tensor (good DRAM page
//     locality, no tail from a static partition), and 7 workgroups per CU overlap one another's
//     load latency;
//   * a wave takes 32 consecutive rows: their code words, flag words, scales and outlier offsets
//     arrive with a few fully coalesced loads and are re-distributed through LDS; every lane then
//     owns two adjacent chunks of a row, i.e. one 16-byte store per lane and 1 KiB contiguous per
//     wave store (rows of 128 elements: 16 such pairs per row, 4 rows per wave store, 8 stores in two
//     rounds of 4; rows of 96 elements have 12 pairs and the wave's 32 rows take two rounds of 3 stores;
//     rows of 64 elements have 8 pairs and 4 stores in one round).  The kernel is close to VALU-bound as
//     well as HBM-bound (counters: the vector ALUs are busy for 85 % of it), so the wave's fixed work -
//     address set-up, staging, barrier, payload window - is spread over as many rows as the register
//     budget of one round allows;
//   * the head's S secondaries (S*16 bytes) and the 24 primaries sit in LDS; the Hamilton product
//     is taken per chunk (16 FMA), which keeps the workgroup small enough to be one-shot;
//   * the outlier payloads of a wave's rows are one contiguous window of the list: requested with
//     one coalesced load as soon as the offsets are known and parked in LDS for the flagged lanes.
#include "hqmq_device.h"

namespace hqmq {

namespace {

constexpr int kDecThreads = 256;
constexpr int kDecWaves = kDecThreads / 64;
constexpr int kPaySlots = 128;                      // outlier payloads of a wave's rows kept in LDS (two per lane)
constexpr int kGeneralRows = 64;                    // rows per workgroup of the general-row kernel

// Sizes of one variant of the tuned kernel: kPairs chunk pairs per row, kRowsW rows per wave.
template <int kPairs, int kRowsW>
struct DecodeShape {
    static constexpr int kRows = kRowsW * kDecWaves;                 // rows per workgroup
    // code words of a row at most: 2 kPairs chunks of w <= 24 bits (w_idx <= 16, b_r <= 8)
    static constexpr int kMaxRowWords = (2 * kPairs * 24 + 31) / 32;
    static constexpr int kLoadsPerLane = (kRowsW * kMaxRowWords + 63) / 64;  // code words per lane
    // every lane parks all its words: whole multiples of 64, + 2 words of padding for the 3-word window
    static constexpr int kStageWords = 64 * kLoadsPerLane + 2;
    static constexpr int kStagePerWave = kStageWords + 3 * kRowsW + 2 * kPaySlots;
    static constexpr int kSubs = kRowsW * kPairs / 64;               // stores of 64 lanes x 16 bytes per wave
    static_assert((kRowsW * kPairs) % 64 == 0, "a wave's rows must fill whole 64-lane stores");
    static_assert(kRowsW <= 64, "one lane per row for the flag word, scale and offset");
};

}  // namespace

// grid = (ceil(T / rows per workgroup), B*H, tensors), block = 256.
// dynamic LDS: prim [48][4] f32 | staging [4 waves][kStagePerWave] u32 | secl [S][4] f32
// (the tables with compile-time sizes first, so that their LDS addresses are immediates)
// blockIdx.z selects the tensor of a batch (all of one shape); the descriptors travel as kernel
// arguments, so a batch needs no device-side table.
// kPairs: chunk pairs (8 elements) per row: 16, 12 or 8 for D = 128, 96, 64; kStageRows: rows per wave (32);
// kGroup: stores of 64 lanes x 16 bytes per round.
template <bool kPow2, int kPairs, int kStageRows, int kGroup>
__global__ __launch_bounds__(kDecThreads) void k_decode(Geometry g, DecodeBatch batch)
{
    typedef DecodeShape<kPairs, kStageRows> Shape;
    constexpr int kSubs = Shape::kSubs, kDecRows = Shape::kRows, kStageWords = Shape::kStageWords;
    constexpr int kStagePerWave = Shape::kStagePerWave, kLoadsPerLane = Shape::kLoadsPerLane;
    const DecodeTensor &dt = batch.t[blockIdx.z];
    EncodedPtrs enc;
    enc.codes = dt.codes;
    enc.sigma = dt.sigma;
    enc.flags = dt.flags;
    enc.row_off = dt.row_off;
    enc.outliers = dt.outliers;
    const uint64_t outlier_capacity = dt.outlier_capacity;
    const float *__restrict__ sec = dt.sec;
    _Float16 *__restrict__ out = dt.out;

    extern __shared__ float lds[];
    float *prim = lds;
    uint32_t *stage_all = reinterpret_cast<uint32_t *>(prim + 48 * 4);
    float *secl = reinterpret_cast<float *>(stage_all + kDecWaves * kStagePerWave);

    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform, and known to be: row
    // addresses become scalar bases with per-lane offsets
    const int seg = blockIdx.y, b = seg / g.H, h = seg % g.H;
    const int tg = blockIdx.x * kDecRows + wv * kStageRows;  // first row of this wave
    const int nrows = min(kStageRows, g.T - tg);              // <= 0: nothing to do for this wave
    const int64_t R0 = (int64_t)seg * g.T + tg;
    const uint32_t w = g.w, w_idx = g.w_idx;
    const uint32_t rw_words = kPairs == 16 ? w : (uint32_t)g.row_words;  // code words per row

    // ---- the wave's encoded rows: coalesced loads, in flight while the tables are set up --------
    uint32_t cwreg[kLoadsPerLane];
    uint32_t fw = 0, sg = 0, ro = 0;
#pragma unroll
    for (int j = 0; j < kLoadsPerLane; ++j)
        cwreg[j] = 0;
    if (nrows > 0) {
        const uint32_t *cw = enc.codes + R0 * rw_words;
        const int ncw = nrows * (int)rw_words;
#pragma unroll
        for (int j = 0; j < kLoadsPerLane; ++j)
            if (lane + 64 * j < ncw)
                cwreg[j] = cw[lane + 64 * j];
        if (lane < nrows) {
            fw = enc.flags[R0 + lane];
            sg = enc.sigma[R0 + lane];
            ro = enc.row_off[R0 + lane];
        }
    }

    // ---- tables: the head's secondaries and the 24 primaries (zero rows up to 47: a code can
    // hold p up to 47, k < 2^w_idx < 48 S; encode never produces p > 23) -------------------------
    const float *sec_h = sec + (size_t)h * g.S * 4;
    for (int s = tid; s < g.S; s += kDecThreads)
        *reinterpret_cast<float4_t *>(secl + 4 * s) = *reinterpret_cast<const float4_t *>(sec_h + 4 * s);
    if (tid < 48 * 4) {
        const int p = tid >> 2, i = tid & 3;
        float v = 0.f;
        if (p < 8)
            v = ((p >> 1) == i) ? ((p & 1) ? -1.f : 1.f) : 0.f;
        else if (p < 24)
            v = (((p - 8) >> (3 - i)) & 1) ? -0.5f : 0.5f;
        prim[tid] = v;
    }

    uint32_t *stage = stage_all + wv * kStagePerWave;
    uint32_t *st_flags = stage + kStageWords;
    uint32_t *st_sigma = st_flags + kStageRows;
    uint32_t *st_roff = st_sigma + kStageRows;
#pragma unroll
    for (int j = 0; j < kLoadsPerLane; ++j)
        stage[lane + 64 * j] = cwreg[j];
    if (lane < 2)
        stage[kStageWords - 2 + lane] = 0;  // padding read by the last row's 3-word window
    if (lane < kStageRows) {
        st_flags[lane] = fw;
        st_sigma[lane] = sg;
        st_roff[lane] = ro;
    }
    __syncthreads();
    if (nrows <= 0)
        return;

    // ---- outlier payloads of the wave's rows: one contiguous window of the list, requested now
    // (its offsets have just arrived) and consumed after the arithmetic below --------------------
    uint2 *st_pay = reinterpret_cast<uint2 *>(st_roff + kStageRows);
    const uint32_t pay_base = st_roff[0];
    const uint32_t pay_n = st_roff[nrows - 1] + __popc(st_flags[nrows - 1]) - pay_base;  // wave-uniform
    // The load is unconditional (a conditional one would be waited for on the spot): lanes past the
    // window, or beyond the list's capacity, re-read a neighbour's entry, and a wave without
    // outliers reads 8 harmless bytes of the offset array instead of a possibly absent list.
    const bool has_pay = pay_n > 0 && (uint64_t)pay_base < outlier_capacity;
    const uint64_t pay_last = has_pay ? min((uint64_t)pay_n, outlier_capacity - pay_base) - 1u : 0u;
    const uint2 *pay_src = has_pay ? reinterpret_cast<const uint2 *>(enc.outliers) + pay_base
                                   : reinterpret_cast<const uint2 *>(enc.row_off);
    const uint2 pay_mine = pay_src[min((uint64_t)lane, pay_last)];
    const uint2 pay_mine2 = pay_src[min((uint64_t)lane + 64u, pay_last)];
    // wave-uniform: the whole window fits the LDS slots and the list's capacity
    const bool window_ok = pay_n <= (uint32_t)kPaySlots && (uint64_t)pay_base + pay_n <= outlier_capacity;

    const uint32_t code_mask = (1u << w) - 1u, idx_mask = (1u << w_idx) - 1u;
    const float inv_L = g.inv_L;
    _Float16 *obase = out + (int64_t)b * g.sb + (int64_t)h * g.sh + (int64_t)tg * g.st;

    // ---- phase 1: codes and flags of the lane's 8 chunks ----------------------------------------------
    struct Sub {
        uint32_t code0, code1, fl, pos;
        float sigma;
    };
    // pair slot 64 sub + lane of the wave: row r of the 16, chunk pair cp of the row (compile-time
    // divisor; for 16 pairs per row r = 4 sub + lane / 16 and cp = lane % 16 for every sub)
    auto row_of = [&](int sub) { return (int)((64u * (uint32_t)sub + (uint32_t)lane) / (uint32_t)kPairs); };
    auto pair_of = [&](int sub) { return (int)((64u * (uint32_t)sub + (uint32_t)lane) % (uint32_t)kPairs); };
    auto phase1 = [&](int sub) {
        Sub o;
        const int r = row_of(sub), cp = pair_of(sub);
        const uint32_t bitpos = (uint32_t)(2 * cp) * w;
        const uint32_t i0 = bitpos >> 5, sh0 = bitpos & 31;
        const uint32_t sh1 = sh0 + w;  // second chunk, relative to word i0 (may exceed 32)
        const bool second_in_low = sh1 < 32;
        const uint32_t *rw = stage + r * rw_words + i0;
        const uint32_t d0 = rw[0], d1 = rw[1], d2 = rw[2];
        const uint32_t word = st_flags[r];
        o.sigma = (float)__builtin_bit_cast(_Float16, (uint16_t)st_sigma[r]);
        o.code0 = __builtin_amdgcn_alignbit(d1, d0, sh0) & code_mask;
        // second chunk: starts sh1 = sh0 + w bits into word i0; the funnel shift takes its amount
        // modulo 32, so the same amount serves both windows and the choice is a plain select
        const uint32_t lo_win = __builtin_amdgcn_alignbit(d1, d0, sh1);
        const uint32_t hi_win = __builtin_amdgcn_alignbit(d2, d1, sh1);
        o.code1 = (second_in_low ? lo_win : hi_win) & code_mask;
        o.fl = (r < nrows) ? ((word >> (2 * cp)) & 3u) : 0u;
        o.pos = st_roff[r] + __popc(word & ((1u << (2 * cp)) - 1u)) - pay_base;  // slot of the first flagged
        return o;
    };
    auto decode_chunk = [&](uint32_t code, float sol) {
        const uint32_t rq = code >> w_idx;
        uint32_t p_off, s_off;  // byte offsets of P_p and q_s in their LDS tables
        if (kPow2) {
            // code = r_q : p : s as bit fields; p has 5 bits (24 S <= 2^w_idx < 48 S); one bit-field
            // extract each, so that the shift by 4 fuses with the table's base address
            p_off = __builtin_amdgcn_ubfe(code, (uint32_t)g.log2_S, 5u) << 4;
            s_off = __builtin_amdgcn_ubfe(code, 0u, (uint32_t)g.log2_S) << 4;
        } else {
            // p = k / S by a biased reciprocal, exact for k < 48 S (see Geometry::inv_S)
            const uint32_t k = code & idx_mask;
            const uint32_t p = (uint32_t)((float)k * g.inv_S);
            p_off = p << 4;
            s_off = (k - __umul24(p, (uint32_t)g.S)) << 4;
        }
        const float4_t P = *reinterpret_cast<const float4_t *>(reinterpret_cast<const char *>(prim) + p_off);
        const float4_t q = *reinterpret_cast<const float4_t *>(reinterpret_cast<const char *>(secl) + s_off);
        const float rh = (float)rq * sol;
        const float R0 = rh * P[0], R1 = rh * P[1], R2 = rh * P[2], R3 = rh * P[3];
        // Hamilton product (r_hat P) (x) q
        float4_t y;
        y[0] = fmaf(-R3, q[3], fmaf(-R2, q[2], fmaf(-R1, q[1], R0 * q[0])));
        y[1] = fmaf(-R3, q[2], fmaf(R2, q[3], fmaf(R1, q[0], R0 * q[1])));
        y[2] = fmaf(R3, q[1], fmaf(R2, q[0], fmaf(-R1, q[3], R0 * q[2])));
        y[3] = fmaf(R3, q[0], fmaf(-R2, q[1], fmaf(R1, q[2], R0 * q[3])));
        return y;
    };
    auto to_half4 = [&](float4_t y) {
        half4_t hv;
        hv[0] = (_Float16)y[0];
        hv[1] = (_Float16)y[1];
        hv[2] = (_Float16)y[2];
        hv[3] = (_Float16)y[3];
        return __builtin_bit_cast(uint2, hv);
    };
    // payload of list slot `slot` of this wave's window (LDS), or straight from memory beyond it
    auto fetch_payload = [&](uint32_t slot) {
        uint2 v = make_uint2(0u, 0u);
        if (slot < (uint32_t)kPaySlots) {
            if ((uint64_t)pay_base + slot < outlier_capacity)
                v = st_pay[slot];
        } else {
            const uint64_t pos = (uint64_t)pay_base + slot;
            if (pos < outlier_capacity)
                v = *reinterpret_cast<const uint2 *>(enc.outliers + 4 * pos);
        }
        return v;
    };
    // ---- phase 2: decode every chunk (all arithmetic, while the payload window is still in flight) ----
    auto phase2 = [&](const Sub &in) {
        const float sol = in.sigma * inv_L;
        float4_t ya = decode_chunk(in.code0, sol), yb = decode_chunk(in.code1, sol);
        // A product r_hat * c_i can only leave the fp16 range when the row's scale is within a
        // factor |c_i| of the largest half; |c_i| <= |q_s| < 2 for any codebook of (near) unit
        // quaternions, so only such rows take the saturating conversion.
        if (in.sigma >= 32752.f) {
            const float lim = 65504.f;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                ya[i] = __builtin_amdgcn_fmed3f(ya[i], -lim, lim);
                yb[i] = __builtin_amdgcn_fmed3f(yb[i], -lim, lim);
            }
        }
        const uint2 oa = to_half4(ya), ob = to_half4(yb);
        return make_uint4(oa.x, oa.y, ob.x, ob.y);
    };
    // ---- phase 3: flagged chunks take their payload; store ---------------------------------------------
    auto phase3 = [&](int sub, const Sub &in, uint4 o) {
        const int r = row_of(sub), cp = pair_of(sub);
        if (window_ok) {
            // every flagged chunk of the wave has its payload in the LDS window: read and select
            // without branching (unflagged lanes read a clamped slot and discard it)
            const uint32_t slot_b = in.pos + (in.fl & 1u);
            const uint2 pa = st_pay[min(in.pos, (uint32_t)kPaySlots - 1u)];
            const uint2 pb = st_pay[min(slot_b, (uint32_t)kPaySlots - 1u)];
            if (in.fl & 1u) {
                o.x = pa.x;
                o.y = pa.y;
            }
            if (in.fl & 2u) {
                o.z = pb.x;
                o.w = pb.y;
            }
        } else if (in.fl) {
            uint32_t slot = in.pos;
            if (in.fl & 1u) {
                const uint2 v = fetch_payload(slot);
                o.x = v.x;
                o.y = v.y;
                ++slot;
            }
            if (in.fl & 2u) {
                const uint2 v = fetch_payload(slot);
                o.z = v.x;
                o.w = v.y;
            }
        }
        if (r < nrows) {
            typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
            const u32x4 ov = {o.x, o.y, o.z, o.w};
            __builtin_nontemporal_store(ov, reinterpret_cast<u32x4 *>(obase + (int64_t)r * g.st + 8 * cp));
        }
    };
    // Rounds of kGroup stores each, kept apart (the scheduling barrier) so that the registers of one round
    // serve the next: the wave's fixed work - loads, staging, barrier, payload window - is spread over
    // twice the rows of a single round at the register count of one.
#pragma unroll
    for (int g0 = 0; g0 < kSubs; g0 += kGroup) {
        Sub sv[kGroup];
        uint4 ov[kGroup];
#pragma unroll
        for (int i = 0; i < kGroup; ++i)
            if (g0 + i < kSubs)
                sv[i] = phase1(g0 + i);
#pragma unroll
        for (int i = 0; i < kGroup; ++i)
            if (g0 + i < kSubs)
                ov[i] = phase2(sv[i]);
        if (g0 == 0) {
            // the window lands in LDS only now, after the first round's arithmetic, which does not need it
            st_pay[lane] = pay_mine;
            st_pay[lane + 64] = pay_mine2;
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        }
#pragma unroll
        for (int i = 0; i < kGroup; ++i)
            if (g0 + i < kSubs)
                phase3(g0 + i, sv[i], ov[i]);
        __builtin_amdgcn_sched_barrier(0);
    }
}

// Decode for head dimensions other than 128 (rows of n_c = ceil(D / 4) <= 32 chunks, ceil(n_c w / 32)
// code words each): the plain mapping, one lane per chunk slot, a 32-lane slot per row, the lanes
// past the row's chunks idle.  Same arithmetic as k_decode; the elements of a last partial chunk that
// lie past D are not written (the truncation of the paper's App. "Padding wrapper for d_h not
// divisible by 4").
// grid = (ceil(T / 64), B*H, tensors), block = 256: 8 rows per pass, 8 passes.
// dynamic LDS: prim [48][4] f32 | secl [S][4] f32
template <bool kPow2>
__global__ __launch_bounds__(kDecThreads) void k_decode_rows(Geometry g, DecodeBatch batch)
{
    const DecodeTensor &dt = batch.t[blockIdx.z];
    const uint64_t outlier_capacity = dt.outlier_capacity;
    _Float16 *__restrict__ out = dt.out;

    extern __shared__ float lds[];
    float *prim = lds;
    float *secl = prim + 48 * 4;

    const int tid = threadIdx.x;
    const int seg = blockIdx.y, b = seg / g.H, h = seg % g.H;
    const float *sec_h = dt.sec + (size_t)h * g.S * 4;
    for (int s = tid; s < g.S; s += kDecThreads)
        *reinterpret_cast<float4_t *>(secl + 4 * s) = *reinterpret_cast<const float4_t *>(sec_h + 4 * s);
    if (tid < 48 * 4) {
        const int p = tid >> 2, i = tid & 3;
        float v = 0.f;
        if (p < 8)
            v = ((p >> 1) == i) ? ((p & 1) ? -1.f : 1.f) : 0.f;
        else if (p < 24)
            v = (((p - 8) >> (3 - i)) & 1) ? -0.5f : 0.5f;
        prim[tid] = v;
    }
    __syncthreads();

    const int c = tid & 31, rsub = tid >> 5;
    if (c >= g.n_c)
        return;
    const uint32_t w = g.w, w_idx = g.w_idx;
    const uint32_t bitpos = (uint32_t)c * w, i0 = bitpos >> 5, sh = bitpos & 31;
    const uint32_t code_mask = (1u << w) - 1u, idx_mask = (1u << w_idx) - 1u;
    for (int pass = 0; pass < kGeneralRows / 8; ++pass) {
        const int t = blockIdx.x * kGeneralRows + pass * 8 + rsub;
        if (t >= g.T)
            break;  // later passes lie further past the end
        const int64_t R = (int64_t)seg * g.T + t;
        const uint32_t *words = dt.codes + R * g.row_words;
        const uint32_t d0 = words[i0];
        const uint32_t d1 = (i0 + 1 < (uint32_t)g.row_words) ? words[i0 + 1] : 0u;
        const uint32_t code = __builtin_amdgcn_alignbit(d1, d0, sh) & code_mask;
        const uint32_t word = dt.flags[R];
        half4_t hv;
        if ((word >> c) & 1u) {
            const uint64_t pos = (uint64_t)dt.row_off[R] + __popc(word & ((1u << c) - 1u));
            uint2 v = make_uint2(0u, 0u);
            if (pos < outlier_capacity)
                v = *reinterpret_cast<const uint2 *>(dt.outliers + 4 * pos);
            hv = __builtin_bit_cast(half4_t, v);
        } else {
            const float sigma = (float)__builtin_bit_cast(_Float16, dt.sigma[R]);
            const uint32_t rq = code >> w_idx;
            uint32_t p, sidx;
            if (kPow2) {
                p = (code >> g.log2_S) & 31u;
                sidx = code & ((uint32_t)g.S - 1u);
            } else {
                const uint32_t k = code & idx_mask;
                p = (uint32_t)((float)k * g.inv_S);  // k / S, exact for k < 48 S (see Geometry::inv_S)
                sidx = k - __umul24(p, (uint32_t)g.S);
            }
            const float4_t P = *reinterpret_cast<const float4_t *>(prim + 4 * p);
            const float4_t q = *reinterpret_cast<const float4_t *>(secl + 4 * sidx);
            const float rh = (float)rq * (sigma * g.inv_L);
            const float R0 = rh * P[0], R1 = rh * P[1], R2 = rh * P[2], R3 = rh * P[3];
            float4_t y;  // Hamilton product (r_hat P) (x) q
            y[0] = fmaf(-R3, q[3], fmaf(-R2, q[2], fmaf(-R1, q[1], R0 * q[0])));
            y[1] = fmaf(-R3, q[2], fmaf(R2, q[3], fmaf(R1, q[0], R0 * q[1])));
            y[2] = fmaf(R3, q[1], fmaf(R2, q[0], fmaf(-R1, q[3], R0 * q[2])));
            y[3] = fmaf(R3, q[0], fmaf(-R2, q[1], fmaf(R1, q[2], R0 * q[3])));
            if (sigma >= 32752.f) {  // only such rows can leave the fp16 range: saturate
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    y[i] = __builtin_amdgcn_fmed3f(y[i], -65504.f, 65504.f);
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
                hv[i] = (_Float16)y[i];
        }
        _Float16 *dst = out + (int64_t)b * g.sb + (int64_t)h * g.sh + (int64_t)t * g.st + 4 * c;
        if (g.vec_ok) {
            *reinterpret_cast<uint2 *>(dst) = __builtin_bit_cast(uint2, hv);
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (4 * c + e < g.D)
                    dst[e] = hv[e];
        }
    }
}

template <int kPairs, int kRowsW, int kGroup>
static void launch_tuned(const Geometry &g, const DecodeBatch &batch, int n_tensors, hipStream_t stream)
{
    typedef DecodeShape<kPairs, kRowsW> Shape;
    const size_t lds = ((size_t)g.S * 4 + 48 * 4) * sizeof(float) + (size_t)kDecWaves * Shape::kStagePerWave * 4;
    dim3 grid((unsigned)((g.T + Shape::kRows - 1) / Shape::kRows), (unsigned)(g.B * g.H), (unsigned)n_tensors);
    if ((g.S & (g.S - 1)) == 0)
        hipLaunchKernelGGL((k_decode<true, kPairs, kRowsW, kGroup>), grid, dim3(kDecThreads), lds, stream, g, batch);
    else
        hipLaunchKernelGGL((k_decode<false, kPairs, kRowsW, kGroup>), grid, dim3(kDecThreads), lds, stream, g, batch);
}

hipError_t launch_decode(const Geometry &g, const DecodeBatch &batch, int n_tensors, hipStream_t stream)
{
    // rows of 128, 96 or 64 elements whose strides keep every 16-byte store aligned take the tuned kernel
    const bool aligned16 = g.sb % 8 == 0 && g.sh % 8 == 0 && g.st % 8 == 0;
    if (g.D == 4 * kChunksPerRow) {
        launch_tuned<16, 32, 4>(g, batch, n_tensors, stream);  // two rounds of 4 stores (one: 6-10 % slower; three, four: slower)
    } else if (aligned16 && g.D == 96) {
        launch_tuned<12, 32, 3>(g, batch, n_tensors, stream);  // two rounds of 3 stores (one round of 16 rows: 13 % slower)
    } else if (aligned16 && g.D == 64) {
        launch_tuned<8, 32, 4>(g, batch, n_tensors, stream);   // one round of 4 stores (64 rows in two rounds: 9 % slower)
    } else {
        const size_t lds_rows = ((size_t)g.S * 4 + 48 * 4) * sizeof(float);
        dim3 grid((unsigned)((g.T + kGeneralRows - 1) / kGeneralRows), (unsigned)(g.B * g.H), (unsigned)n_tensors);
        if ((g.S & (g.S - 1)) == 0)
            hipLaunchKernelGGL(k_decode_rows<true>, grid, dim3(kDecThreads), lds_rows, stream, g, batch);
        else
            hipLaunchKernelGGL(k_decode_rows<false>, grid, dim3(kDecThreads), lds_rows, stream, g, batch);
    }
    return hipGetLastError();
}

}  // namespace hqmq
