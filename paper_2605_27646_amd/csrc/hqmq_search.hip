// HQMQ encode, second half: outlier flags, per-row scale, nearest-codeword search, radius code and
// bit packing (paper Alg. 1 "Encode", App. D "Encode").
//
// Search formulation.  The score of codeword (p, s) is <u, P_p q_s>.  Right multiplication by
// conj(q_s) is an isometry of R^4 up to the common factor |q_s|^2, so
//     <u, P_p q_s> = <u conj(q_s), P_p>,
// and for a fixed s the best primary is the 24-cell vertex nearest to v = u conj(q_s):
//     max_p <v, P_p> = max( max_i |v_i| , (|v_0|+|v_1|+|v_2|+|v_3|)/2 )
// (first term: the 8 axis elements +-1, +-i, +-j, +-k; second: the 16 half-integer elements).
// The map u -> v is linear, v = A(q_s) u with a 4x4 matrix per secondary, so all S products of
// 32 chunks are one [4S x 4] x [4 x 32] contraction with K = 4 on the matrix cores (how it is fed
// to them is described at the kernel).  One MFMA gives every lane the four components of v for
// four (chunk, secondary) pairs; the closed form and the running argmax over s are a handful of
// VALU instructions per pair.  The search stays exhaustive over all S secondaries and, through
// the closed form, over all 24 primaries.
//
// The kernel is bound by VALU issue: with four waves on a SIMD the matrix products run behind the other
// waves' vector work (counters: the VALU is busy for the whole kernel, the MFMA pipe for a quarter of it),
// so the VALU count per (chunk, secondary) pair is what is minimised: the running argmax
// is kept per group of 16 secondaries (8 per lane) with v_max3 chains, one compare-and-select per
// group, and the winner inside the winning group is found afterwards by re-scoring its candidates.
//
// The matrix pass is a screen, not the decision.  It runs on v_mfma_f32_32x32x16_f16 with every fp32
// factor split into two fp16 parts (24 bits), i.e. four products per term, half of what a
// three-part split costs on the matrix cores and a quarter of the fp32 shape's time.  A screened score is
// within 7e-7 of the true one.  Next to its best group every lane keeps the runner-up score; a chunk whose
// winning group is not ahead of every other group by 6e-6 of its score is searched again over all S secondaries with
// plain fp32 arithmetic.  Either way the choice between secondaries is made on fp32 closed-form scores.
//
// Work split: a workgroup (4, 8 or 16 wave64) owns 64, 256 or 512 rows of one (b, h) segment, so the A
// matrices of the head sit in LDS once per workgroup.  A wave takes 64 chunks, one per lane, at a
// time and runs them as two 32-chunk MFMA column groups: two whole rows of 128 elements in
// k_search, 64 consecutive chunks of the workgroup's flattened rows in k_search_flat (any other
// head dimension).  The per-chunk steps (scale, radius code, direction search) are shared.
#include "hqmq_device.h"

namespace hqmq {

namespace {

__device__ __forceinline__ void wave_lds_sync()
{
    // LDS serves the instructions of one wave in order; this only stops the compiler from moving
    // LDS accesses of other lanes' data across the point.
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__device__ __forceinline__ uint16_t double_to_half_rne_sat(double v)
{
    // v >= 0 and finite.  Round to nearest even from the full 53-bit significand (no double
    // rounding through fp32), saturate at 65504.
    if (!(v < 65504.0))
        return 0x7bff;
    unsigned long long bits = (unsigned long long)__double_as_longlong(v);
    int e = (int)(bits >> 52) - 1023;
    if (e < -40)
        return 0;  // far below half of the smallest subnormal 2^-24
    unsigned long long m = (bits & 0x000fffffffffffffull) | 0x0010000000000000ull;
    int E = e < -14 ? -14 : e;
    int sh = 42 + (E - e);  // 42 .. 68
    if (sh > 63)
        return 0;
    unsigned long long q = m >> sh;
    unsigned long long rem = m & ((1ull << sh) - 1ull);
    unsigned long long half = 1ull << (sh - 1);
    if (rem > half || (rem == half && (q & 1ull)))
        ++q;
    uint32_t out = ((uint32_t)(E + 14) << 10) + (uint32_t)q;
    return out > 0x7bff ? (uint16_t)0x7bff : (uint16_t)out;
}

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
constexpr float kOperandScale = 1024.f;

__device__ __forceinline__ uint32_t pack2(_Float16 lo, _Float16 hi)
{
    typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
    const half2_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, v);
}

template <int kCtrl>
__device__ __forceinline__ unsigned long long dpp_move64(unsigned long long v)
{
    const int lo = __builtin_amdgcn_update_dpp(0, (int)(uint32_t)v, kCtrl, 0xf, 0xf, true);
    const int hi = __builtin_amdgcn_update_dpp(0, (int)(uint32_t)(v >> 32), kCtrl, 0xf, 0xf, true);
    return ((unsigned long long)(uint32_t)hi << 32) | (uint32_t)lo;
}

template <int kCtrl>
__device__ __forceinline__ double dpp_move_f64(double v)
{
    return __longlong_as_double((long long)dpp_move64<kCtrl>((unsigned long long)__double_as_longlong(v)));
}

__device__ __forceinline__ unsigned long long umax64(unsigned long long a, unsigned long long b)
{
    return a > b ? a : b;
}

__device__ __forceinline__ double half_bits_to_double(uint16_t h)
{
    return (double)(float)__builtin_bit_cast(_Float16, h);
}

// Nearest 24-cell vertex to v in the order of the primary table: p = 0..7 are +1, -1, +i, -i,
// +j, -j, +k, -k, p = 8 + 8 b0 + 4 b1 + 2 b2 + b3 is ((-1)^b0, (-1)^b1, (-1)^b2, (-1)^b3)/2.
// Exact ties go to the lowest p.
__device__ __forceinline__ int nearest_primary(float v0, float v1, float v2, float v3, float &score)
{
    float a0 = fabsf(v0), a1 = fabsf(v1), a2 = fabsf(v2), a3 = fabsf(v3);
    float ax = a0;
    int pi = (v0 < 0.f) ? 1 : 0;
    if (a1 > ax) { ax = a1; pi = 2 + ((v1 < 0.f) ? 1 : 0); }
    if (a2 > ax) { ax = a2; pi = 4 + ((v2 < 0.f) ? 1 : 0); }
    if (a3 > ax) { ax = a3; pi = 6 + ((v3 < 0.f) ? 1 : 0); }
    float hs = 0.5f * (((a0 + a1) + a2) + a3);
    int ph = 8 + ((v0 < 0.f) ? 8 : 0) + ((v1 < 0.f) ? 4 : 0) + ((v2 < 0.f) ? 2 : 0) + ((v3 < 0.f) ? 1 : 0);
    if (ax >= hs) {
        score = ax;
        return pi;
    }
    score = hs;
    return ph;
}


// sigma = fp16(sqrt(rmax)), round to nearest even, saturating.  The fp32 square root is within
// 2 ulp(fp32) of the exact one, so it rounds to the same fp16 value unless it lies within a few
// fp32 ulp of a rounding boundary (the 13 dropped bits close to 0x1000) or the result is
// subnormal; only then is the fp64 recipe run.
__device__ __forceinline__ uint16_t sigma_of_row_max(double rmax)
{
    const float sf = __builtin_amdgcn_sqrtf((float)rmax);  // 1 ulp; a flushed subnormal takes the fp64 recipe below
    const uint32_t sb = __float_as_uint(sf);
    const int dist = (int)(sb & 0x1fffu) - 0x1000;
    const bool slow = rmax != 0.0 && sf < 65504.f && (sf < 0x1.0p-14f || (dist >= -8 && dist <= 8));
    uint16_t sigma16 = sf >= 65504.f ? (uint16_t)0x7bff : __builtin_bit_cast(uint16_t, (_Float16)sf);
    if (__any(slow)) {
        if (slow)
            sigma16 = double_to_half_rne_sat(sqrt(rmax));
    }
    return sigma16;
}

// Radius code r_q = clamp(rint(sqrt(r2) * L / sigma), 0, L), defined in fp64.  An fp32
// evaluation with the hardware's 1-ulp square root (r_f) and reciprocal is off by at most
// 6e-7 * L (five roundings of <= 1.2e-7 each); it rounds the same way unless it lands within
// that distance of a rounding boundary, and only then is the fp64 recipe run (about one wave
// in two hundred at L = 63).
__device__ __forceinline__ int radius_code(double r2, float r_f, uint16_t sigma16, double Lq)
{
    int rq = 0;
    const float sigma_f = (float)__builtin_bit_cast(_Float16, sigma16);
    bool exact_needed = false;
    if (sigma16 != 0 && r2 != 0.0) {
        const float qf = fminf(r_f * (float)Lq * __builtin_amdgcn_rcpf(sigma_f), (float)Lq);
        const float fr = qf - floorf(qf);
        exact_needed = fabsf(fr - 0.5f) < 6e-7f * (float)Lq + 1e-6f;
        rq = (int)rintf(qf);
    }
    if (__any(exact_needed)) {
        if (exact_needed) {
            const double sigma = half_bits_to_double(sigma16);
            double q = rint((sqrt(r2) * Lq) / sigma);
            q = q < 0.0 ? 0.0 : (q > Lq ? Lq : q);
            rq = (int)q;
        }
    }
    return rq;
}

// Direction of a chunk in fp32: kOperandScale times the unit vector (zeros for a zero chunk).
struct Direction {
    float u0, u1, u2, u3;
};
__device__ __forceinline__ Direction unit_direction(const half4_t xv, double r2, float r_f)
{
    // times kOperandScale, the factor the matrix operands carry: a power of two, so every comparison
    // between scores comes out as for the unit vector itself
    const float inv = r2 != 0.0 ? __builtin_amdgcn_rcpf(r_f) * kOperandScale : 0.f;
    Direction d;
    d.u0 = (float)xv[0] * inv;
    d.u1 = (float)xv[1] * inv;
    d.u2 = (float)xv[2] * inv;
    d.u3 = (float)xv[3] * inv;
    return d;
}

typedef float float16_t __attribute__((ext_vector_type(16)));

// x = h + l to 24 bits (|x - h - l| <= 2^-24 |x|), each part an fp16
struct Parts2 {
    _Float16 h, l;
};
// Hides how an fp32 value was computed.  split2 needs it: left to itself the compiler folds the
// multiplication that produced x into one of the two conversions (v_fma_mixlo_f16 rounds the exact product
// once) and converts the rounded x for the other (rounded twice); where x sits on the midpoint between two
// fp16 values the two disagree by one fp16 step and h + l misses x by 2^-11 |x|.  Seen once in 786,432
// chunks; harmless only when the product is exact (a scaling by a power of two).
__device__ __forceinline__ float opaque(float x)
{
    asm volatile("" : "+v"(x));
    return x;
}
// x: a value that went through opaque(), or an exact scaling of one.
__device__ __forceinline__ Parts2 split2(float x)
{
    Parts2 p;
    p.h = (_Float16)x;
    p.l = (_Float16)(x - (float)p.h);
    return p;
}

// v = u conj(q) in fp32 and its closed-form score max_p <v, P_p>
__device__ __forceinline__ float score_secondary(const float *q, float u0, float u1, float u2, float u3, float &v0,
                                                 float &v1, float &v2, float &v3)
{
    const float a = q[0], bq = q[1], cq = q[2], d = q[3];
    v0 = fmaf(d, u3, fmaf(cq, u2, fmaf(bq, u1, a * u0)));
    v1 = fmaf(cq, u3, fmaf(-d, u2, fmaf(a, u1, -bq * u0)));
    v2 = fmaf(-bq, u3, fmaf(a, u2, fmaf(d, u1, -cq * u0)));
    v3 = fmaf(a, u3, fmaf(bq, u2, fmaf(-cq, u1, -d * u0)));
    const float a0 = fabsf(v0), a1 = fabsf(v1), a2 = fabsf(v2), a3 = fabsf(v3);
    return fmaxf(fmaxf(fmaxf(fmaxf(a0, a1), a2), a3), 0.5f * (((a0 + a1) + a2) + a3));  // two v_max3
}

// Maximum of a 64-bit key over the wave (every lane gets it).
__device__ __forceinline__ unsigned long long wave_umax64(unsigned long long k)
{
    k = umax64(k, dpp_move64<0xB1>(k));   // quad_perm [1, 0, 3, 2]
    k = umax64(k, dpp_move64<0x4E>(k));   // quad_perm [2, 3, 0, 1]
    k = umax64(k, dpp_move64<0x141>(k));  // row_half_mirror
    k = umax64(k, dpp_move64<0x140>(k));  // row_mirror
    k = umax64(k, (unsigned long long)__shfl_xor((long long)k, 16, 64));
    k = umax64(k, (unsigned long long)__shfl_xor((long long)k, 32, 64));
    return k;
}

// Two groups of secondaries whose screened maxima lie closer than this fraction of the larger one are
// not told apart by the screen.  Its error is below 7e-7 |q_s| per score (operands carried to 2^-24 each,
// fp32 accumulation, three fp32 additions; 2.9e-7 measured), the best score is at least |q_s| / sqrt(2),
// so the band is at least three times that bound on the error of the two scores compared (seven times
// the measured value), whatever the common scale
// (the scores of the matrix pass carry a factor kOperandScale^2 = 2^20).
constexpr float kScreenBand = 6.0e-6f;

// Exhaustive nearest-codeword search for the wave's 64 chunks (one per lane, direction u as
// unit_direction returns it): returns
// the chunk's code word (rq << w_idx) | k with k = p S + s of the best joint codeword; 0 for a
// flagged chunk (also to be passed for a lane without a chunk) and for a zero chunk (r2 == 0).
// Called by all 64 lanes.  amat / secl: the head's A operands and secondaries in LDS.
//
// Three steps.  Screen: all S secondaries on the matrix cores with operands split in two fp16
// parts; lane (col = l % 32, half = l / 32) sees, for the chunks col and 32 + col, the secondaries
// 16 grp + 2 t + half (t = 0..7) of every group grp, and keeps per chunk slot the best group, its
// score and the runner-up score.  Decide: the two lanes of a chunk exchange their results; a clear
// winner (ahead of every other lane-group by more than the band) names 8 candidate secondaries, which
// are scored again in fp32.  Otherwise (a few chunks in a thousand) the wave scores all S secondaries
// of that chunk in fp32, 64 at a time.  The decision between secondaries is therefore always taken
// on fp32 closed-form scores, the lowest s winning exact ties.
//
// kCoop (a workgroup whose rows fill a single pass): all kWaves waves of the workgroup hold the same 64
// chunks, each screens its share of the groups, the per-chunk results (best lane-group, its score, the
// runner-up) meet in `merge` [kWaves][64][3], and wave 0 alone decides and returns the code words (the other
// waves return 0).  The merged triple is what one wave screening every group would have found, except when two
// waves tie for the best score exactly; the runner-up then equals the best and the chunk takes the fp32 search,
// as any tie between groups does.
template <bool kCoop = false, int kWaves = 1, bool kScreen = true>
__device__ __forceinline__ uint32_t search_codeword(const Geometry &g, int lane, const Direction u, bool flagged,
                                                    double r2, int rq, const uint4 *amat, const float *secl,
                                                    int wv = 0, float *merge = nullptr)
{
    const float u0 = opaque(u.u0), u1 = opaque(u.u1), u2 = opaque(u.u2), u3 = opaque(u.u3);
    const int half = lane >> 5;
    // B operands: lane (col, half) supplies components 2 half, 2 half + 1 of chunk 32 j + col in the
    // slots [h l h l | h l h l]; chunk 32 half + col is its own, the other one its partner's (lane ^ 32)
    half8_t bop[2];
    {
        const Parts2 p0 = split2(u0), p1 = split2(u1), p2 = split2(u2), p3 = split2(u3);
        const uint32_t k0 = pack2(p0.h, p0.l), k1 = pack2(p1.h, p1.l), k2 = pack2(p2.h, p2.l), k3 = pack2(p3.h, p3.l);
        const uint32_t own_a = half ? k2 : k0, own_b = half ? k3 : k1;
        const uint32_t snd_a = half ? k0 : k2, snd_b = half ? k1 : k3;
        const uint32_t rcv_a = (uint32_t)__shfl_xor((int)snd_a, 32, 64), rcv_b = (uint32_t)__shfl_xor((int)snd_b, 32, 64);
        const uint32_t j0a = half ? rcv_a : own_a, j0b = half ? rcv_b : own_b;
        const uint32_t j1a = half ? own_a : rcv_a, j1b = half ? own_b : rcv_b;
        bop[0] = __builtin_bit_cast(half8_t, make_uint4(j0a, j0a, j0b, j0b));
        bop[1] = __builtin_bit_cast(half8_t, make_uint4(j1a, j1a, j1b, j1b));
    }

    // ---- screen ----------------------------------------------------------------------------------------
    float best[2] = {-1.f, -1.f}, second[2] = {-1.f, -1.f};
    int bkey[2] = {0, 0};
    float16_t zero16;
#pragma unroll
    for (int e = 0; e < 16; ++e)
        zero16[e] = 0.f;
    // groups this wave screens: those held as matrix operands (none beyond kScreenMaxS secondaries: the
    // screen is then skipped and every chunk takes the fp32 search below)
    const int n_grp = kScreen ? g.S16 : 0;
    const int per_wave = kCoop ? (n_grp + kWaves - 1) / kWaves : n_grp;
    const int grp_begin = kCoop ? min(wv * per_wave, n_grp) : 0;
    const int grp_end = kCoop ? min(grp_begin + per_wave, n_grp) : n_grp;
    const uint4 *arow = amat + lane;
    half8_t a0 = __builtin_bit_cast(half8_t, make_uint4(0u, 0u, 0u, 0u)), a1 = a0;
    float16_t ahead = zero16;
    if (kScreen) {
        a0 = __builtin_bit_cast(half8_t, arow[2 * min(grp_begin, n_grp - 1) * 64]);
        a1 = __builtin_bit_cast(half8_t, arow[2 * min(grp_begin, n_grp - 1) * 64 + 64]);
        // the product of (tile 0, chunk slot 0) of the next group is issued before the arithmetic on the last
        // product of this one: a VALU instruction right behind the MFMA it depends on idles for the depth of
        // the matrix pipeline
        ahead = __builtin_amdgcn_mfma_f32_32x32x16_f16(a0, bop[0], zero16, 0, 0, 0);
    }
    for (int grp = grp_begin; grp < grp_end; ++grp) {
        // the next group's operands replace this group's as soon as their last product is issued (the
        // last group re-reads itself; that product is dropped)
        const uint4 *anext = arow + 2 * min(grp + 1, n_grp - 1) * 64;
        // over the group's 8 secondaries on this lane: GA = largest |v_i| (best axis element), GH = largest
        // |v_0|+|v_1|+|v_2|+|v_3| (twice the best half-integer element)
        float GA[2], GH[2];
#pragma unroll
        for (int k = 0; k < 4; ++k) {  // (tile k / 2, chunk slot k % 2)
            const int j = k & 1;
            const float16_t c = ahead;
            if (k == 0) {
                ahead = __builtin_amdgcn_mfma_f32_32x32x16_f16(a0, bop[1], zero16, 0, 0, 0);
                a0 = __builtin_bit_cast(half8_t, anext[0]);
            } else if (k == 1) {
                ahead = __builtin_amdgcn_mfma_f32_32x32x16_f16(a1, bop[0], zero16, 0, 0, 0);
            } else if (k == 2) {
                ahead = __builtin_amdgcn_mfma_f32_32x32x16_f16(a1, bop[1], zero16, 0, 0, 0);
                a1 = __builtin_bit_cast(half8_t, anext[64]);
            } else {
                ahead = __builtin_amdgcn_mfma_f32_32x32x16_f16(a0, bop[0], zero16, 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
            float t[16], h[4];
#pragma unroll
            for (int e = 0; e < 16; ++e)
                t[e] = fabsf(c[e]);
#pragma unroll
            for (int i = 0; i < 4; ++i)  // secondary i of the tile's four
                h[i] = ((t[4 * i] + t[4 * i + 1]) + t[4 * i + 2]) + t[4 * i + 3];
            // v_max3 chains; the group's first tile starts them from its own values (|v| >= 0: no zero needed)
            float ga, gh;
            if (k < 2) {
                ga = fmaxf(fmaxf(t[0], t[1]), t[2]);
#pragma unroll
                for (int e = 3; e < 15; e += 2)
                    ga = fmaxf(fmaxf(ga, t[e]), t[e + 1]);
                ga = fmaxf(ga, t[15]);
                gh = fmaxf(fmaxf(fmaxf(h[0], h[1]), h[2]), h[3]);
            } else {
                ga = GA[j];
#pragma unroll
                for (int e = 0; e < 16; e += 2)
                    ga = fmaxf(fmaxf(ga, t[e]), t[e + 1]);
                gh = fmaxf(fmaxf(fmaxf(fmaxf(GH[j], h[0]), h[1]), h[2]), h[3]);
            }
            GA[j] = ga;
            GH[j] = gh;
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const float M = fmaxf(GA[j], 0.5f * GH[j]);
            second[j] = __builtin_amdgcn_fmed3f(M, best[j], second[j]);  // second <= best on entry
            if (M > best[j]) {
                best[j] = M;
                bkey[j] = 16 * grp;
            }
        }
    }

    // ---- decide: chunk 32 j + col was screened by lanes col and 32 + col (slot j of each) and is
    // owned by lane 32 j + col, i.e. slot `half` of the owner and of its partner ------------------------
    const float my_b = half ? best[1] : best[0], my_s = half ? second[1] : second[0];
    const int my_k = half ? bkey[1] : bkey[0];
    const float ot_b = __shfl_xor(half ? best[0] : best[1], 32, 64);
    const float ot_s = __shfl_xor(half ? second[0] : second[1], 32, 64);
    const int ot_k = __shfl_xor(half ? bkey[0] : bkey[1], 32, 64);
    const bool other = ot_b > my_b;
    float top = other ? ot_b : my_b;
    float runner = fmaxf(fmaxf(fminf(my_b, ot_b), my_s), ot_s);
    int first = (other ? ot_k : my_k) + (other ? 1 - half : half);  // candidates first + 2 t
    if (kCoop) {
        float *mine = merge + (wv * 64 + lane) * 3;
        mine[0] = top;
        mine[1] = runner;
        mine[2] = __int_as_float(first);
        __syncthreads();
        if (wv != 0)
            return 0u;
#pragma unroll
        for (int k = 1; k < kWaves; ++k) {  // a wave without groups left its initial -1: never the best
            const float *theirs = merge + (k * 64 + lane) * 3;
            const float tb = theirs[0], tr = theirs[1];
            const int tf = __float_as_int(theirs[2]);
            const bool better = tb > top;
            runner = fmaxf(fmaxf(fminf(top, tb), runner), tr);
            first = better ? tf : first;
            top = better ? tb : top;
        }
    }
    const bool live = !flagged && r2 != 0.0;
    const bool unclear = live && (!kScreen || !(top - runner >= kScreenBand * top));

    // The 8 candidates first + 2 t in ascending order, strict comparison: the lowest s wins a tie.  Padding
    // secondaries (zeros, s >= S) score 0 and every real one scores at least |q_s| / sqrt(2) > 0 for a
    // non-zero chunk, so a group that won the screen never yields a padding index; the bound below only
    // keeps the index inside the codebook should the input break the contract (non-finite values).
    int bs = first;
    if (live && kScreen) {
        const float *cq = secl + 4 * first;  // < 16 S16 entries: inside the padded table
        float bsc = -1.f;
        int bt = 0;
#pragma unroll
        for (int tt = 0; tt < 8; ++tt) {
            float v0, v1, v2, v3;
            const float sc = score_secondary(cq + 8 * tt, u0, u1, u2, u3, v0, v1, v2, v3);
            const bool take = sc > bsc;
            bsc = take ? sc : bsc;
            bt = take ? tt : bt;
        }
        bs = min(first + 2 * bt, g.S - 1);
    }
    // the unclear chunks, one at a time: every lane scores the secondaries lane, lane + 64, ...; the key
    // orders by score, then by descending s (scores are positive, so their bit patterns order like them)
    unsigned long long todo = __ballot(unclear);
    while (todo) {  // wave-uniform
        const int src = __ffsll((long long)todo) - 1;
        todo &= todo - 1ull;
        const float e0 = __uint_as_float((uint32_t)__builtin_amdgcn_readlane((int)__float_as_uint(u0), src));
        const float e1 = __uint_as_float((uint32_t)__builtin_amdgcn_readlane((int)__float_as_uint(u1), src));
        const float e2 = __uint_as_float((uint32_t)__builtin_amdgcn_readlane((int)__float_as_uint(u2), src));
        const float e3 = __uint_as_float((uint32_t)__builtin_amdgcn_readlane((int)__float_as_uint(u3), src));
        unsigned long long key = 0ull;
        for (int s = lane; s < g.S; s += 64) {
            float v0, v1, v2, v3;
            const float sc = score_secondary(secl + 4 * s, e0, e1, e2, e3, v0, v1, v2, v3);
            key = umax64(key, ((unsigned long long)__float_as_uint(sc) << 32) | (0xffffffffu - (uint32_t)s));
        }
        key = wave_umax64(key);
        if (lane == src)
            bs = (int)min(0xffffffffu - (uint32_t)key, (uint32_t)g.S - 1u);
    }

    uint32_t code = 0;
    if (live) {
        float w0, w1, w2, w3, sc;
        (void)score_secondary(secl + 4 * bs, u0, u1, u2, u3, w0, w1, w2, w3);
        const int p = nearest_primary(w0, w1, w2, w3, sc);
        code = ((uint32_t)rq << g.w_idx) | (uint32_t)(p * g.S + bs);
    }
    return code;
}

}  // namespace

// The K = 4 contraction v = A(q_s) u on v_mfma_f32_32x32x16_f16: a product covers 8 secondaries (32 rows =
// 8 x 4 components of v) and 32 chunks (columns); its K = 16 are the 4 terms of the contraction times the
// 4 products of a two-part split (both operands are scaled by 2^10 first so that the low parts stay
// normal).  Lane l of an operand holds row (column) l % 32 and the terms 2 (l / 32), 2 (l / 32) + 1, each in
// four fp16 slots: A as [h h l l], B as [h l h l].  The four fp16 x fp16 products are exact in fp32 and
// add up inside the matrix core.  Lane l of the result holds, for column l % 32, the rows
// 8 i + 4 (l / 32) + c (i, c = 0..3): all four components of v for the secondaries 2 i + l / 32 of the tile.
// The scores come out scaled by 2^20, which no comparison notices.
//
// Dynamic LDS layout:
//   amat  [2*S16][64] x 16 B   MFMA A operands, one 64-lane tile per 8 secondaries
//                              (copied from the table k_prepare_operands built for the head)
//   secl  [16*S16][4] f32      the head's secondaries (zero padded to a multiple of 16)
//   pack  [kWaves][2][32] u32 row code words being assembled
//   rcnt  [search_rows] u32    outliers per row of the workgroup
// The search's MFMA A operands of every head, built once per call into the workspace (the workgroups
// of the search then only copy their head's table into LDS).  grid = (ceil(4 S16 64 / 256), H, tensors).
// Entry idx of a head's operand table: tile idx / 64 of 8 secondaries, lane l = idx % 64 holding row
// l % 32 = 4 (secondary in tile) + i and the factors k = 2 (l / 32), 2 (l / 32) + 1 of that row, each in the
// slots [h h l l].
__device__ __forceinline__ uint4 operand_entry(const float *sec_h, int S, int idx)
{
    const int tile = idx >> 6, l = idx & 63;
    const int row = l & 31, kh = l >> 5;
    const int i = row & 3;
    const int sidx = 8 * tile + (row >> 2);
    float a = 0.f, bq = 0.f, c = 0.f, d = 0.f;  // zero rows pad S up to a multiple of 16
    if (sidx < S) {
        const float *q = sec_h + 4 * sidx;
        a = q[0], bq = q[1], c = q[2], d = q[3];
    }
    // v = u (x) conj(q):  v0 =  a u0 + b u1 + c u2 + d u3
    //                     v1 = -b u0 + a u1 - d u2 + c u3
    //                     v2 = -c u0 + d u1 + a u2 - b u3
    //                     v3 = -d u0 - c u1 + b u2 + a u3
    auto entry = [&](int k) -> float {  // A[i][k]
        if (i == 0)
            return (k == 0) ? a : (k == 1) ? bq : (k == 2) ? c : d;
        if (i == 1)
            return (k == 0) ? -bq : (k == 1) ? a : (k == 2) ? -d : c;
        if (i == 2)
            return (k == 0) ? -c : (k == 1) ? d : (k == 2) ? a : -bq;
        return (k == 0) ? -d : (k == 1) ? -c : (k == 2) ? bq : a;
    };
    const float va = entry(2 * kh), vb = entry(2 * kh + 1);
    const Parts2 pa = split2(opaque(va) * kOperandScale), pb = split2(opaque(vb) * kOperandScale);
    return make_uint4(pack2(pa.h, pa.h), pack2(pa.l, pa.l), pack2(pb.h, pb.h), pack2(pb.l, pb.l));
}

__global__ __launch_bounds__(kThreads) void k_prepare_operands(Geometry g, WorkspaceOffsets wo, EncodeBatch batch)
{
    const EncodeTensor &tn = batch.t[blockIdx.z];
    const Workspace ws = carve_workspace(tn.ws, wo);
    const int h = blockIdx.y;
    const int idx = blockIdx.x * kThreads + threadIdx.x;
    if (idx < g.A16 * kATiles * 64)
        ws.aop[(size_t)h * g.A16 * kATiles * 64 + idx] = operand_entry(tn.sec + (size_t)h * g.S * 4, g.S, idx);
}

// kWaves: 4 (several workgroups per CU); 16 for workgroups of 256 or 512 rows whose tables would leave
// room for fewer than four such workgroups (one per CU, four waves on every SIMD); 8 when tables and row
// state are so large that only one workgroup fits a CU and 16 waves do not: twice the waves then share
// the tables and keep two waves on every SIMD.
// This kernel is for rows of 128 elements (32 chunks: two rows per wave); k_search_flat below takes
// every other head dimension.
// kFused: the form for tensors of a few rows whose thresholds are known beforehand (appended tokens with
// supplied thresholds, extraction switched off): no kernel runs before this one, so it takes its thresholds
// from the caller's array (+infinity without one), builds the head's operand table itself, and reports a
// non-finite input through bit 31 of its workgroup total, which the list kernel turns into the status word.
template <int kWaves, int kRows, bool kFused = false, bool kScreen = true>
__global__ __launch_bounds__(64 * kWaves, kFused ? 1 : 4) void k_search(Geometry g, WorkspaceOffsets wo, EncodeBatch batch)
{
    constexpr int kThreadsS = 64 * kWaves;
    const EncodeTensor &tn = batch.t[blockIdx.z];
    const Workspace ws = carve_workspace(tn.ws, wo);
    const EncodedPtrs enc = tn.enc;
    const _Float16 *__restrict__ x = tn.x;
    const float *__restrict__ sec = tn.sec;
    extern __shared__ float smem[];
    uint4 *amat = reinterpret_cast<uint4 *>(smem);
    float *secl = reinterpret_cast<float *>(amat + (size_t)(kScreen ? g.S16 : 0) * kATiles * 64);
    uint32_t *pack = reinterpret_cast<uint32_t *>(secl + (size_t)g.S16 * 16 * 4);
    uint32_t *rcnt = pack + kWaves * 2 * 32;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform, and known to be
    // by_head (kFused, several batch entries of a few rows each): one workgroup per head takes the rows of all
    // batch entries, so that the head's tables are built once; its rows are the pairs (b, t), b-major
    const bool by_head = kFused && g.fused_by_head != 0;
    const int seg = blockIdx.y, b = by_head ? 0 : seg / g.H, h = by_head ? seg : seg % g.H;
    const int t0 = blockIdx.x * kRows;
    const int n_here = by_head ? g.B * g.T : g.T;  // rows this workgroup column addresses
    const float *sec_h = sec + (size_t)h * g.S * 4;
    // row v of the column: its batch entry and token, the address of its chunk c, its linear row index
    struct RowAt {
        const _Float16 *chunk;
        int64_t R;
    };
    auto row_at = [&](int v, int c) {
        const int bb = by_head ? v / g.T : b;
        const int tt = by_head ? v - bb * g.T : v;
        RowAt r;
        r.chunk = x + (int64_t)bb * g.sb + (int64_t)h * g.sh + (int64_t)tt * g.st + 4 * c;
        r.R = ((int64_t)bb * g.H + h) * g.T + tt;
        return r;
    };
    // kFused (a launch of a few rows, bound by latency): a workgroup with one or two rows (one appended token)
    // runs its single pass on all its waves together (search_codeword's cooperative form), and the first
    // chunk is requested before the tables
    const bool coop = kFused && n_here - t0 <= 2;  // uniform over the workgroup
    __shared__ float merge[kFused ? kWaves * 64 * 3 : 1];
    half4_t first_chunk = {0, 0, 0, 0};
    if (kFused) {
        const int v = t0 + (coop ? 0 : wv * 2) + (lane >> 5);
        if (v < n_here)
            first_chunk = load_chunk(row_at(v, lane & 31).chunk);
    }

    // ---- setup: secondaries and A operands into LDS ---------------------------------------
    for (int s = tid; s < g.S16 * 16; s += kThreadsS) {
        float4_t q = {0.f, 0.f, 0.f, 0.f};
        if (s < g.S)
            q = *reinterpret_cast<const float4_t *>(sec_h + 4 * s);
        *reinterpret_cast<float4_t *>(secl + 4 * s) = q;
    }
    if (kFused) {
        for (int idx = tid; idx < (kScreen ? g.S16 : 0) * kATiles * 64; idx += kThreadsS)
            amat[idx] = operand_entry(sec_h, g.S, idx);
        if (coop)  // the one pass writes the counters of rows 0 and 1 only
            for (int r = tid; r < kRows; r += kThreadsS)
                rcnt[r] = 0;
    } else {
        const uint4 *src = ws.aop + (size_t)h * (kScreen ? g.S16 : 0) * kATiles * 64;
        for (int idx = tid; idx < (kScreen ? g.S16 : 0) * kATiles * 64; idx += kThreadsS)
            amat[idx] = src[idx];
    }

    __syncthreads();

    const double thr = !kFused ? ws.thr[h] : tn.thr_given ? tn.thr_given[h] : __longlong_as_double(0x7ff0000000000000LL);
    if (kFused && blockIdx.x == 0 && b == 0 && tid == 0)
        ws.thr[h] = thr;  // what hqmq_thresholds reads back
    uint32_t bad_seen = 0;  // kFused: this lane saw a ballot with a non-finite chunk in it
    const double Lq = (double)((1 << g.b_r) - 1);
    const int c = lane & 31, half_id = lane >> 5;
    uint32_t *my_pack = pack + wv * 64;

    const int n_it = coop ? 1 : kRows / (2 * kWaves);
    for (int it = 0; it < n_it; ++it) {
        const int r_in_block = coop ? half_id : it * 2 * kWaves + wv * 2 + half_id;
        const int t = t0 + r_in_block;
        const bool valid = t < n_here;
        if (!coop && t0 + it * 2 * kWaves + wv * 2 >= n_here) {  // wave-uniform: both rows of this iteration lie past the end
            if (c == 0)
                rcnt[r_in_block] = 0;
            continue;
        }

        // ---- chunk, norm, flag, row scale --------------------------------------------------
        const RowAt here = row_at(valid ? t : t0, c);
        half4_t xv = (kFused && it == 0) ? first_chunk : valid ? load_chunk(here.chunk) : half4_t{0, 0, 0, 0};
        const double r2 = chunk_norm2(xv);
        const bool flagged = valid && (r2 > thr);
        const unsigned long long ballot = __ballot(flagged);
        const uint32_t word = half_id ? (uint32_t)(ballot >> 32) : (uint32_t)ballot;
        if (g.check_finite) {  // uniform
            const bool bad = valid && chunk_nonfinite(xv);
            if (__ballot(bad) != 0ull) {
                if (kFused)
                    bad_seen = 1u;
                else if (lane == 0)
                    atomicOr(enc.status, HQMQ_STATUS_NONFINITE);
            }
        }

        // max over the 32 lanes of the row: four DPP steps inside each 16-lane row (after each step the
        // running maxima are uniform over a block twice as large, so the mirror patterns pair the right
        // blocks), one swap across rows
        double rmax = flagged ? 0.0 : r2;
        rmax = fmax(rmax, dpp_move_f64<0xB1>(rmax));   // quad_perm [1, 0, 3, 2]
        rmax = fmax(rmax, dpp_move_f64<0x4E>(rmax));   // quad_perm [2, 3, 0, 1]
        rmax = fmax(rmax, dpp_move_f64<0x141>(rmax));  // row_half_mirror
        rmax = fmax(rmax, dpp_move_f64<0x140>(rmax));  // row_mirror
        rmax = fmax(rmax, __shfl_xor(rmax, 16, 64));
        const uint16_t sigma16 = sigma_of_row_max(rmax);
        const float r_f = __builtin_amdgcn_sqrtf((float)r2);
        const int rq = radius_code(r2, r_f, sigma16, Lq);
        const Direction u = unit_direction(xv, r2, r_f);
        my_pack[lane] = 0;  // after the previous iteration's reads of it: LDS serves a wave in order
        uint32_t code;
        if (coop) {
            code = search_codeword<true, kWaves>(g, lane, u, flagged, r2, rq, amat, secl, wv, merge);
            if (wv != 0)
                continue;  // wave 0 holds the result and writes the two rows
        } else {
            code = search_codeword<false, 1, kScreen>(g, lane, u, flagged, r2, rq, amat, secl);
        }

        // ---- pack the row: chunk c at bits [c*w, (c+1)*w) -----------------------------------------
        {
            uint32_t bitpos = (uint32_t)c * g.w;
            uint32_t d0 = bitpos >> 5, sh = bitpos & 31;
            uint32_t *rowp = my_pack + half_id * 32;
            if (code) {
                atomicOr(&rowp[d0], code << sh);
                if (sh + g.w > 32)
                    atomicOr(&rowp[d0 + 1], code >> (32 - sh));
            }
        }
        wave_lds_sync();
        if (valid) {
            const int64_t R = here.R;
            if (c < g.w)
                enc.codes[R * g.w + c] = my_pack[half_id * 32 + c];
            if (c == 0) {
                enc.sigma[R] = sigma16;
                enc.flags[R] = word;
            }
        }
        if (c == 0)
            rcnt[r_in_block] = valid ? __popc(word) : 0;
    }

    // ---- outlier offsets local to the workgroup and its total; the global prefix is added by the
    // scan / gather kernels that follow --------------------------------------------------------------
    const uint32_t bad_any = kFused ? (uint32_t)__syncthreads_or((int)bad_seen) : (__syncthreads(), 0u);
    if (wv == 0) {
        uint32_t carry = 0;
#pragma unroll
        for (int part = 0; part < kRows / 64; ++part) {
            const int r = 64 * part + lane;
            const uint32_t cnt = rcnt[r];
            uint32_t inc = cnt;
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) {
                uint32_t o = __shfl_up(inc, d, 64);
                if (lane >= d)
                    inc += o;
            }
            if (by_head) {
                // (64 rows at most, one part) every batch entry's rows are a run of their own in the list's
                // order: offsets restart at each run, and each run reports its total as a workgroup would
                const int run = r / g.T, start = run * g.T;
                const uint32_t before_run = __shfl(inc - cnt, min(start, 63), 64);
                if (r < n_here) {
                    enc.row_off[row_at(r, 0).R] = inc - cnt - before_run;
                    if (r - start == g.T - 1)
                        ws.block_sum[(size_t)run * g.H + h] = (inc - before_run) | (bad_any ? 0x80000000u : 0u);
                }
            } else if (t0 + r < g.T) {
                enc.row_off[row_at(t0 + r, 0).R] = carry + inc - cnt;
            }
            carry += __shfl(inc, 63, 64);
        }
        if (lane == 0 && !by_head)  // a workgroup holds at most 512 x 32 outliers: bit 31 is free for the flag
            ws.block_sum[(size_t)seg * g.n_search_blocks_per_seg + blockIdx.x] = carry | (bad_any ? 0x80000000u : 0u);
    }
}


// The same search for any head dimension: rows of n_c = ceil(D / 4) <= 32 chunks.  A workgroup owns
// 64 or 256 rows of one (b, h) segment and treats their chunks as one flat list, 64 consecutive
// chunks per wave and iteration, so that every lane of every matrix product carries a chunk whatever
// n_c is.  Rows then straddle waves, so what the row-per-half-wave kernel does with cross-lane
// operations goes through LDS here:
//   pass 1  every chunk's squared norm once: flagged chunks set their bit in the row's flag word,
//           the others take part in the row's maximum (atomics on LDS); one lane per row then turns
//           the maximum into the fp16 scale and writes scale and flag word out;
//   pass 2  the chunks again (second read from L2): radius code against the row's scale, direction
//           search, code word OR-ed into the row's slot of the packing area;
//   end     the packing area goes out as one contiguous block, then the outlier offsets as above.
// Dynamic LDS: amat | secl as in k_search, then rowmax u64 [kRows] | fword u32 [kRows] |
// sig u32 [kRows] | rcnt u32 [kRows] | pack u32 [kRows * row_words].
// kFused: as in k_search.
template <int kWaves, int kRows, bool kFused = false, bool kScreen = true>
__global__ __launch_bounds__(64 * kWaves) void k_search_flat(Geometry g, WorkspaceOffsets wo, EncodeBatch batch)
{
    constexpr int kThreadsS = 64 * kWaves;
    static_assert(kRows % 64 == 0 && kRows <= kThreadsS, "one thread per row in the scale pass");
    const EncodeTensor &tn = batch.t[blockIdx.z];
    const Workspace ws = carve_workspace(tn.ws, wo);
    const EncodedPtrs enc = tn.enc;
    const _Float16 *__restrict__ x = tn.x;
    extern __shared__ float smem[];
    uint4 *amat = reinterpret_cast<uint4 *>(smem);
    float *secl = reinterpret_cast<float *>(amat + (size_t)(kScreen ? g.S16 : 0) * kATiles * 64);
    unsigned long long *rowmax = reinterpret_cast<unsigned long long *>(secl + (size_t)g.S16 * 16 * 4);
    uint32_t *fword = reinterpret_cast<uint32_t *>(rowmax + kRows);
    uint32_t *sig = fword + kRows;
    uint32_t *rcnt = sig + kRows;
    uint32_t *pack = rcnt + kRows;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int seg = blockIdx.y, b = seg / g.H, h = seg % g.H;
    const int t0 = blockIdx.x * kRows;
    const int nrows = min(kRows, g.T - t0);       // >= 1 by the grid's size
    const int nchunks = nrows * g.n_c;
    const int row_words = g.row_words;
    const int64_t row0 = (int64_t)seg * g.T + t0;  // linear index of the workgroup's first row
    const float *sec_h = tn.sec + (size_t)h * g.S * 4;

    // ---- setup: tables into LDS, per-row state cleared ------------------------------------------
    for (int s = tid; s < g.S16 * 16; s += kThreadsS) {
        float4_t q = {0.f, 0.f, 0.f, 0.f};
        if (s < g.S)
            q = *reinterpret_cast<const float4_t *>(sec_h + 4 * s);
        *reinterpret_cast<float4_t *>(secl + 4 * s) = q;
    }
    if (kFused) {
        for (int idx = tid; idx < (kScreen ? g.S16 : 0) * kATiles * 64; idx += kThreadsS)
            amat[idx] = operand_entry(sec_h, g.S, idx);
    } else {
        const uint4 *src = ws.aop + (size_t)h * (kScreen ? g.S16 : 0) * kATiles * 64;
        for (int idx = tid; idx < (kScreen ? g.S16 : 0) * kATiles * 64; idx += kThreadsS)
            amat[idx] = src[idx];
    }
    for (int i = tid; i < kRows; i += kThreadsS) {
        rowmax[i] = 0ull;
        fword[i] = 0u;
    }
    for (int i = tid; i < kRows * row_words; i += kThreadsS)
        pack[i] = 0u;
    __syncthreads();

    const double thr = !kFused ? ws.thr[h] : tn.thr_given ? tn.thr_given[h] : __longlong_as_double(0x7ff0000000000000LL);
    if (kFused && blockIdx.x == 0 && b == 0 && tid == 0)
        ws.thr[h] = thr;  // what hqmq_thresholds reads back
    uint32_t bad_seen = 0;
    const double Lq = (double)((1 << g.b_r) - 1);
    const _Float16 *base = x + (int64_t)b * g.sb + (int64_t)h * g.sh + (int64_t)t0 * g.st;

    // ---- pass 1: flags and row maxima ---------------------------------------------------------------
    for (int q = tid; q < nchunks; q += kThreadsS) {
        const int r = row_of_chunk(q, g), c = q - r * g.n_c;
        const half4_t xv = load_row_chunk<false>(base + (int64_t)r * g.st, c, g);
        const double r2 = chunk_norm2(xv);
        if (g.check_finite && chunk_nonfinite(xv)) {
            if (kFused)
                bad_seen = 1u;
            else
                atomicOr(enc.status, HQMQ_STATUS_NONFINITE);
        }
        if (r2 > thr)
            atomicOr(&fword[r], 1u << c);
        else
            atomicMax(&rowmax[r], key_of(r2));  // non-negative doubles order like their bit patterns
    }
    const uint32_t bad_any = kFused ? (uint32_t)__syncthreads_or((int)bad_seen) : (__syncthreads(), 0u);
    if (tid < kRows) {
        uint32_t word = 0;
        if (tid < nrows) {
            word = fword[tid];
            const uint16_t sigma16 = sigma_of_row_max(__longlong_as_double((long long)rowmax[tid]));
            sig[tid] = sigma16;
            enc.sigma[row0 + tid] = sigma16;
            enc.flags[row0 + tid] = word;
        }
        rcnt[tid] = __popc(word);
    }
    __syncthreads();

    // ---- pass 2: radius codes and the direction search ----------------------------------------------
    for (int q0 = wv * 64; q0 < nchunks; q0 += kThreadsS) {  // wave-uniform trip count
        const int q = q0 + lane;
        const bool valid = q < nchunks;
        const int r = valid ? row_of_chunk(q, g) : 0, c = valid ? q - r * g.n_c : 0;
        const half4_t xv = valid ? load_row_chunk<false>(base + (int64_t)r * g.st, c, g) : half4_t{0, 0, 0, 0};
        const double r2 = chunk_norm2(xv);
        const bool flagged = valid && (r2 > thr);
        const uint16_t sigma16 = (uint16_t)sig[r];
        const float r_f = __builtin_amdgcn_sqrtf((float)r2);
        const int rq = radius_code(r2, r_f, sigma16, Lq);
        const Direction u = unit_direction(xv, r2, r_f);
        const uint32_t code = search_codeword<false, 1, kScreen>(g, lane, u, flagged || !valid, r2, rq, amat, secl);
        if (code) {
            const uint32_t bitpos = (uint32_t)c * g.w;
            const uint32_t d0 = bitpos >> 5, sh = bitpos & 31;
            uint32_t *rowp = pack + r * row_words;
            atomicOr(&rowp[d0], code << sh);
            if (sh + g.w > 32)
                atomicOr(&rowp[d0 + 1], code >> (32 - sh));
        }
    }
    __syncthreads();

    // ---- the workgroup's code words: one contiguous block ------------------------------------------
    {
        uint32_t *dst = enc.codes + row0 * row_words;
        for (int i = tid; i < nrows * row_words; i += kThreadsS)
            dst[i] = pack[i];
    }
    // ---- outlier offsets local to the workgroup and its total ---------------------------------------
    if (wv == 0) {
        uint32_t carry = 0;
#pragma unroll
        for (int part = 0; part < kRows / 64; ++part) {
            const int r = 64 * part + lane;
            const uint32_t cnt = rcnt[r];
            uint32_t inc = cnt;
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) {
                uint32_t o = __shfl_up(inc, d, 64);
                if (lane >= d)
                    inc += o;
            }
            if (r < nrows)
                enc.row_off[row0 + r] = carry + inc - cnt;
            carry += __shfl(inc, 63, 64);
        }
        if (lane == 0)
            ws.block_sum[(size_t)seg * g.n_search_blocks_per_seg + blockIdx.x] = carry | (bad_any ? 0x80000000u : 0u);
    }
}

// The search kernels' dynamic LDS exceeds the 64 KiB a kernel gets by default once S > 208: raises the limit
// of every variant on the current device.  Stateless; the caller (the library's per-device set-up) runs it
// once per device, before any launch and outside any stream capture.
hipError_t prepare_search_kernels()
{
    const void *variants[17] = {reinterpret_cast<const void *>(k_search<4, kSearchRowsSmall, true>),
                                reinterpret_cast<const void *>(k_search<8, kSearchRowsSmall, true>),
                                reinterpret_cast<const void *>(k_search_flat<4, kSearchRowsSmall, true>),
                                reinterpret_cast<const void *>(k_search_flat<8, kSearchRowsSmall, true>),
                                reinterpret_cast<const void *>(k_search_flat<16, kSearchRowsLarge>),
                                reinterpret_cast<const void *>(k_search_flat<16, kSearchRowsHuge>),
                                reinterpret_cast<const void *>(k_search<4, kSearchRowsSmall>),
                                reinterpret_cast<const void *>(k_search<4, kSearchRowsLarge>),
                                reinterpret_cast<const void *>(k_search<8, kSearchRowsSmall>),
                                reinterpret_cast<const void *>(k_search<8, kSearchRowsLarge>),
                                reinterpret_cast<const void *>(k_search<16, kSearchRowsLarge>),
                                reinterpret_cast<const void *>(k_search<16, kSearchRowsHuge>),
                                reinterpret_cast<const void *>(k_search_flat<4, kSearchRowsSmall>),
                                reinterpret_cast<const void *>(k_search_flat<4, kSearchRowsLarge>),
                                reinterpret_cast<const void *>(k_search_flat<8, kSearchRowsSmall>),
                                reinterpret_cast<const void *>(k_search<4, kSearchRowsSmall, false, false>),
                                reinterpret_cast<const void *>(k_search_flat<4, kSearchRowsSmall, false, false>)};
    hipError_t err = hipSuccess;
    // the first four (the fused forms, only ever launched with 64 rows per workgroup) also hold static LDS (the
    // workgroup-wide OR, the merge buffer of the cooperative pass: up to 6 KiB), which counts against the same 160 KiB
    for (int i = 0; i < 17 && err == hipSuccess; ++i)
        err = hipFuncSetAttribute(variants[i], hipFuncAttributeMaxDynamicSharedMemorySize,
                                  (int)kLdsPerCu - (i < 4 ? 8192 : 0));
    return err;
}

// The fused form exists for the workgroup shapes that short segments get: 64 rows, 4 or 8 waves.
bool search_fused_available(const Geometry &g)
{
    if (g.A16 == 0)
        return false;  // no screen: the general form
    const int waves = search_waves_for(g.S16, g.A16, g.D, g.row_words, g.search_rows);
    return g.search_rows == kSearchRowsSmall && (waves == 4 || waves == 8);
}

hipError_t launch_search_fused(const Geometry &g, const WorkspaceOffsets &wo, const EncodeBatch &batch, int n_tensors,
                               hipStream_t stream)
{
    dim3 grid((g.T + g.search_rows - 1) / g.search_rows, g.fused_by_head ? g.H : g.B * g.H, (unsigned)n_tensors);
    const int waves = search_waves_for(g.S16, g.A16, g.D, g.row_words, g.search_rows);
    const size_t lds = search_lds_bytes(g.S16, g.A16, g.D, g.row_words, waves, g.search_rows);
    if (g.D == 4 * kChunksPerRow) {
        if (waves == 8)
            hipLaunchKernelGGL((k_search<8, kSearchRowsSmall, true>), grid, dim3(512), lds, stream, g, wo, batch);
        else
            hipLaunchKernelGGL((k_search<4, kSearchRowsSmall, true>), grid, dim3(256), lds, stream, g, wo, batch);
    } else {
        if (waves == 8)
            hipLaunchKernelGGL((k_search_flat<8, kSearchRowsSmall, true>), grid, dim3(512), lds, stream, g, wo, batch);
        else
            hipLaunchKernelGGL((k_search_flat<4, kSearchRowsSmall, true>), grid, dim3(256), lds, stream, g, wo, batch);
    }
    return hipGetLastError();
}

hipError_t launch_search(const Geometry &g, const WorkspaceOffsets &wo, const EncodeBatch &batch, int n_tensors,
                         hipStream_t stream)
{
    dim3 grid((g.T + g.search_rows - 1) / g.search_rows, g.B * g.H, (unsigned)n_tensors);
    const bool full = g.D == 4 * kChunksPerRow;
    const int waves = search_waves_for(g.S16, g.A16, g.D, g.row_words, g.search_rows);
    const size_t lds = search_lds_bytes(g.S16, g.A16, g.D, g.row_words, waves, g.search_rows);
    if (g.A16 > 0)
        hipLaunchKernelGGL(k_prepare_operands, dim3((g.A16 * kATiles * 64 + kThreads - 1) / kThreads, g.H, (unsigned)n_tensors),
                           dim3(kThreads), 0, stream, g, wo, batch);
    const bool large = g.search_rows == kSearchRowsLarge;
#define HQMQ_LAUNCH(KERNEL, W, R) hipLaunchKernelGGL((KERNEL<W, R>), grid, dim3(64 * W), lds, stream, g, wo, batch)
    if (g.A16 == 0) {
        // more secondaries than the matrix-core screen holds: 64 rows on 4 waves, every chunk scored in fp32
        if (full)
            hipLaunchKernelGGL((k_search<4, kSearchRowsSmall, false, false>), grid, dim3(256), lds, stream, g, wo, batch);
        else
            hipLaunchKernelGGL((k_search_flat<4, kSearchRowsSmall, false, false>), grid, dim3(256), lds, stream, g, wo, batch);
    } else if (full) {
        if (g.search_rows == kSearchRowsHuge)  // only chosen together with 16 waves
            HQMQ_LAUNCH(k_search, 16, kSearchRowsHuge);
        else if (large && waves == 16)
            HQMQ_LAUNCH(k_search, 16, kSearchRowsLarge);
        else if (large && waves == 8)
            HQMQ_LAUNCH(k_search, 8, kSearchRowsLarge);
        else if (large)
            HQMQ_LAUNCH(k_search, 4, kSearchRowsLarge);
        else if (waves == 8)
            HQMQ_LAUNCH(k_search, 8, kSearchRowsSmall);
        else
            HQMQ_LAUNCH(k_search, 4, kSearchRowsSmall);
    } else {
        // 256 rows per workgroup are only chosen when two 4-wave workgroups fit a CU
        if (g.search_rows == kSearchRowsHuge)  // only chosen together with 16 waves
            HQMQ_LAUNCH(k_search_flat, 16, kSearchRowsHuge);
        else if (large && waves == 16)
            HQMQ_LAUNCH(k_search_flat, 16, kSearchRowsLarge);
        else if (large)
            HQMQ_LAUNCH(k_search_flat, 4, kSearchRowsLarge);
        else if (waves == 8)
            HQMQ_LAUNCH(k_search_flat, 8, kSearchRowsSmall);
        else
            HQMQ_LAUNCH(k_search_flat, 4, kSearchRowsSmall);
    }
#undef HQMQ_LAUNCH
    return hipGetLastError();
}

}  // namespace hqmq
