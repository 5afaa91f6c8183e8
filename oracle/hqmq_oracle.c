/*
 * HQMQ reference oracle (plain C, IEEE fp64).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, literal statement of what the
 * HQMQ KV-cache encode / decode path computes.  It exists so that the GPU library can
 * be checked against it; nothing in the product path may include, link or call it, and
 * it shares no code, tables or constants with the GPU sources.
 *
 * Every function follows the paper's own statement of the step it implements:
 *   - Hurwitz primary codebook 2T ............ Sec. 2 "Quaternions and the 24-cell",
 *                                              App. D "The Hurwitz primary codebook 2T"
 *   - joint codebook q_p * q_s ............... Eq. (1)
 *   - chunking, r = |x|, u = x / r ........... Sec. 3 "Setup", Alg. 1 (encode)
 *   - exhaustive argmax over p in [24], s in [S] ... Alg. 1 (encode), App. D "Encode"
 *   - radius quantiser ....................... Sec. 3 "Radius quantization", Alg. 1
 *   - Med3x outlier extraction ............... Sec. 3 "Median-multiplier outlier
 *                                              extraction", Alg. 1, App. D "Outlier extraction"
 *   - decode ................................. Alg. 1 (decode), App. D "Decode"
 *   - secondary codebook initialisation ...... App. D "Secondary codebook initialization"
 *   - single-query attention over the
 *     reconstructed K and V .................. App. F (fused attention: softmax(Q K^T scale) V)
 *
 * Where the paper leaves a choice open (median of an even count, tie-break, rounding,
 * bit layout, ...) the reading taken is stated at the function that needs it.
 *
 * There is no blocking, no algebraic shortcut (no isometry rewrite, no closed-form
 * nearest vertex), no radix select: medians come from a library sort, the search scores
 * all 24*S products one by one.  Arithmetic order is written out and the file is
 * compiled with -ffp-contract=off so the compiler cannot fuse or reorder it.
 *
 * Tensor layout: X is fp16 (passed as uint16 bit patterns) of logical shape
 * [B, H, T, 4*Nc], last axis contiguous, 1 <= Nc <= 32 chunks per row (head dimensions 64,
 * 96 and 128 of the paper's models give Nc = 16, 24, 32; a head dimension that is not a
 * multiple of 4 is zero-padded to the next one by the caller and cut back after decode:
 * App. "Padding wrapper for d_h not divisible by 4").
 * A "row" is one (b, h, t) vector; its linear index is (b*H + h)*T + t; chunk c of a row
 * is elements 4c .. 4c+3 and its linear chunk index is row*Nc + c.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define HQO_NC_MAX 32 /* most chunks a row may have (head dimension 128) */

/* ------------------------------------------------------------------------------------
 * fp16 <-> fp64
 * ---------------------------------------------------------------------------------- */

/* Exact widening of an IEEE binary16 bit pattern. */
double hqo_half_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1f;
    int m = h & 0x3ff;
    double v;
    if (e == 0)
        v = ldexp((double)m, -24); /* subnormal or zero: m * 2^-24 */
    else if (e == 31)
        v = (m == 0) ? INFINITY : NAN;
    else
        v = ldexp((double)(m + 1024), e - 25); /* (1 + m/1024) * 2^(e-15) */
    return sign ? -v : v;
}

/* Round a double to the nearest binary16 value, ties to even, saturating at the largest
 * finite value 65504 instead of overflowing to infinity.  Written from the definition of
 * the format: within a binade [2^e, 2^(e+1)) the representable values are the integer
 * multiples of 2^(e-10); below 2^-14 the spacing stays 2^-24. */
uint16_t hqo_double_to_half(double v)
{
    uint16_t sign = 0;
    if (v != v)
        return 0x7e00;
    if (signbit(v)) {
        sign = 0x8000;
        v = -v;
    }
    if (v >= 65504.0)
        return (uint16_t)(sign | 0x7bff);
    if (v == 0.0)
        return sign;
    int e;
    (void)frexp(v, &e); /* v = f * 2^e with f in [0.5, 1)  ->  binade exponent is e-1 */
    e -= 1;
    if (e < -14)
        e = -14;
    /* n = v / 2^(e-10) is exact (power-of-two scaling); nearbyint rounds half to even in
     * the default rounding mode. */
    double n = nearbyint(ldexp(v, 10 - e));
    /* n in [0, 2048]; 2048 means the value rounded up into the next binade. */
    long ni = (long)n;
    if (e == -14 && ni < 1024)
        return (uint16_t)(sign | ni); /* subnormal (or zero) */
    if (ni == 2048) {
        ni = 1024;
        e += 1;
    }
    if (e > 15)
        return (uint16_t)(sign | 0x7bff);
    return (uint16_t)(sign | ((e + 15) << 10) | (ni - 1024));
}

/* ------------------------------------------------------------------------------------
 * Quaternion algebra and the primary codebook 2T
 * ---------------------------------------------------------------------------------- */

/* Hamilton product, components ordered (real, i, j, k). */
void hqo_hamilton(const double a[4], const double b[4], double out[4])
{
    double a1 = a[0], b1 = a[1], c1 = a[2], d1 = a[3];
    double a2 = b[0], b2 = b[1], c2 = b[2], d2 = b[3];
    out[0] = a1 * a2 - b1 * b2 - c1 * c2 - d1 * d2;
    out[1] = a1 * b2 + b1 * a2 + c1 * d2 - d1 * c2;
    out[2] = a1 * c2 - b1 * d2 + c1 * a2 + d1 * b2;
    out[3] = a1 * d2 + b1 * c2 - c1 * b2 + d1 * a2;
}

/* The 24 unit Hurwitz quaternions in the order this build fixes (the paper lists the
 * set, not an order):  p = 0..7  ->  +1, -1, +i, -i, +j, -j, +k, -k;
 * p = 8 + 8*b0 + 4*b1 + 2*b2 + b3  ->  1/2 * ((-1)^b0, (-1)^b1, (-1)^b2, (-1)^b3). */
void hqo_primary(int p, double q[4])
{
    int i;
    if (p < 0 || p >= 24) { /* the group has 24 elements: any other index names none */
        for (i = 0; i < 4; ++i)
            q[i] = NAN;
        return;
    }
    if (p < 8) {
        for (i = 0; i < 4; ++i)
            q[i] = 0.0;
        q[p / 2] = (p % 2) ? -1.0 : 1.0;
    } else {
        int bits = p - 8;
        for (i = 0; i < 4; ++i)
            q[i] = ((bits >> (3 - i)) & 1) ? -0.5 : 0.5;
    }
}

/* Joint codeword k = p*S + s of one head:  P[p] (x) sec[s], the primary on the left
 * (Eq. 1, Alg. 1).  The secondary is used exactly as stored in fp32. */
void hqo_codeword(const float *sec, int S, int k, double c[4])
{
    double P[4], q[4];
    int p = k / S, s = k % S, i;
    hqo_primary(p, P);
    for (i = 0; i < 4; ++i)
        q[i] = (double)sec[4 * s + i];
    hqo_hamilton(P, q, c);
}

/* ------------------------------------------------------------------------------------
 * Secondary codebooks: S i.i.d. N(0, I4) draws, normalised, per (layer, role, head).
 * The paper fixes only the distribution and "a seed"; the generator below is this
 * build's choice and the GPU library's host code implements the same one separately:
 * a counter-based SplitMix64 stream, Box-Muller in fp64, normalise in fp64, round to
 * fp32; a draw with squared norm below 1e-12 is redrawn with the next attempt counter.
 * ---------------------------------------------------------------------------------- */

static uint64_t hqo_mix64(uint64_t z)
{
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}

/* n-th output of the SplitMix64 sequence whose state starts at `start`. */
static uint64_t hqo_stream(uint64_t start, uint64_t n)
{
    return hqo_mix64(start + (n + 1) * 0x9E3779B97F4A7C15ULL);
}

void hqo_build_codebooks(uint64_t seed, int n_layers, int n_heads, int S, float *sec)
{
    const double two_pi = 6.283185307179586476925286766559;
    uint64_t start = hqo_mix64(seed);
    int64_t total = (int64_t)n_layers * 2 * n_heads * S;
    for (int64_t idx = 0; idx < total; ++idx) {
        for (uint64_t attempt = 0; attempt < 16; ++attempt) {
            double g[4];
            for (int pair = 0; pair < 2; ++pair) {
                uint64_t n = (((uint64_t)idx * 16 + attempt) * 2 + (uint64_t)pair) * 2;
                uint64_t w1 = hqo_stream(start, n), w2 = hqo_stream(start, n + 1);
                double u1 = ((double)(w1 >> 11) + 1.0) * 0x1.0p-53; /* (0, 1] */
                double u2 = (double)(w2 >> 11) * 0x1.0p-53;         /* [0, 1) */
                double rad = sqrt(-2.0 * log(u1));
                g[2 * pair] = rad * cos(two_pi * u2);
                g[2 * pair + 1] = rad * sin(two_pi * u2);
            }
            double n2 = ((g[0] * g[0] + g[1] * g[1]) + g[2] * g[2]) + g[3] * g[3];
            if (n2 < 1e-12 && attempt < 15)
                continue;
            double nrm = sqrt(n2);
            for (int i = 0; i < 4; ++i)
                sec[4 * idx + i] = (float)(g[i] / nrm);
            break;
        }
    }
}

/* ------------------------------------------------------------------------------------
 * Encode steps
 * ---------------------------------------------------------------------------------- */

/* Squared chunk norms.  Inputs are widened exactly; each product of two fp16 values is
 * exact in fp64, so the only roundings are the three additions, taken left to right. */
void hqo_norm2(const uint16_t *x, int64_t n_chunks, double *r2)
{
    for (int64_t i = 0; i < n_chunks; ++i) {
        double x0 = hqo_half_to_double(x[4 * i + 0]);
        double x1 = hqo_half_to_double(x[4 * i + 1]);
        double x2 = hqo_half_to_double(x[4 * i + 2]);
        double x3 = hqo_half_to_double(x[4 * i + 3]);
        r2[i] = ((x0 * x0 + x1 * x1) + x2 * x2) + x3 * x3;
    }
}

static int hqo_cmp_double(const void *a, const void *b)
{
    double x = *(const double *)a, y = *(const double *)b;
    return (x > y) - (x < y);
}

/* Lower median: element (n-1)/2 of the sorted list (an actual data value; the paper
 * says "median" and every batch here has an even count).  Returns 0 for n == 0. */
double hqo_lower_median(const double *v, int64_t n)
{
    if (n <= 0)
        return 0.0;
    double *tmp = (double *)malloc((size_t)n * sizeof(double));
    memcpy(tmp, v, (size_t)n * sizeof(double));
    qsort(tmp, (size_t)n, sizeof(double), hqo_cmp_double);
    double m = tmp[(n - 1) / 2];
    free(tmp);
    return m;
}

/* Median of the squared chunk norms of each head, over all (b, t, c) of the batch:
 * "per (layer, head, role) ... across the current batch".  Squaring is monotone on
 * non-negative norms, so the median of r^2 is the square of the median of r. */
void hqo_head_medians(const double *r2, int B, int H, int T, int Nc, double *m2)
{
    int64_t per_bh = (int64_t)T * Nc;
    double *buf = (double *)malloc((size_t)B * (size_t)per_bh * sizeof(double));
    for (int h = 0; h < H; ++h) {
        for (int b = 0; b < B; ++b)
            memcpy(buf + (int64_t)b * per_bh, r2 + ((int64_t)b * H + h) * per_bh,
                   (size_t)per_bh * sizeof(double));
        m2[h] = hqo_lower_median(buf, (int64_t)B * per_bh);
    }
    free(buf);
}

/* Outlier test r > C * r_med, strict, evaluated on squares: r^2 > fl(fl(C*C) * m2[h])
 * with C widened from fp32.  use_outliers == 0 switches extraction off (no flags). */
void hqo_flags(const double *r2, const double *m2, float C, int use_outliers, int B, int H,
               int T, int Nc, uint8_t *flag)
{
    double c = (double)C;
    double c2 = c * c;
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < H; ++h) {
            double thr = c2 * m2[h];
            int64_t base = ((int64_t)b * H + h) * T * Nc;
            for (int64_t i = 0; i < (int64_t)T * Nc; ++i)
                flag[base + i] = (use_outliers && r2[base + i] > thr) ? 1 : 0;
        }
}

/* Outlier storage: one flag bit per chunk (bit c of the row's word), the flagged chunks'
 * four fp16 bit patterns copied verbatim in ascending linear chunk order, the exclusive
 * prefix count per row (row_off has n_rows+1 entries), and the count per head
 * (n_out[0..H-1]) plus the total (n_out[H]).  Returns the total; writes at most `cap`
 * payload entries. */
int64_t hqo_extract_outliers(const uint16_t *x, const uint8_t *flag, int B, int H, int T, int Nc,
                             uint32_t *flag_words, uint32_t *row_off, uint32_t *n_out,
                             uint16_t *payload, int64_t cap)
{
    int64_t n_rows = (int64_t)B * H * T, count = 0;
    for (int h = 0; h <= H; ++h)
        n_out[h] = 0;
    for (int64_t row = 0; row < n_rows; ++row) {
        int h = (int)((row / T) % H);
        uint32_t word = 0;
        row_off[row] = (uint32_t)count;
        for (int c = 0; c < Nc; ++c) {
            int64_t chunk = row * Nc + c;
            if (flag[chunk]) {
                word |= (uint32_t)1 << c;
                if (count < cap)
                    memcpy(payload + 4 * count, x + 4 * chunk, 4 * sizeof(uint16_t));
                ++count;
                ++n_out[h];
            }
        }
        flag_words[row] = word;
    }
    row_off[n_rows] = (uint32_t)count;
    n_out[H] = (uint32_t)count;
    return count;
}

/* Per-row radius scale: the largest norm among the row's unflagged chunks ("per-token-max
 * scale", one fp16 per (b, h, t)), rounded to fp16 ties-to-even, saturating.  Outliers
 * are excluded because they are stored separately and would otherwise set the scale. */
void hqo_row_sigma(const double *r2, const uint8_t *flag, int64_t n_rows, int Nc, uint16_t *sigma16)
{
    for (int64_t row = 0; row < n_rows; ++row) {
        double smax = 0.0;
        for (int c = 0; c < Nc; ++c) {
            int64_t chunk = row * Nc + c;
            if (!flag[chunk]) {
                double r = sqrt(r2[chunk]);
                if (r > smax)
                    smax = r;
            }
        }
        sigma16[row] = hqo_double_to_half(smax);
    }
}

/* Score of one joint codeword against the unit direction of chunk x (fp16 bit
 * patterns):  < x / |x| , P[p] (x) sec[s] >, summed left to right. */
double hqo_score(const uint16_t *x4, const float *sec, int S, int k)
{
    double x[4], u[4], c[4];
    for (int i = 0; i < 4; ++i)
        x[i] = hqo_half_to_double(x4[i]);
    double r = sqrt(((x[0] * x[0] + x[1] * x[1]) + x[2] * x[2]) + x[3] * x[3]);
    for (int i = 0; i < 4; ++i)
        u[i] = x[i] / r;
    hqo_codeword(sec, S, k, c);
    return ((u[0] * c[0] + u[1] * c[1]) + u[2] * c[2]) + u[3] * c[3];
}

/* Exhaustive nearest-codeword search for one chunk: all 24*S products, p outer, s inner,
 * flat index k = p*S + s, a candidate replaces the incumbent only when strictly greater
 * (so the lowest k wins an exact tie).  Also returns the best score and the best score
 * among all other k (for the near-tie rule of the parity tests).  A zero chunk has no
 * direction: k = 0, best = second = 0. */
void hqo_search_chunk(const uint16_t *x4, const float *sec, int S, int32_t *k_out,
                      double *best_out, double *second_out)
{
    double x[4], u[4];
    for (int i = 0; i < 4; ++i)
        x[i] = hqo_half_to_double(x4[i]);
    double r2 = ((x[0] * x[0] + x[1] * x[1]) + x[2] * x[2]) + x[3] * x[3];
    if (r2 == 0.0) {
        *k_out = 0;
        *best_out = 0.0;
        *second_out = 0.0;
        return;
    }
    double r = sqrt(r2);
    for (int i = 0; i < 4; ++i)
        u[i] = x[i] / r;
    double best = -INFINITY, second = -INFINITY;
    int32_t kb = 0;
    for (int p = 0; p < 24; ++p) {
        double P[4];
        hqo_primary(p, P);
        for (int s = 0; s < S; ++s) {
            double q[4], c[4];
            for (int i = 0; i < 4; ++i)
                q[i] = (double)sec[4 * s + i];
            hqo_hamilton(P, q, c);
            double score = ((u[0] * c[0] + u[1] * c[1]) + u[2] * c[2]) + u[3] * c[3];
            if (score > best) {
                second = best;
                best = score;
                kb = p * S + s;
            } else if (score > second) {
                second = score;
            }
        }
    }
    *k_out = kb;
    *best_out = best;
    *second_out = second;
}

/* Radius code:  r_q = clamp(rint(r * L / sigma), 0, L),  L = 2^b_r - 1, rint = round half
 * to even, sigma = the STORED fp16 scale widened to fp64 (so that encode and decode use
 * the same number); sigma == 0 gives 0. */
int32_t hqo_radius_code(double r2, uint16_t sigma16, int b_r)
{
    double L = (double)((1 << b_r) - 1);
    double sigma = hqo_half_to_double(sigma16);
    if (sigma == 0.0)
        return 0;
    double q = nearbyint((sqrt(r2) * L) / sigma);
    if (q < 0.0)
        q = 0.0;
    if (q > L)
        q = L;
    return (int32_t)q;
}

/* Smallest j with 2^j >= 24*S: the index width ceil(log2(24 S)). */
int hqo_index_bits(int S)
{
    int j = 0;
    while (((int64_t)1 << j) < (int64_t)24 * S)
        ++j;
    return j;
}

/* Search + radius code for the selected rows of a tensor (sel == NULL: every row).
 * Flagged chunks and rows not selected get k = -1 and r_q = -1 here; best/second are
 * left at 0 for them.  The loop over rows is independent per row and is the only thing
 * parallelised (a plain parallel-for) so the oracle finishes in reasonable time. */
void hqo_search_rows(const uint16_t *x, const uint8_t *flag, const uint16_t *sigma16,
                     const float *sec_all /* [H][S][4] */, int B, int H, int T, int Nc, int S, int b_r,
                     const uint8_t *sel, int32_t *k, double *best, double *second,
                     int32_t *rq)
{
    int64_t n_rows = (int64_t)B * H * T;
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t row = 0; row < n_rows; ++row) {
        int h = (int)((row / T) % H);
        const float *sec = sec_all + (int64_t)h * S * 4;
        for (int c = 0; c < Nc; ++c) {
            int64_t chunk = row * Nc + c;
            k[chunk] = -1;
            rq[chunk] = -1;
            best[chunk] = 0.0;
            second[chunk] = 0.0;
            if ((sel && !sel[row]) || flag[chunk])
                continue;
            double r2;
            hqo_norm2(x + 4 * chunk, 1, &r2);
            hqo_search_chunk(x + 4 * chunk, sec, S, &k[chunk], &best[chunk], &second[chunk]);
            rq[chunk] = (r2 == 0.0) ? 0 : hqo_radius_code(r2, sigma16[row], b_r);
        }
    }
}

/* ------------------------------------------------------------------------------------
 * Code words and their packing.  code = (r_q << w_idx) | k, width w = w_idx + b_r; a
 * flagged chunk carries code 0.  The Nc codes of a row are concatenated LSB first: chunk
 * c occupies bits [c*w, (c+1)*w) of the row's ceil(Nc*w/32) little-endian 32-bit words
 * (w words when Nc = 32); the unused high bits of the last word are zero.
 * ---------------------------------------------------------------------------------- */

int hqo_row_words(int Nc, int w)
{
    return (Nc * w + 31) / 32;
}

void hqo_pack_row(const uint32_t *code32 /* [Nc] */, int Nc, int w, uint32_t *words /* [row_words] */)
{
    for (int i = 0; i < hqo_row_words(Nc, w); ++i)
        words[i] = 0;
    for (int c = 0; c < Nc; ++c)
        for (int bit = 0; bit < w; ++bit)
            if ((code32[c] >> bit) & 1u) {
                int pos = c * w + bit;
                words[pos / 32] |= (uint32_t)1 << (pos % 32);
            }
}

void hqo_unpack_row(const uint32_t *words /* [row_words] */, int Nc, int w, uint32_t *code32 /* [Nc] */)
{
    for (int c = 0; c < Nc; ++c) {
        uint32_t v = 0;
        for (int bit = 0; bit < w; ++bit) {
            int pos = c * w + bit;
            if ((words[pos / 32] >> (pos % 32)) & 1u)
                v |= (uint32_t)1 << bit;
        }
        code32[c] = v;
    }
}

/* Pack rows whose k / r_q are known (k >= 0 or flagged); rows with an unflagged k < 0
 * (not searched) are written as zeros. */
void hqo_pack_rows(const int32_t *k, const int32_t *rq, const uint8_t *flag, int64_t n_rows, int Nc,
                   int S, int b_r, uint32_t *codes /* [n_rows][row_words] */)
{
    int w_idx = hqo_index_bits(S), w = w_idx + b_r;
    int rw = hqo_row_words(Nc, w);
    for (int64_t row = 0; row < n_rows; ++row) {
        uint32_t code32[HQO_NC_MAX];
        for (int c = 0; c < Nc; ++c) {
            int64_t chunk = row * Nc + c;
            if (flag[chunk] || k[chunk] < 0)
                code32[c] = 0;
            else
                code32[c] = ((uint32_t)rq[chunk] << w_idx) | (uint32_t)k[chunk];
        }
        hqo_pack_row(code32, Nc, w, codes + row * rw);
    }
}

/* ------------------------------------------------------------------------------------
 * Decode:  x_hat = r_hat * (P[p] (x) sec[s]),  r_hat = r_q * sigma / L,  rounded to fp16
 * (ties to even, saturating); flagged chunks take their stored fp16 payload verbatim, the
 * j-th flagged chunk of a row sitting at payload[row_off[row] + j].
 * Also returns r_hat per chunk (fp64, 0 for flagged chunks) for tolerance checks, and, when
 * out64 is given, the reconstruction before the final fp16 rounding (flagged chunks: their
 * fp16 payload widened).
 * ---------------------------------------------------------------------------------- */
void hqo_decode64(const uint32_t *codes, const uint16_t *sigma16, const uint32_t *flag_words,
                  const uint32_t *row_off, const uint16_t *payload, const float *sec_all, int B,
                  int H, int T, int Nc, int S, int b_r, uint16_t *out, double *r_hat, double *out64);

void hqo_decode(const uint32_t *codes, const uint16_t *sigma16, const uint32_t *flag_words,
                const uint32_t *row_off, const uint16_t *payload, const float *sec_all, int B,
                int H, int T, int Nc, int S, int b_r, uint16_t *out /* [rows][4 Nc] */, double *r_hat)
{
    hqo_decode64(codes, sigma16, flag_words, row_off, payload, sec_all, B, H, T, Nc, S, b_r, out, r_hat, 0);
}

void hqo_decode64(const uint32_t *codes, const uint16_t *sigma16, const uint32_t *flag_words,
                const uint32_t *row_off, const uint16_t *payload, const float *sec_all, int B,
                  int H, int T, int Nc, int S, int b_r, uint16_t *out /* [rows][4 Nc] */, double *r_hat,
                  double *out64 /* [rows][4 Nc] or NULL */)
{
    int w_idx = hqo_index_bits(S), w = w_idx + b_r;
    int rw = hqo_row_words(Nc, w);
    double L = (double)((1 << b_r) - 1);
    int64_t n_rows = (int64_t)B * H * T;
    for (int64_t row = 0; row < n_rows; ++row) {
        int h = (int)((row / T) % H);
        const float *sec = sec_all + (int64_t)h * S * 4;
        uint32_t code32[HQO_NC_MAX];
        hqo_unpack_row(codes + row * rw, Nc, w, code32);
        double sigma = hqo_half_to_double(sigma16[row]);
        int64_t next = row_off[row];
        for (int c = 0; c < Nc; ++c) {
            int64_t chunk = row * Nc + c;
            if ((flag_words[row] >> c) & 1u) {
                memcpy(out + 4 * chunk, payload + 4 * next, 4 * sizeof(uint16_t));
                if (out64)
                    for (int i = 0; i < 4; ++i)
                        out64[4 * chunk + i] = hqo_half_to_double(payload[4 * next + i]);
                ++next;
                if (r_hat)
                    r_hat[chunk] = 0.0;
                continue;
            }
            int32_t kk = (int32_t)(code32[c] & (((uint32_t)1 << w_idx) - 1u));
            int32_t q = (int32_t)(code32[c] >> w_idx);
            double rh = ((double)q * sigma) / L;
            double cw[4];
            hqo_codeword(sec, S, kk, cw);
            for (int i = 0; i < 4; ++i) {
                out[4 * chunk + i] = hqo_double_to_half(rh * cw[i]);
                if (out64)
                    out64[4 * chunk + i] = rh * cw[i];
            }
            if (r_hat)
                r_hat[chunk] = rh;
        }
    }
}

/* ------------------------------------------------------------------------------------
 * Single-query attention over a reconstructed cache (the paper's fused HQMQ-attention kernel,
 * App. F: S = Q K^T scale, O = softmax(S) V with K and V decoded inside the loop; here for one
 * query token per sequence, the decode step of generation).  q: fp16 [B][Hq][D]; K, V: fp64
 * [B][H][T][D] as returned by hqo_decode64 (reconstruction before fp16 rounding, outliers as
 * stored); query head hq reads kv head hq / (Hq / H) (grouped-query attention).  Plain softmax
 * with the row maximum subtracted, everything in fp64; out16 = result rounded to fp16.  lse64
 * (optional): the natural logarithm of the softmax denominator sum_t exp(scale * <q, K_t>), as
 * maximum + log of the shifted sum.
 * ---------------------------------------------------------------------------------- */
void hqo_attend_lse(const uint16_t *q, const double *K, const double *V, int B, int Hq, int H, int T,
                    int D, double scale, uint16_t *out16, double *out64, double *lse64);
void hqo_attend_masked(const uint16_t *q, const double *K, const double *V, int B, int Hq, int H, int T,
                       int D, double scale, const int32_t *visible, uint16_t *out16, double *out64,
                       double *lse64);

void hqo_attend(const uint16_t *q, const double *K, const double *V, int B, int Hq, int H, int T,
                int D, double scale, uint16_t *out16, double *out64)
{
    hqo_attend_lse(q, K, V, B, Hq, H, T, D, scale, out16, out64, 0);
}

void hqo_attend_lse(const uint16_t *q, const double *K, const double *V, int B, int Hq, int H, int T,
                    int D, double scale, uint16_t *out16, double *out64, double *lse64)
{
    hqo_attend_masked(q, K, V, B, Hq, H, T, D, scale, 0, out16, out64, lse64);
}

/* The same with a causal limit: query head hq of sequence b attends to the tokens t < visible[b*Hq + hq]
 * only (App. F: the fused kernel masks causally); visible == NULL or a value >= T: all T tokens.  A head
 * that sees no token has an empty softmax: output 0, lse = -infinity. */
void hqo_attend_masked(const uint16_t *q, const double *K, const double *V, int B, int Hq, int H, int T_all,
                       int D, double scale, const int32_t *visible, uint16_t *out16, double *out64,
                       double *lse64)
{
    int G = Hq / H;
    double *p = (double *)malloc((size_t)(T_all > 0 ? T_all : 1) * sizeof(double));
    for (int b = 0; b < B; ++b)
        for (int hq = 0; hq < Hq; ++hq) {
            int h = hq / G;
            const double *Kh = K + ((int64_t)b * H + h) * T_all * D;
            const double *Vh = V + ((int64_t)b * H + h) * T_all * D;
            const uint16_t *qv = q + ((int64_t)b * Hq + hq) * D;
            int T = T_all; /* tokens this head sees */
            if (visible && visible[(int64_t)b * Hq + hq] < T_all)
                T = visible[(int64_t)b * Hq + hq] < 0 ? 0 : visible[(int64_t)b * Hq + hq];
            if (T == 0) {
                if (lse64)
                    lse64[(int64_t)b * Hq + hq] = -INFINITY;
                for (int d = 0; d < D; ++d) {
                    int64_t at = ((int64_t)b * Hq + hq) * D + d;
                    if (out64)
                        out64[at] = 0.0;
                    out16[at] = 0;
                }
                continue;
            }
            double m = -INFINITY;
            for (int t = 0; t < T; ++t) {
                double s = 0.0;
                for (int d = 0; d < D; ++d)
                    s += hqo_half_to_double(qv[d]) * Kh[(int64_t)t * D + d];
                p[t] = scale * s;
                if (p[t] > m)
                    m = p[t];
            }
            double l = 0.0;
            for (int t = 0; t < T; ++t) {
                p[t] = exp(p[t] - m);
                l += p[t];
            }
            if (lse64)
                lse64[(int64_t)b * Hq + hq] = m + log(l);
            for (int d = 0; d < D; ++d) {
                double o = 0.0;
                for (int t = 0; t < T; ++t)
                    o += p[t] * Vh[(int64_t)t * D + d];
                o /= l;
                int64_t at = ((int64_t)b * Hq + hq) * D + d;
                if (out64)
                    out64[at] = o;
                out16[at] = hqo_double_to_half(o);
            }
        }
    free(p);
}
