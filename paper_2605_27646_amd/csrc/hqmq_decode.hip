// HQMQ decode (paper Alg. 1 "Decode", App. D "Decode"): x_hat = r_hat * (P_p (x) q_s) with
// r_hat = r_q * sigma / (2^b_r - 1); flagged chunks are restored verbatim from the outlier list.
//
// HBM-bound: per chunk it reads w/8 bytes of code (+ 1/8 flag, 1/16 scale, 1/8 offset) and
// writes 8 bytes of fp16.  One lane per chunk, two rows per wave, so a wave's store is 512
// contiguous bytes.  The head's secondaries sit in LDS; the primary is never looked up: P_p is
// rebuilt from the bits of p (a signed axis or a sign pattern times 1/2) and multiplied out.
#include "hqmq_device.h"

namespace hqmq {

__global__ __launch_bounds__(kThreads) void k_decode(Geometry g, EncodedPtrs enc,
                                                     uint64_t outlier_capacity,
                                                     const float *__restrict__ sec,
                                                     _Float16 *__restrict__ out)
{
    extern __shared__ float secl[];  // [S][4]
    const int tid = threadIdx.x;
    const int seg = blockIdx.y, b = seg / g.H, h = seg % g.H;
    const float *sec_h = sec + (size_t)h * g.S * 4;
    for (int s = tid; s < g.S; s += kThreads)
        *reinterpret_cast<float4_t *>(secl + 4 * s) = *reinterpret_cast<const float4_t *>(sec_h + 4 * s);
    __syncthreads();

    const int c = tid & 31, sub = tid >> 5;
    const int t0 = blockIdx.x * kDecodeRows;
    const int t1 = min(g.T, t0 + kDecodeRows);
    const int64_t row0 = (int64_t)seg * g.T;
    _Float16 *obase = out + (int64_t)b * g.sb + (int64_t)h * g.sh + 4 * c;

    const uint32_t w = g.w, w_idx = g.w_idx;
    const uint32_t bitpos = (uint32_t)c * w;
    const uint32_t d0 = bitpos >> 5, sh = bitpos & 31;
    const uint32_t d1 = (d0 + 1 < w) ? d0 + 1 : d0;
    const uint32_t code_mask = (1u << w) - 1u, idx_mask = (1u << w_idx) - 1u;
    const float inv_L = 1.0f / (float)((1 << g.b_r) - 1);

    for (int t = t0 + sub; t < t1; t += 8) {
        const int64_t R = row0 + t;
        const uint32_t *cw = enc.codes + R * w;
        const uint32_t lo = cw[d0], hi = cw[d1];
        const uint32_t word = enc.flags[R];
        const float sigma = (float)__builtin_bit_cast(_Float16, enc.sigma[R]);
        half4_t o;
        if ((word >> c) & 1u) {
            uint64_t pos = (uint64_t)enc.row_off[R] + __popc(word & ((1u << c) - 1u));
            uint2 raw = make_uint2(0u, 0u);
            if (pos < outlier_capacity)
                raw = *reinterpret_cast<const uint2 *>(enc.outliers + 4 * pos);
            o = __builtin_bit_cast(half4_t, raw);
        } else {
            const uint32_t code = __builtin_amdgcn_alignbit(hi, lo, sh) & code_mask;
            const uint32_t k = code & idx_mask, rq = code >> w_idx;
            const uint32_t p = (g.S == 1) ? k : __umulhi(k, g.s_magic);
            const uint32_t s = k - p * (uint32_t)g.S;
            const float4_t q = *reinterpret_cast<const float4_t *>(secl + 4 * s);
            // P_p from the bits of p
            float P0, P1, P2, P3;
            if (p < 8) {
                const float sg = (p & 1u) ? -1.f : 1.f;
                const uint32_t ax = p >> 1;
                P0 = ax == 0 ? sg : 0.f;
                P1 = ax == 1 ? sg : 0.f;
                P2 = ax == 2 ? sg : 0.f;
                P3 = ax == 3 ? sg : 0.f;
            } else {
                const uint32_t bt = p - 8;
                P0 = (bt & 8u) ? -0.5f : 0.5f;
                P1 = (bt & 4u) ? -0.5f : 0.5f;
                P2 = (bt & 2u) ? -0.5f : 0.5f;
                P3 = (bt & 1u) ? -0.5f : 0.5f;
            }
            // Hamilton product P (x) q
            const float c0 = P0 * q[0] - P1 * q[1] - P2 * q[2] - P3 * q[3];
            const float c1 = P0 * q[1] + P1 * q[0] + P2 * q[3] - P3 * q[2];
            const float c2 = P0 * q[2] - P1 * q[3] + P2 * q[0] + P3 * q[1];
            const float c3 = P0 * q[3] + P1 * q[2] - P2 * q[1] + P3 * q[0];
            const float rh = ((float)rq * sigma) * inv_L;
            const float lim = 65504.f;
            o[0] = (_Float16)fminf(fmaxf(rh * c0, -lim), lim);
            o[1] = (_Float16)fminf(fmaxf(rh * c1, -lim), lim);
            o[2] = (_Float16)fminf(fmaxf(rh * c2, -lim), lim);
            o[3] = (_Float16)fminf(fmaxf(rh * c3, -lim), lim);
        }
        *reinterpret_cast<uint2 *>(obase + (int64_t)t * g.st) = __builtin_bit_cast(uint2, o);
    }
}

hipError_t launch_decode(const Geometry &g, const EncodedPtrs &enc, uint64_t outlier_capacity,
                         const float *sec, _Float16 *out, hipStream_t stream)
{
    dim3 grid((g.T + kDecodeRows - 1) / kDecodeRows, g.B * g.H);
    size_t lds = (size_t)g.S * 4 * sizeof(float);
    hipLaunchKernelGGL(k_decode, grid, dim3(kThreads), lds, stream, g, enc, outlier_capacity, sec, out);
    return hipGetLastError();
}

}  // namespace hqmq
