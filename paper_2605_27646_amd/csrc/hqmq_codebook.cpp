// hqmq_build_codebooks: the seeded secondary codebooks (paper App. D "Secondary codebook
// initialization": i.i.d. 4-dim standard Gaussians, normalised; the seed is fixed when the
// cache is set up and the codebooks are never trained).
//
// Generator: counter based, so any entry can be produced alone.  Word n of the stream of a
// seed is SplitMix64's finaliser applied to start + (n + 1) * golden, start = finaliser(seed).
// Entry e (linear index over [layer][role][head][s]), attempt a, uses the four words
// 4 * (16 e + a) .. + 3: two Box-Muller pairs in fp64 (u1 in (0, 1], u2 in [0, 1) from the top
// 53 bits).  The 4-vector is normalised in fp64 and rounded to fp32; a vector with squared norm
// below 1e-12 (probability ~1e-25) is redrawn with the next attempt.
#include <cmath>
#include <cstdint>

#include "hqmq.h"

namespace {

struct Stream {
    uint64_t start;
    explicit Stream(uint64_t seed) : start(finalise(seed)) {}
    static uint64_t finalise(uint64_t z)
    {
        z ^= z >> 30;
        z *= 0xBF58476D1CE4E5B9ull;
        z ^= z >> 27;
        z *= 0x94D049BB133111EBull;
        z ^= z >> 31;
        return z;
    }
    uint64_t word(uint64_t n) const { return finalise(start + (n + 1) * 0x9E3779B97F4A7C15ull); }
};

inline void box_muller(uint64_t w1, uint64_t w2, double &g0, double &g1)
{
    const double scale = 1.0 / 9007199254740992.0;  // 2^-53
    const double u1 = (static_cast<double>(w1 >> 11) + 1.0) * scale;
    const double u2 = static_cast<double>(w2 >> 11) * scale;
    const double radius = std::sqrt(-2.0 * std::log(u1));
    const double angle = 6.283185307179586476925286766559 * u2;
    g0 = radius * std::cos(angle);
    g1 = radius * std::sin(angle);
}

}  // namespace

extern "C" int32_t hqmq_build_codebooks(uint64_t seed, int32_t n_layers, int32_t n_kv_heads,
                                        int32_t S, float *sec_host)
{
    if (!sec_host || n_layers <= 0 || n_kv_heads <= 0 || S <= 0)
        return HQMQ_ERR_INVALID_ARG;
    if (S > HQMQ_MAX_S)
        return HQMQ_ERR_UNSUPPORTED;  // the same limit as hqmq_encode / hqmq_decode
    const Stream stream(seed);
    const uint64_t entries = static_cast<uint64_t>(n_layers) * 2u * n_kv_heads * S;
    for (uint64_t e = 0; e < entries; ++e) {
        float *dst = sec_host + 4 * e;
        for (uint64_t attempt = 0;; ++attempt) {
            const uint64_t n = 4 * (16 * e + attempt);
            double g[4];
            box_muller(stream.word(n), stream.word(n + 1), g[0], g[1]);
            box_muller(stream.word(n + 2), stream.word(n + 3), g[2], g[3]);
            const double norm2 = ((g[0] * g[0] + g[1] * g[1]) + g[2] * g[2]) + g[3] * g[3];
            if (norm2 < 1e-12 && attempt < 15)
                continue;
            const double norm = std::sqrt(norm2);
            for (int i = 0; i < 4; ++i)
                dst[i] = static_cast<float>(g[i] / norm);
            break;
        }
    }
    return HQMQ_OK;
}
