/*
 * Seeded synthetic input generator (host, plain C + OpenMP).
 *
 * This module holds none of the attention method's arithmetic: it only draws
 * random tensors.  Every element is a pure function of
 * (seed, tensor_id, flat element index), so the same call always returns the
 * same bits and any sub-range can be regenerated independently.
 *
 * Draws:  u64 = splitmix64-style finaliser of a key built from
 * (seed, tensor_id, index, draw#);  uniforms -> Box-Muller normals;
 * Student-t(nu=3) = z / sqrt((g1^2+g2^2+g3^2)/3).
 * Output: bf16 bit patterns (round-to-nearest-even from fp32).
 */
#include <math.h>
#include <stdint.h>
#include <stddef.h>

static inline uint64_t mix64(uint64_t z) {
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

static inline uint64_t draw(uint64_t seed, uint64_t tensor, uint64_t idx, uint64_t j) {
    uint64_t k = mix64(seed * 0xD6E8FEB86659FD93ull + tensor);
    k = mix64(k ^ (idx * 0xA0761D6478BD642Full));
    return mix64(k + j * 0xE7037ED1A0B428DBull);
}

/* uniform in (0,1] with 53 bits */
static inline double unif(uint64_t r) { return ((double)(r >> 11) + 1.0) * (1.0 / 9007199254740992.0); }

static inline void normal_pair(uint64_t a, uint64_t b, double* z0, double* z1) {
    double u1 = unif(a), u2 = unif(b);
    double r = sqrt(-2.0 * log(u1));
    double t = 6.283185307179586476925 * u2;
    *z0 = r * cos(t);
    *z1 = r * sin(t);
}

static inline uint16_t f32_to_bf16_rne(float f) {
    union { float f; uint32_t u; } c; c.f = f;
    uint32_t u = c.u;
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7FFFu + lsb;
    return (uint16_t)(u >> 16);
}

/*
 * Fill out[B*H*L*d] (layout [B,H,L,d], d innermost) with bf16 bit patterns.
 *   dist            0: N(0,1)      1: Student-t(nu=3)
 *   scale           multiplies every draw
 *   n_chan, chan_mult   per (b,h): n_chan distinct channels (seeded choice) are
 *                       multiplied by chan_mult (0 => none)
 *   tok_mod, tok_mult   token l is an outlier token iff
 *                       hash(seed, l) % tok_mod == 0; its whole row is
 *                       multiplied by tok_mult (tok_mod 0 => none).  The token
 *                       set depends on the seed only, not on tensor_id.
 */
int synth_fill_bf16(uint16_t* out, int B, int H, long L, int d,
                    uint64_t seed, uint64_t tensor_id, int dist, double scale,
                    int n_chan, double chan_mult, int tok_mod, double tok_mult)
{
    if (!out || B < 1 || H < 1 || L < 1 || d < 1 || d > 1024 || n_chan > d) return -1;
    long rows = (long)B * H * L;
    #pragma omp parallel for schedule(static)
    for (long row = 0; row < rows; ++row) {
        long l = row % L;
        long bh = row / L;
        /* channel multipliers for this (b,h) */
        double cm[1024];
        for (int c = 0; c < d; ++c) cm[c] = 1.0;
        if (n_chan > 0) {
            /* seeded partial Fisher-Yates on channel indices */
            int perm[1024];
            for (int c = 0; c < d; ++c) perm[c] = c;
            for (int t = 0; t < n_chan; ++t) {
                uint64_t r = draw(seed ^ 0x5bd1e995u, tensor_id + 1000, (uint64_t)bh, (uint64_t)t);
                int pick = t + (int)(r % (uint64_t)(d - t));
                int tmp = perm[t]; perm[t] = perm[pick]; perm[pick] = tmp;
                cm[perm[t]] = chan_mult;
            }
        }
        double rm = 1.0;
        if (tok_mod > 0) {
            uint64_t r = draw(seed ^ 0x2545F491u, 7777, (uint64_t)l, 0);
            if (r % (uint64_t)tok_mod == 0) rm = tok_mult;
        }
        for (int c = 0; c < d; ++c) {
            uint64_t idx = (uint64_t)row * (uint64_t)d + (uint64_t)c;
            double z0, z1, x;
            normal_pair(draw(seed, tensor_id, idx, 0), draw(seed, tensor_id, idx, 1), &z0, &z1);
            if (dist == 0) {
                x = z0;
            } else {
                double g2, g3;
                normal_pair(draw(seed, tensor_id, idx, 2), draw(seed, tensor_id, idx, 3), &g2, &g3);
                double chi = (z1 * z1 + g2 * g2 + g3 * g3) / 3.0;
                x = z0 / sqrt(chi);
            }
            x *= scale * cm[c] * rm;
            out[idx] = f32_to_bf16_rne((float)x);
        }
    }
    return 0;
}
