/*
 * Seeded synthetic-input generator, CPU side.
 *
 * This file only manufactures INPUTS (gradient values, packet-survival bits):
 * it contains none of the protocol's arithmetic.  Both the CPU checker and the
 * GPU library consume what it produces.  A device-side twin of grad_fill()
 * lives in gen.hip; the two follow the same integer recipe and are compared
 * bit for bit by a GPU test.
 *
 * Recipe (all integer until one exact int->float conversion and one IEEE
 * multiply, so every platform produces identical bits):
 *   mix(x)   : the published SplitMix64 output function
 *   key      : mix(mix(seed + 0x100000001B3 * stream) + sub)
 *   h_j(e)   : mix(key + (3e + j) * GOLDEN), j = 0,1,2
 *   S(e)     : sum of the twelve 16-bit fields of h_0,h_1,h_2   (Irwin-Hall, n = 12)
 *   z(e)     : 2 S - 12 * 65535            (integer, |z| < 2^20, std ~ 131072)
 *   value(e) : (float) z * c               with c = (float)(sigma / 131072)
 *   tail     : if tail_ppm > 0 and the top 32 bits of mix(key ^ TAIL + e * GOLDEN),
 *              scaled to [0, 1e6), fall below tail_ppm: value *= tail_mul
 */
#include <stdint.h>
#include <stddef.h>

#define GOLDEN 0x9E3779B97F4A7C15ULL
#define TAILSALT 0xD1B54A32D192ED03ULL

static inline uint64_t mix64(uint64_t x) {
    x ^= x >> 30; x *= 0xBF58476D1CE4E5B9ULL;
    x ^= x >> 27; x *= 0x94D049BB133111EBULL;
    x ^= x >> 31;
    return x;
}

uint64_t dblp_gen_key(uint64_t seed, uint64_t stream, uint64_t sub) {
    return mix64(mix64(seed + 0x100000001B3ULL * stream) + sub);
}

static inline uint32_t fields16(uint64_t h) {
    return (uint32_t)(h & 0xFFFF) + (uint32_t)((h >> 16) & 0xFFFF) +
           (uint32_t)((h >> 32) & 0xFFFF) + (uint32_t)(h >> 48);
}

/* out[i] = value(e0 + i), i < n.  scale = c above. */
void dblp_gen_grad_fill(float* out, uint64_t e0, uint64_t n, uint64_t key,
                        float scale, uint32_t tail_ppm, float tail_mul) {
    #pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < (int64_t)n; ++i) {
        uint64_t e = e0 + (uint64_t)i;
        uint32_t s = fields16(mix64(key + (3 * e + 0) * GOLDEN)) +
                     fields16(mix64(key + (3 * e + 1) * GOLDEN)) +
                     fields16(mix64(key + (3 * e + 2) * GOLDEN));
        int32_t z = 2 * (int32_t)s - 12 * 65535;
        float v = (float)z * scale;
        if (tail_ppm) {
            uint64_t t = mix64((key ^ TAILSALT) + e * GOLDEN) >> 32;
            if (((t * 1000000ULL) >> 32) < tail_ppm) v = v * tail_mul;
        }
        out[i] = v;
    }
}

/* Uniform 32-bit draw number `idx` of a keyed stream. */
static inline uint32_t draw32(uint64_t key, uint64_t idx) {
    return (uint32_t)(mix64(key + idx * GOLDEN) >> 32);
}

/* i.i.d. loss: survive[i] = 1 unless draw < loss_q32 (= loss probability * 2^32). */
void dblp_gen_bernoulli(uint8_t* survive, uint64_t n, uint64_t key, uint32_t loss_q32) {
    for (uint64_t i = 0; i < n; ++i) survive[i] = draw32(key, i) >= loss_q32;
}

/*
 * Two-state Gilbert-Elliott chain over positions 0..n-1 of one sender's
 * stream.  Starts in the good state.  Per position: first the loss draw in
 * the current state, then the state transition.
 */
void dblp_gen_gilbert_elliott(uint8_t* survive, uint64_t n, uint64_t key,
                              uint32_t loss_good_q32, uint32_t loss_bad_q32,
                              uint32_t p_g2b_q32, uint32_t p_b2g_q32) {
    int bad = 0;
    for (uint64_t i = 0; i < n; ++i) {
        uint32_t u_loss = draw32(key, 2 * i);
        uint32_t u_move = draw32(key, 2 * i + 1);
        survive[i] = u_loss >= (bad ? loss_bad_q32 : loss_good_q32);
        if (bad) { if (u_move < p_b2g_q32) bad = 0; }
        else     { if (u_move < p_g2b_q32) bad = 1; }
    }
}
