/*
 * Seeded synthetic-input generator (counter based).
 *
 * This file holds no arithmetic of the SPD method: it only turns a 64-bit key
 * and an element index into a reproducible pseudo-random normal deviate, so
 * that any tensor (or any slice of one) can be regenerated independently on any
 * host.  Both the CPU oracle and the HIP path are fed from here; they share the
 * data, never code.
 *
 * Determinism: only IEEE double add/mul/div/sqrt, integer ops and own polynomials
 * are used (no libm, no fused multiply-add; compile with -ffp-contract=off), so
 * the stream is bit-identical on every x86-64 host and for any thread count.
 */
#include <stdint.h>
#include <stddef.h>

static inline uint64_t mix64(uint64_t z) {
    z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ULL;
    z ^= z >> 27; z *= 0x94D049BB133111EBULL;
    z ^= z >> 31;
    return z;
}

/* natural log of k / 2^24 for integer k in [1, 2^24] */
static inline double ln_u24(uint32_t k) {
    union { double d; uint64_t u; } c; c.d = (double)k;          /* exact */
    int e = (int)(c.u >> 52) - 1023;                              /* floor(log2 k) */
    c.u = (c.u & 0x000FFFFFFFFFFFFFULL) | 0x3FF0000000000000ULL;  /* mantissa in [1, 2) */
    double m = c.d;
    double s = (m - 1.0) / (m + 1.0);              /* [0, 1/3) */
    double s2 = s * s;
    /* 2 * atanh(s), odd series to s^21 */
    double p = 1.0 / 21.0;
    p = p * s2 + 1.0 / 19.0;
    p = p * s2 + 1.0 / 17.0;
    p = p * s2 + 1.0 / 15.0;
    p = p * s2 + 1.0 / 13.0;
    p = p * s2 + 1.0 / 11.0;
    p = p * s2 + 1.0 / 9.0;
    p = p * s2 + 1.0 / 7.0;
    p = p * s2 + 1.0 / 5.0;
    p = p * s2 + 1.0 / 3.0;
    p = p * s2 + 1.0;
    return 2.0 * s * p + (double)(e - 24) * 0.69314718055994530942;
}

/* cos(2*pi*j/2^24), quarter-wave reduction + even Taylor series on [0, pi/2] */
static inline double cos_turn24(uint32_t j) {
    uint32_t q = j >> 22;                  /* quadrant 0..3 */
    uint32_t f = j & 0x3FFFFFu;            /* position inside the quadrant */
    /* cos in quadrants 1 and 3 is +-sin of the offset = cos(pi/2 - offset) */
    uint32_t g = (q & 1u) ? (0x400000u - f) : f;
    double x = (double)g * (1.57079632679489661923 / 4194304.0);   /* [0, pi/2] */
    double x2 = x * x;
    double c = 1.0 / 6402373705728000.0;   /* 1/18! */
    c = c * x2 - 1.0 / 20922789888000.0;   /* 1/16! */
    c = c * x2 + 1.0 / 87178291200.0;      /* 1/14! */
    c = c * x2 - 1.0 / 479001600.0;        /* 1/12! */
    c = c * x2 + 1.0 / 3628800.0;          /* 1/10! */
    c = c * x2 - 1.0 / 40320.0;            /* 1/8!  */
    c = c * x2 + 1.0 / 720.0;              /* 1/6!  */
    c = c * x2 - 1.0 / 24.0;
    c = c * x2 + 0.5;
    c = 1.0 - c * x2;
    return (q == 1u || q == 2u) ? -c : c;
}

static inline float normal_at(uint64_t key, uint64_t idx) {
    uint64_t z = mix64(key + (idx + 1) * 0x9E3779B97F4A7C15ULL);
    uint32_t k = (uint32_t)(z >> 40) + 1u;          /* 1 .. 2^24  -> u1 in (0,1] */
    uint32_t j = (uint32_t)(z & 0xFFFFFFu);         /* 0 .. 2^24-1 -> u2 in [0,1) */
    double r = __builtin_sqrt(-2.0 * ln_u24(k));      /* IEEE sqrt: correctly rounded */
    return (float)(r * cos_turn24(j));
}

static inline float round_bf16(float v) {
    union { float f; uint32_t u; } c; c.f = v;
    c.u += 0x7FFFu + ((c.u >> 16) & 1u);            /* round to nearest even */
    c.u &= 0xFFFF0000u;
    return c.f;
}

uint64_t spd_inputs_key(uint64_t seed, uint64_t tensor_id, uint64_t layer, uint64_t rank) {
    uint64_t k = mix64(seed * 0xD6E8FEB86659FD93ULL + 0x1234567ULL);
    k = mix64(k ^ (tensor_id + 0x632BE59BD9B4E019ULL));
    k = mix64(k ^ (layer * 0xA0761D6478BD642FULL + 1ULL));
    k = mix64(k ^ (rank * 0xE7037ED1A0B428DBULL + 2ULL));
    return k;
}

/* out[i] = mean + std * N(0,1)[first + i], optionally rounded to bf16-representable fp32 */
void spd_inputs_normal(float *out, size_t n, uint64_t key, uint64_t first,
                       float mean, float std, int to_bf16) {
    #pragma omp parallel for schedule(static)
    for (ptrdiff_t i = 0; i < (ptrdiff_t)n; ++i) {
        float v = mean + std * normal_at(key, first + (uint64_t)i);
        out[i] = to_bf16 ? round_bf16(v) : v;
    }
}
