/*
 * Seeded, counter-based synthetic input generator.
 *
 * Holds none of the attention method's arithmetic: it only turns (seed, index) into
 * reproducible pseudo-random values, so the CPU oracle and the GPU path can be fed the very
 * same arrays.  Every value depends on (seed, absolute index) alone, so any sub-range of a
 * huge tensor (e.g. one KV block out of a 21 GB pool) can be produced on its own.
 *
 * Build: gcc -O2 -fopenmp -shared -fPIC gen.c -o libmpagen.so -lm
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

static inline uint64_t mix64(uint64_t z)
{
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

/* 64 random bits for (seed, counter). */
uint64_t mpagen_bits(uint64_t seed, uint64_t counter)
{
    return mix64(mix64(seed) ^ (counter * 0xD1342543DE82EF95ull + 0x632BE59BD9B4E019ull));
}

static inline uint16_t f32_to_bf16_rne(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x40u); /* quiet NaN */
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

/* IEEE half, round to nearest even; overflow to infinity, subnormals kept. */
static inline uint16_t f32_to_f16_rne(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    const uint32_t sign = (u >> 16) & 0x8000u;
    const uint32_t a = u & 0x7FFFFFFFu;
    if (a > 0x7F800000u) return (uint16_t)(sign | 0x7E00u);            /* NaN */
    if (a >= 0x47800000u) return (uint16_t)(sign | 0x7C00u);           /* >= 65536: infinity (65520.. rounds up below) */
    if (a < 0x33000000u) return (uint16_t)sign;                         /* < 2^-25: zero */
    int32_t e = (int32_t)(a >> 23) - 127;                               /* unbiased exponent */
    uint32_t m = (a & 0x7FFFFFu) | 0x800000u;                           /* 24-bit significand */
    int shift = e >= -14 ? 13 : 13 + (-14 - e);                         /* bits dropped */
    uint32_t kept = m >> shift, rem = m & ((1u << shift) - 1u), halfway = 1u << (shift - 1);
    if (rem > halfway || (rem == halfway && (kept & 1u))) ++kept;
    /* normal: kept has the hidden bit at position 10 (or 11 after a carry): adding the exponent
       field absorbs both; subnormal: kept < 1024 (or exactly 1024 = smallest normal) */
    uint32_t h = e >= -14 ? (uint32_t)((e + 15 - 1) << 10) + kept : kept;
    return (uint16_t)(sign | h);
}

static inline uint16_t f32_to_16(float f, int dtype) { return dtype == 2 ? f32_to_f16_rne(f) : f32_to_bf16_rne(f); }

static inline double normal_at(uint64_t seed, uint64_t counter)
{
    uint64_t z = mpagen_bits(seed, counter);
    double u1 = ((double)(z >> 40) + 0.5) * (1.0 / 16777216.0);          /* (0,1), 24 bits */
    double u2 = ((double)((z >> 16) & 0xFFFFFFull) + 0.5) * (1.0 / 16777216.0);
    return sqrt(-2.0 * log(u1)) * cos(6.283185307179586476925 * u2);
}

/* out[i] = N(0,1) drawn at counter offset+i, rounded to bf16 (dtype 1) or fp16 (dtype 2), i in [0,n). */
void mpagen_fill_normal_16(uint16_t *out, uint64_t n, uint64_t seed, uint64_t offset, int dtype)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < (int64_t)n; ++i)
        out[i] = f32_to_16((float)normal_at(seed, offset + (uint64_t)i), dtype);
}

/* Rounding alone, for the tests that pin it against a library conversion. */
void mpagen_round_16(const float *in, uint16_t *out, uint64_t n, int dtype)
{
    for (uint64_t i = 0; i < n; ++i) out[i] = f32_to_16(in[i], dtype);
}

/* Same, for nseg segments of seglen values each; segment s starts at counter offsets[s]. */
void mpagen_fill_normal_16_segments(uint16_t *out, uint64_t nseg, uint64_t seglen,
                                    uint64_t seed, const uint64_t *offsets, int dtype)
{
#pragma omp parallel for schedule(static)
    for (int64_t s = 0; s < (int64_t)nseg; ++s) {
        uint16_t *o = out + (uint64_t)s * seglen;
        uint64_t base = offsets[s];
        for (uint64_t i = 0; i < seglen; ++i)
            o[i] = f32_to_16((float)normal_at(seed, base + i), dtype);
    }
}

/* out[i] = 64 random bits at counter offset+i (integer draws are finished in Python). */
void mpagen_fill_bits(uint64_t *out, uint64_t n, uint64_t seed, uint64_t offset)
{
    for (uint64_t i = 0; i < n; ++i) out[i] = mpagen_bits(seed, offset + i);
}
