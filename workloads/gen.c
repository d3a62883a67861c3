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

static inline double normal_at(uint64_t seed, uint64_t counter)
{
    uint64_t z = mpagen_bits(seed, counter);
    double u1 = ((double)(z >> 40) + 0.5) * (1.0 / 16777216.0);          /* (0,1), 24 bits */
    double u2 = ((double)((z >> 16) & 0xFFFFFFull) + 0.5) * (1.0 / 16777216.0);
    return sqrt(-2.0 * log(u1)) * cos(6.283185307179586476925 * u2);
}

/* out[i] = bf16(N(0,1) drawn at counter offset+i), i in [0,n). */
void mpagen_fill_normal_bf16(uint16_t *out, uint64_t n, uint64_t seed, uint64_t offset)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < (int64_t)n; ++i)
        out[i] = f32_to_bf16_rne((float)normal_at(seed, offset + (uint64_t)i));
}

/* Same, for nseg segments of seglen values each; segment s starts at counter offsets[s]. */
void mpagen_fill_normal_bf16_segments(uint16_t *out, uint64_t nseg, uint64_t seglen,
                                      uint64_t seed, const uint64_t *offsets)
{
#pragma omp parallel for schedule(static)
    for (int64_t s = 0; s < (int64_t)nseg; ++s) {
        uint16_t *o = out + (uint64_t)s * seglen;
        uint64_t base = offsets[s];
        for (uint64_t i = 0; i < seglen; ++i)
            o[i] = f32_to_bf16_rne((float)normal_at(seed, base + i));
    }
}

/* out[i] = 64 random bits at counter offset+i (integer draws are finished in Python). */
void mpagen_fill_bits(uint64_t *out, uint64_t n, uint64_t seed, uint64_t offset)
{
    for (uint64_t i = 0; i < n; ++i) out[i] = mpagen_bits(seed, offset + i);
}
