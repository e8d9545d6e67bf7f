/*
 * Seeded synthetic-input generator shared by the CPU oracle's tests and the
 * GPU harness.  It holds no arithmetic of the training method: it only turns
 * (seed, stream, index) into reproducible pseudo-random numbers so that both
 * sides consume the same bytes.
 *
 * Every value is a pure function of (seed, stream, index): a 64-bit mix of the
 * three gives two uniforms, and the Box-Muller cosine branch turns them into
 * one standard normal.  Because the generator is counter based, any sub-range
 * of a tensor can be produced independently and in parallel.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

static inline uint64_t mix64(uint64_t z)
{
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

static inline double std_normal(uint64_t seed, uint64_t stream, uint64_t index)
{
    uint64_t key = mix64(mix64(seed) ^ (stream * 0xD1B54A32D192ED03ull));
    uint64_t a = mix64(key ^ (2 * index));
    uint64_t b = mix64(key ^ (2 * index + 1));
    /* u1 in (0,1], u2 in [0,1) */
    double u1 = ((double)(a >> 11) + 1.0) * (1.0 / 9007199254740992.0);
    double u2 = (double)(b >> 11) * (1.0 / 9007199254740992.0);
    return sqrt(-2.0 * log(u1)) * cos(6.283185307179586476925 * u2);
}

/* out[i] = mean + std * z(seed, stream, first + i), as float.
 * If keep_bits16 != 0 the low 16 bits of each float are cleared, so that the
 * value is exactly representable with an 8-bit significand (a bf16 pattern
 * widened to fp32); this is a property of the generated data, not a cast the
 * consumers have to agree on. */
void zpp_synth_normal_f32(uint64_t seed, uint64_t stream, uint64_t first,
                          uint64_t count, double mean, double std,
                          int keep_bits16, float *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < (int64_t)count; ++i) {
        float v = (float)(mean + std * std_normal(seed, stream, first + (uint64_t)i));
        if (keep_bits16) {
            uint32_t u;
            memcpy(&u, &v, 4);
            u &= 0xFFFF0000u;
            memcpy(&v, &u, 4);
        }
        out[i] = v;
    }
}

/* Same stream as above, in double precision (no truncation option). */
void zpp_synth_normal_f64(uint64_t seed, uint64_t stream, uint64_t first,
                          uint64_t count, double mean, double std, double *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < (int64_t)count; ++i)
        out[i] = mean + std * std_normal(seed, stream, first + (uint64_t)i);
}

void zpp_synth_fill_f32(uint64_t count, float value, float *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < (int64_t)count; ++i)
        out[i] = value;
}
