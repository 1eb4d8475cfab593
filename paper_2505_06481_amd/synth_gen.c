/*
 * Seeded synthetic-input generator (host only).
 *
 * A counter-based generator: sample i of stream (seed, stream) depends only on
 * (seed, stream, i), so the output is identical for any thread count and any
 * chunking.  It produces raw input buffers (uniform and normal variates, stored
 * as fp64, fp32 or bf16) and nothing else: none of the MoE layer's arithmetic
 * lives here.  The same bytes are handed to the CPU oracle and uploaded to the
 * GPU; nothing is ever regenerated on the device.
 *
 * Mixing function: the 64-bit finaliser of SplitMix64 (Steele, Lea, Flood,
 * "Fast splittable pseudorandom number generators", OOPSLA 2014), applied to a
 * keyed counter.  Normals: Box-Muller in double precision from two uniforms.
 */
#include <math.h>
#include <stdint.h>
#include <stddef.h>
#include <string.h>

static inline uint64_t mix64(uint64_t z)
{
    z ^= z >> 30;
    z *= 0xBF58476D1CE4E5B9ull;
    z ^= z >> 27;
    z *= 0x94D049BB133111EBull;
    z ^= z >> 31;
    return z;
}

static inline uint64_t stream_key(uint64_t seed, uint64_t stream)
{
    return mix64(mix64(seed + 0x9E3779B97F4A7C15ull) ^ (stream * 0xD1342543DE82EF95ull + 0x632BE59BD9B4E019ull));
}

/* j-th 64-bit word of the stream */
static inline uint64_t word(uint64_t key, uint64_t j)
{
    return mix64(key + j * 0x9E3779B97F4A7C15ull);
}

/* uniform in (0,1): 53 random bits, centred so that 0 and 1 never occur */
static inline double unif(uint64_t w)
{
    return ((double)(w >> 11) + 0.5) * (1.0 / 9007199254740992.0);
}

static inline void normal_pair(uint64_t key, uint64_t pair, double *z0, double *z1)
{
    double u1 = unif(word(key, 2 * pair));
    double u2 = unif(word(key, 2 * pair + 1));
    double r = sqrt(-2.0 * log(u1));
    double a = 6.283185307179586476925286766559 * u2;
    *z0 = r * cos(a);
    *z1 = r * sin(a);
}

static inline uint16_t f32_to_bf16_rne(float x)
{
    uint32_t u;
    memcpy(&u, &x, 4);
    u += 0x7FFFu + ((u >> 16) & 1u); /* finite inputs only */
    return (uint16_t)(u >> 16);
}

void synth_uniform_f64(uint64_t seed, uint64_t stream, size_t n, double *out)
{
    uint64_t key = stream_key(seed, stream);
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < n; ++i)
        out[i] = unif(word(key, i));
}

void synth_normal_f32(uint64_t seed, uint64_t stream, size_t n, double sigma, float *out)
{
    uint64_t key = stream_key(seed, stream);
    size_t npair = (n + 1) / 2;
#pragma omp parallel for schedule(static)
    for (size_t p = 0; p < npair; ++p) {
        double z0, z1;
        normal_pair(key, p, &z0, &z1);
        out[2 * p] = (float)(sigma * z0);
        if (2 * p + 1 < n)
            out[2 * p + 1] = (float)(sigma * z1);
    }
}

void synth_normal_bf16(uint64_t seed, uint64_t stream, size_t n, double sigma, uint16_t *out)
{
    uint64_t key = stream_key(seed, stream);
    size_t npair = (n + 1) / 2;
#pragma omp parallel for schedule(static)
    for (size_t p = 0; p < npair; ++p) {
        double z0, z1;
        normal_pair(key, p, &z0, &z1);
        out[2 * p] = f32_to_bf16_rne((float)(sigma * z0));
        if (2 * p + 1 < n)
            out[2 * p + 1] = f32_to_bf16_rne((float)(sigma * z1));
    }
}
