/*
 * Seeded bulk fillers for synthetic model files.
 *
 * This file holds no arithmetic of the decoding method: it only produces
 * reproducible pseudo-random bf16 values.  Every value is a pure function of
 * (seed, stream, element index), so the result does not depend on the number
 * of threads or on the order in which tensors are filled.
 *
 * Counter-based generator: a 64-bit finaliser (two rounds of xor-shift /
 * multiply, constants from the splitmix64 generator) applied to a counter
 * built from seed, stream and pair index.  One 64-bit output feeds one
 * Box-Muller pair.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>

static inline uint64_t mix64(uint64_t z)
{
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

static inline uint64_t counter_bits(uint64_t seed, uint64_t stream, uint64_t idx)
{
    uint64_t k = mix64(seed ^ mix64(stream * 0xD1342543DE82EF95ull + 0x632BE59BD9B4E019ull));
    return mix64(k ^ mix64(idx));
}

/* float -> bf16, round to nearest even (inputs here are never NaN) */
static inline uint16_t f32_to_bf16(float f)
{
    union { float f; uint32_t u; } v;
    v.f = f;
    uint32_t r = v.u + 0x7FFFu + ((v.u >> 16) & 1u);
    return (uint16_t)(r >> 16);
}

/* dst[i] = bf16(N(0, std^2)), i in [0, n) */
void eeg_fill_normal_bf16(uint16_t *dst, size_t n, uint64_t seed, uint64_t stream, double std)
{
    const size_t pairs = (n + 1) / 2;
    const double two_pi = 6.283185307179586476925286766559;
#pragma omp parallel for schedule(static)
    for (size_t p = 0; p < pairs; ++p) {
        uint64_t b = counter_bits(seed, stream, p);
        /* u1 in (0,1], u2 in [0,1): 32 bits each */
        double u1 = ((double)(uint32_t)(b >> 32) + 1.0) * (1.0 / 4294967296.0);
        double u2 = (double)(uint32_t)b * (1.0 / 4294967296.0);
        double r = sqrt(-2.0 * log(u1)) * std;
        double a = two_pi * u2;
        dst[2 * p] = f32_to_bf16((float)(r * cos(a)));
        if (2 * p + 1 < n)
            dst[2 * p + 1] = f32_to_bf16((float)(r * sin(a)));
    }
}

/* dst[i] = bf16(U[lo, hi)) */
void eeg_fill_uniform_bf16(uint16_t *dst, size_t n, uint64_t seed, uint64_t stream, double lo, double hi)
{
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < n; ++i) {
        uint64_t b = counter_bits(seed, stream, i);
        double u = (double)(b >> 11) * (1.0 / 9007199254740992.0);
        dst[i] = f32_to_bf16((float)(lo + (hi - lo) * u));
    }
}

/* dst[i] = bf16(value) */
void eeg_fill_const_bf16(uint16_t *dst, size_t n, double value)
{
    uint16_t v = f32_to_bf16((float)value);
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < n; ++i)
        dst[i] = v;
}
