/*
 * Seeded synthetic-input generator for the window-over-history attention workloads.
 *
 * This file holds no attention arithmetic: it only fills buffers with reproducible
 * pseudo-random numbers.  Every element is a pure function of (seed, tag, flat index), so
 * the result does not depend on thread count or on the order elements are produced in.
 *
 *   key   = splitmix64(seed + tag * GOLDEN)
 *   u     = splitmix64(key + index)
 *   u1    = (top 24 bits of u + 1) / 2^24      in (0, 1]
 *   u2    = (next 24 bits of u)    / 2^24      in [0, 1)
 *   z     = sqrt(-2 ln u1) * cos(2 pi u2)      Box-Muller, evaluated in double
 *   value = (float)z * mul * (row is "peaky" ? peaky_factor : 1)
 *
 * A row (index / rowlen) is peaky iff peaky_mod > 0 and
 * splitmix64(splitmix64(seed + (tag + 1000) * GOLDEN) + row) % peaky_mod == 0.
 *
 * Output is fp32, or bf16 obtained from the fp32 value by round-to-nearest-even.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

#define GOLDEN 0x9E3779B97F4A7C15ULL

static inline uint64_t splitmix64(uint64_t x)
{
    uint64_t z = x + GOLDEN;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}

static inline uint16_t f32_to_bf16_rne(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x40u); /* quiet NaN */
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

/* dtype: 0 = fp32 (out is float*), 1 = bf16 (out is uint16_t*).  Returns 0, or -1 on bad args. */
int tlin_gen_normal(void *out, int dtype, uint64_t seed, uint64_t tag, size_t n, float mul,
                    size_t rowlen, uint32_t peaky_mod, float peaky_factor)
{
    if (!out || (dtype != 0 && dtype != 1) || rowlen == 0) return -1;
    const uint64_t key = splitmix64(seed + tag * GOLDEN);
    const uint64_t pkey = splitmix64(seed + (tag + 1000) * GOLDEN);
    const double two_pi = 6.283185307179586476925286766559;
    ptrdiff_t i;
#pragma omp parallel for schedule(static)
    for (i = 0; i < (ptrdiff_t)n; ++i) {
        uint64_t u = splitmix64(key + (uint64_t)i);
        double u1 = (double)((u >> 40) + 1) * (1.0 / 16777216.0);
        double u2 = (double)((u >> 16) & 0xFFFFFFu) * (1.0 / 16777216.0);
        float z = (float)(sqrt(-2.0 * log(u1)) * cos(two_pi * u2));
        float v = z * mul;
        if (peaky_mod) {
            uint64_t row = (uint64_t)i / rowlen;
            if (splitmix64(pkey + row) % peaky_mod == 0) v *= peaky_factor;
        }
        if (dtype == 0) ((float *)out)[i] = v;
        else ((uint16_t *)out)[i] = f32_to_bf16_rne(v);
    }
    return 0;
}
