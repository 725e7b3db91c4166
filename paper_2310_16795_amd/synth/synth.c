/*
 * Seeded synthetic input generator.
 *
 * Produces the random inputs of the workloads (ternary symbol matrices,
 * per-row scales, activation vectors, uniform draws for routing) from a
 * counter-based generator: element i of stream `seed` is a pure function
 * of (seed, i), so any slice can be regenerated anywhere, in any order, on
 * any number of threads.  This file holds no part of the compression
 * method itself: no dictionary, no coding, no matrix product.  It serves
 * the tests, the benchmark and the CPU oracle alike so that all of them
 * see identical inputs.
 *
 * Generator: the SplitMix64 output function (Steele, Lea, Flood 2014)
 * applied to seed + (i + 1) * golden-gamma.
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

static inline uint64_t mix64(uint64_t seed, uint64_t ctr)
{
    uint64_t z = seed + (ctr + 1u) * 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

/* uniform double in [0,1) with 53 random bits */
static inline double u01(uint64_t h) { return (double)(h >> 11) * (1.0 / 9007199254740992.0); }

/* float -> bfloat16 bits, round to nearest even (finite inputs) */
static inline uint16_t f32_to_bf16(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

/* float -> IEEE binary16 bits, round to nearest even (normal range only) */
static inline uint16_t f32_to_f16(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    uint32_t sign = (u >> 16) & 0x8000u;
    int32_t e = (int32_t)((u >> 23) & 0xFF) - 127 + 15;
    uint32_t m = u & 0x7FFFFFu;
    if (e <= 0) { /* subnormal half: shift the implicit one in */
        if (e < -10) return (uint16_t)sign;
        m |= 0x800000u;
        uint32_t shift = (uint32_t)(14 - e);
        uint32_t half = m >> shift;
        uint32_t rem = m & ((1u << shift) - 1u);
        uint32_t mid = 1u << (shift - 1);
        if (rem > mid || (rem == mid && (half & 1u))) half++;
        return (uint16_t)(sign | half);
    }
    if (e >= 31) return (uint16_t)(sign | 0x7C00u);
    uint32_t half = ((uint32_t)e << 10) | (m >> 13);
    uint32_t rem = m & 0x1FFFu;
    if (rem > 0x1000u || (rem == 0x1000u && (half & 1u))) half++;
    return (uint16_t)(sign | half);
}

/*
 * Ternary matrix, row-major int8 in {-1,0,+1}.
 * Element (r,c) is 0 with probability p0_row[r] (or p0_all when p0_row is
 * NULL), otherwise -1 or +1 with equal probability.  One 64-bit draw feeds
 * two neighbouring elements: 31 bits decide zero/non-zero, one bit the sign.
 */
void synth_ternary(uint64_t seed, int64_t rows, int64_t cols, double p0_all,
                   const double *p0_row, int8_t *out)
{
    int64_t half_cols = (cols + 1) / 2;
    for (int64_t r = 0; r < rows; r++) {
        double p0 = p0_row ? p0_row[r] : p0_all;
        if (p0 < 0.0) p0 = 0.0;
        if (p0 > 1.0) p0 = 1.0;
        uint32_t thr = (uint32_t)(p0 * 2147483648.0); /* of 2^31 */
        int8_t *o = out + r * cols;
        for (int64_t j = 0; j < half_cols; j++) {
            uint64_t h = mix64(seed, (uint64_t)(r * half_cols + j));
            uint32_t a = (uint32_t)h, b = (uint32_t)(h >> 32);
            int8_t va = ((a >> 1) < thr) ? 0 : ((a & 1u) ? 1 : -1);
            int8_t vb = ((b >> 1) < thr) ? 0 : ((b & 1u) ? 1 : -1);
            o[2 * j] = va;
            if (2 * j + 1 < cols) o[2 * j + 1] = vb;
        }
    }
}

/* n standard-normal values (Box-Muller on two draws), rounded to bfloat16 */
void synth_normal_bf16(uint64_t seed, int64_t n, uint16_t *out)
{
    for (int64_t i = 0; i < n; i++) {
        double u1 = u01(mix64(seed, (uint64_t)(2 * i)));
        double u2 = u01(mix64(seed, (uint64_t)(2 * i + 1)));
        double rad = sqrt(-2.0 * log(1.0 - u1)); /* 1-u1 in (0,1] */
        double z = rad * cos(6.283185307179586476925 * u2);
        out[i] = f32_to_bf16((float)z);
    }
}

/* n values uniform in [lo,hi), rounded to binary16 */
void synth_uniform_f16(uint64_t seed, int64_t n, double lo, double hi, uint16_t *out)
{
    for (int64_t i = 0; i < n; i++) {
        double u = u01(mix64(seed, (uint64_t)i));
        out[i] = f32_to_f16((float)(lo + (hi - lo) * u));
    }
}

/* n uniform doubles in [0,1), starting at counter `first` */
void synth_uniform_f64(uint64_t seed, int64_t first, int64_t n, double *out)
{
    for (int64_t i = 0; i < n; i++) out[i] = u01(mix64(seed, (uint64_t)(first + i)));
}
