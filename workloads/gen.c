/*
 * Seeded synthetic inputs for the feature-row gather: table fills and ID lists.
 *
 * This module serves both the CPU oracle's tests and the GPU library's tests
 * and benchmark.  It contains input generation only -- nothing of the gather
 * itself -- and is built by the host C compiler with OpenMP.
 *
 * Every value is a pure function of (seed, flat element number), so a table of
 * any size can be filled in parallel, refilled identically, and any single
 * element recomputed later without the table.  The shapes stand in for the
 * workloads of PyTorch-Direct (arXiv 2101.07956): the random-index
 * microbenchmark of Section 5.1 and the feature widths / node counts of its
 * dataset table; the paper's own datasets are not used.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* 64-bit counter-based mixer (the splitmix64 output function applied to
 * counter + seed * odd constant). */
static inline uint64_t mix64(uint64_t seed, uint64_t counter)
{
    uint64_t z = counter + seed * 0x9E3779B97F4A7C15ull + 0x632BE59BD9B4E019ull;
    z ^= z >> 30;
    z *= 0xBF58476D1CE4E5B9ull;
    z ^= z >> 27;
    z *= 0x94D049BB133111EBull;
    z ^= z >> 31;
    return z;
}

uint64_t wl_mix64(uint64_t seed, uint64_t counter) { return mix64(seed, counter); }

/* uniform in [-1, 1): 24 random bits k -> k * 2^-23 - 1, exactly representable */
static inline float uniform_pm1(uint64_t seed, uint64_t e)
{
    return (float)(mix64(seed, e) >> 40) * (1.0f / 8388608.0f) - 1.0f;
}

float wl_uniform_f32_at(uint64_t seed, uint64_t e) { return uniform_pm1(seed, e); }

/* dst[k] = uniform(seed, first + k), 0 <= k < n */
void wl_fill_uniform_f32(float *dst, uint64_t seed, uint64_t first, uint64_t n)
{
#pragma omp parallel for schedule(static)
    for (int64_t k = 0; k < (int64_t)n; ++k)
        dst[k] = uniform_pm1(seed, first + (uint64_t)k);
}

/* binary32 -> binary16, round to nearest even (generator-side narrowing; the
 * gather under test only ever widens) */
static inline uint16_t f32_to_f16_rne(float x)
{
    uint32_t u;
    memcpy(&u, &x, 4);
    const uint32_t sign = (u >> 16) & 0x8000u;
    const uint32_t a = u & 0x7fffffffu;
    if (a >= 0x7f800000u)                       /* inf / nan */
        return (uint16_t)(sign | 0x7c00u | ((a > 0x7f800000u) ? 0x200u : 0u));
    if (a >= 0x477ff000u)                       /* rounds to >= 65520 -> inf */
        return (uint16_t)(sign | 0x7c00u);
    if (a < 0x33000001u)                        /* <= 2^-25 -> zero */
        return (uint16_t)sign;
    const int e = (int)(a >> 23) - 127;         /* unbiased */
    uint32_t m = (a & 0x7fffffu) | 0x800000u;   /* 24-bit significand */
    int shift;                                   /* bits dropped */
    uint32_t base;
    if (e >= -14) {                             /* normal half */
        shift = 13;
        base = (uint32_t)(e + 15) << 10;
        m &= 0x7fffffu;
    } else {                                    /* subnormal half */
        shift = 13 + (-14 - e);
        base = 0;
    }
    uint32_t q = m >> shift;
    const uint32_t rem = m & ((1u << shift) - 1u);
    const uint32_t half = 1u << (shift - 1);
    if (rem > half || (rem == half && (q & 1u)))
        ++q;                                    /* may carry into the exponent: still correct */
    return (uint16_t)(sign | (base + q));
}

uint16_t wl_f32_to_f16_rne(float x) { return f32_to_f16_rne(x); }

/* standard normal via Box-Muller on the pair (e >> 1); even e takes the cosine
 * branch, odd e the sine branch */
static inline float normal01(uint64_t seed, uint64_t e)
{
    const uint64_t p = e >> 1;
    const uint64_t h1 = mix64(seed, 2 * p);
    const uint64_t h2 = mix64(seed, 2 * p + 1);
    const float u1 = ((float)(h1 >> 40) + 1.0f) * (1.0f / 16777216.0f); /* (0, 1] */
    const float u2 = (float)(h2 >> 40) * (1.0f / 16777216.0f);          /* [0, 1) */
    const float rad = sqrtf(-2.0f * logf(u1));
    const float ang = 6.28318530717958647692f * u2;
    return rad * ((e & 1u) ? sinf(ang) : cosf(ang));
}

uint16_t wl_normal_f16_at(uint64_t seed, uint64_t e) { return f32_to_f16_rne(normal01(seed, e)); }

/* dst[k] = fp16(N(0,1))(seed, first + k) */
void wl_fill_normal_f16(uint16_t *dst, uint64_t seed, uint64_t first, uint64_t n)
{
#pragma omp parallel for schedule(static)
    for (int64_t k = 0; k < (int64_t)n; ++k)
        dst[k] = f32_to_f16_rne(normal01(seed, first + (uint64_t)k));
}

/* dst[k] = all 32-bit (or 16-bit) patterns in turn: element e holds e mod 2^w.
 * "Tag table": the expected gather result has a closed form, idx[i]*D + j. */
void wl_fill_tag_u32(uint32_t *dst, uint64_t first, uint64_t n)
{
#pragma omp parallel for schedule(static)
    for (int64_t k = 0; k < (int64_t)n; ++k)
        dst[k] = (uint32_t)(first + (uint64_t)k);
}

void wl_fill_tag_u16(uint16_t *dst, uint64_t first, uint64_t n)
{
#pragma omp parallel for schedule(static)
    for (int64_t k = 0; k < (int64_t)n; ++k)
        dst[k] = (uint16_t)(first + (uint64_t)k);
}

/* uniform row IDs in [0, N) with replacement (multiply-high range reduction) */
static inline int64_t uniform_row(uint64_t seed, uint64_t k, uint64_t N)
{
    return (int64_t)(((__uint128_t)mix64(seed, k) * (__uint128_t)N) >> 64);
}

void wl_indices_uniform_i64(int64_t *dst, uint64_t seed, uint64_t M, uint64_t N)
{
#pragma omp parallel for schedule(static)
    for (int64_t k = 0; k < (int64_t)M; ++k)
        dst[k] = uniform_row(seed, (uint64_t)k, N);
}

void wl_indices_uniform_i32(int32_t *dst, uint64_t seed, uint64_t M, uint64_t N)
{
#pragma omp parallel for schedule(static)
    for (int64_t k = 0; k < (int64_t)M; ++k)
        dst[k] = (int32_t)uniform_row(seed, (uint64_t)k, N);
}
