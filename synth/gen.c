/*
 * Seeded synthetic-input generator for vocabulary-wide logit rows.
 *
 * This file only manufactures inputs.  It contains none of the method's
 * arithmetic (no soft-max, no interpolation, no loss) and is shared by the
 * CPU oracle's tests and the GPU path's tests / benchmark so that both sides
 * see the same bytes.
 *
 * Randomness is counter based: the value of element (t, j) depends only on
 * (seed, stream, t, j), never on generation order, so rows can be produced in
 * any chunking and by any number of threads and re-generated one by one.
 *
 *   hash(c)      = SplitMix64 output function applied to  key + (c+1)*gamma
 *   two normals  = Box-Muller on the two 24-bit halves of one hash
 *
 * Build: gcc -O2 -fopenmp -shared -fPIC gen.c -lm
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

static inline uint64_t mix64(uint64_t z)
{
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

static inline uint64_t stream_key(uint64_t seed, uint32_t stream)
{
    return mix64(seed ^ (0xA0761D6478BD642Full * (uint64_t)(stream + 1u)));
}

static inline uint64_t hash_at(uint64_t key, uint64_t counter)
{
    return mix64(key + (counter + 1ull) * 0x9E3779B97F4A7C15ull);
}

/* uniform in (0,1) from 24 bits */
static inline float u24(uint32_t bits24) { return ((float)bits24 + 0.5f) * (1.0f / 16777216.0f); }

static inline void normal_pair(uint64_t h, float *a, float *b)
{
    float u1 = u24((uint32_t)(h >> 40));
    float u2 = u24((uint32_t)(h >> 8) & 0xFFFFFFu);
    float r = sqrtf(-2.0f * logf(u1));
    float ang = 6.28318530717958647692f * u2;
    *a = r * cosf(ang);
    *b = r * sinf(ang);
}

/* float -> bfloat16 bits, round to nearest even (finite inputs only here) */
static inline uint16_t f32_to_bf16_rne(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

/* 1 if row t gets its chosen-token entry boosted */
static inline int row_boosted(uint64_t seed, uint32_t stream, int64_t t, float prob)
{
    uint64_t h = hash_at(stream_key(seed, stream ^ 0x80000000u), (uint64_t)t);
    return u24((uint32_t)(h >> 40)) < prob;
}

/*
 * Fill rows t0 .. t0+nrows-1 of a [*, V] matrix with sigma * N(0,1) (+ boost at
 * column chosen[t] for boosted rows), written to out[(t-t0)*ld + j].
 * dtype: 0 = float32, 1 = bfloat16 bits (uint16).  chosen may be NULL (no boost).
 * Padding columns V..ld-1 are filled with a large finite positive sentinel so that
 * a reader that wrongly includes them is caught.
 */
void synth_logit_rows(void *out, int dtype, int64_t t0, int64_t nrows, int64_t V, int64_t ld,
                      uint64_t seed, uint32_t stream, float sigma,
                      const int32_t *chosen, float boost, float boost_prob)
{
    const uint64_t key = stream_key(seed, stream);
    const int64_t pairs = (V + 1) / 2;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < nrows; ++r) {
        const int64_t t = t0 + r;
        int64_t yb = -1;
        if (chosen && boost_prob > 0.0f && row_boosted(seed, stream, t, boost_prob)) {
            yb = chosen[t];
        }
        float *of = (float *)out + r * ld;
        uint16_t *ob = (uint16_t *)out + r * ld;
        for (int64_t k = 0; k < pairs; ++k) {
            float a, b;
            normal_pair(hash_at(key, (uint64_t)t * (uint64_t)pairs + (uint64_t)k), &a, &b);
            int64_t j = 2 * k;
            float va = sigma * a + (j == yb ? boost : 0.0f);
            float vb = sigma * b + (j + 1 == yb ? boost : 0.0f);
            if (dtype == 0) {
                of[j] = va;
                if (j + 1 < V) of[j + 1] = vb;
            } else {
                ob[j] = f32_to_bf16_rne(va);
                if (j + 1 < V) ob[j + 1] = f32_to_bf16_rne(vb);
            }
        }
        for (int64_t j = V; j < ld; ++j) {
            if (dtype == 0) of[j] = 1.0e30f;
            else ob[j] = f32_to_bf16_rne(1.0e30f);
        }
    }
}

/* 1/0 per row: whether synth_logit_rows boosts row t (for reporting) */
void synth_row_boost_flags(uint8_t *flags, int64_t t0, int64_t nrows, uint64_t seed,
                           uint32_t stream, float boost_prob)
{
    for (int64_t r = 0; r < nrows; ++r)
        flags[r] = (uint8_t)row_boosted(seed, stream, t0 + r, boost_prob);
}
