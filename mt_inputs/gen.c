/*
 * Seeded synthetic inputs for the streamed training step: weights and token
 * streams.  This file holds NO arithmetic of the training method; it only
 * produces reproducible random numbers, so that the CPU oracle and the GPU
 * library can be fed the same bytes without sharing any code of their own.
 *
 * Generator: counter based.  Element i of stream (seed, stream_id) depends only
 * on (seed, stream_id, i), so tensors can be produced in parallel, in any order,
 * and a model with fewer layers shares its leading tensors with a deeper one.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>

static inline uint64_t mix64(uint64_t z) {
    /* finaliser of the splitmix64 sequence (public domain constants) */
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

static inline uint64_t stream_key(uint64_t seed, uint64_t stream_id) {
    return mix64(mix64(seed) ^ (stream_id * 0xD1342543DE82EF95ull + 0x632BE59BD9B4E019ull));
}

static inline uint64_t draw(uint64_t key, uint64_t counter) {
    return mix64(key + counter * 0x9E3779B97F4A7C15ull);
}

/* uniform in (0,1] from the top 53 bits */
static inline double u01(uint64_t r) { return ((double)(r >> 11) + 1.0) * (1.0 / 9007199254740992.0); }

/* out[i] = mean + std * N(0,1), Box-Muller on counters (2p, 2p+1) for the pair p = i/2 */
void mti_fill_normal(float *out, size_t n, uint64_t seed, uint64_t stream_id, float mean, float std) {
    const uint64_t key = stream_key(seed, stream_id);
    const size_t pairs = (n + 1) / 2;
#pragma omp parallel for schedule(static)
    for (size_t p = 0; p < pairs; ++p) {
        double u1 = u01(draw(key, 2 * p));
        double u2 = u01(draw(key, 2 * p + 1));
        double r = sqrt(-2.0 * log(u1));
        double a = 6.283185307179586476925286766559 * u2;
        out[2 * p] = (float)(mean + std * r * cos(a));
        if (2 * p + 1 < n) out[2 * p + 1] = (float)(mean + std * r * sin(a));
    }
}

void mti_fill_const(float *out, size_t n, float value) {
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < n; ++i) out[i] = value;
}

/* out[i] uniform integer in [0, bound) */
void mti_fill_tokens(int32_t *out, size_t n, uint64_t seed, uint64_t stream_id, int32_t bound) {
    const uint64_t key = stream_key(seed, stream_id);
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < n; ++i) {
        uint64_t r = draw(key, i);
        /* multiply-shift maps 64 random bits onto [0,bound) with bias < 2^-32 */
        out[i] = (int32_t)(((r >> 32) * (uint64_t)bound) >> 32);
    }
}
